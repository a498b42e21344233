"""CPU oracle (test infrastructure only).

Independent of the GPU library: nothing under this package imports, links or reads
anything of the HIP path, and the product never imports this package.  Only the tests,
the smoke check and the benchmark's cpu_baseline leg use it.
"""
