"""Build libftuner.so (host logic + HIP dispatcher kernels) for gfx950, in-tree.

hipcc cross-compiles without a GPU.  Objects go to paper_2407_21418_amd/_build/, the
library to paper_2407_21418_amd/libftuner.so.
"""
import concurrent.futures as cf
import os
import subprocess
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libftuner.so")
INC = os.path.join(os.path.dirname(HERE), "include")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INC, "-I", CSRC,
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _run(cmd, log):
    t = time.time()
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l]
    with open(log, "w") as f:
        f.write(" ".join(cmd) + "\n" + "\n".join(lines) + "\n")
    if p.returncode != 0:
        raise RuntimeError("build step failed: %s\n%s" % (" ".join(cmd), "\n".join(lines[-40:])))
    return time.time() - t


def _resource_usage(log):
    """The compiler's kernel-resource-usage remarks of one object, as {name: value}."""
    out = {}
    with open(log) as f:
        for line in f:
            if "remark:" not in line or "[-Rpass-analysis" not in line:
                continue
            body = line.split("remark:", 1)[1].split("[-Rpass-analysis", 1)[0].strip()
            if ":" in body:
                k, v = body.rsplit(":", 1)
                k, v = k.strip(), v.strip()
                if k in ("VGPRs", "AGPRs", "ScratchSize [bytes/lane]", "VGPRs Spill", "SGPRs Spill", "Occupancy [waves/SIMD]"):
                    out[k] = int(v)
    return out


def _stale(obj, srcs):
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(s) > t for s in srcs)


def build(verbose=True, remarks=True, jobs=None, incremental=False, trace=False):
    """incremental=True recompiles only objects older than the sources they include.
    trace=True builds the development variant libftuner_trace.so (-DFT_TRACE: workgroups leave
    timestamps, see FT_MARK) from objects of its own; the product library is not touched."""
    global OUT, LIB, COMMON
    if trace:
        OUT, LIB = os.path.join(HERE, "_build_trace"), os.path.join(HERE, "libftuner_trace.so")
        # FT_DEBUG_DEFS / FT_TRACE_LIB: other development switches (see gemm_fast.h) and the file to write
        extra = os.environ.get("FT_DEBUG_DEFS", "-DFT_TRACE").split()
        COMMON = [c for c in COMMON if not c.startswith("-DFT_DEBUG") and c != "-DFT_TRACE"] + extra
        LIB = os.environ.get("FT_TRACE_LIB", LIB)
    os.makedirs(OUT, exist_ok=True)
    hdrs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + \
           [os.path.join(INC, "ftuner.h")]
    steps = []
    for dt in (0, 1):
        for cl in (0, 1, 2):
            obj = os.path.join(OUT, f"dispatch_dt{dt}_c{cl}.o")
            # (launches whose rows are whole 16-byte chunks: bodies without the code for ragged rows)
            cmd = [HIPCC] + COMMON + [f"-DFT_DT={dt}", f"-DFT_CLASS={cl}", "-DFT_NO_RAGGED=1", "-c",
                                      os.path.join(CSRC, "dispatch.hip"), "-o", obj]
            cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
            steps.append((obj, cmd))
            obj = os.path.join(OUT, f"dispatch_dt{dt}_rg_c{cl}.o")          # the same bodies with that code
            cmd = [HIPCC] + COMMON + [f"-DFT_DT={dt}", f"-DFT_CLASS={cl}", "-DFT_RG=1", "-c",
                                      os.path.join(CSRC, "dispatch.hip"), "-o", obj]
            cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
            steps.append((obj, cmd))
    for dt in (0, 1):                         # two-team bodies: workgroups of eight waves
        for cl in (0, 1):
            obj = os.path.join(OUT, f"dispatch_dt{dt}_pp_c{cl}.o")
            cmd = [HIPCC] + COMMON + [f"-DFT_DT={dt}", f"-DFT_CLASS={cl}", "-DFT_PP=1", "-DFT_NO_RAGGED=1", "-c",
                                      os.path.join(CSRC, "dispatch.hip"), "-o", obj]
            cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
            steps.append((obj, cmd))
    gen = []
    for dt in (0, 1):
        for cl in (2, 1):
            obj = os.path.join(OUT, f"dispatch_dt{dt}_gen_c{cl}.o")
            cmd = [HIPCC] + COMMON + [f"-DFT_DT={dt}", f"-DFT_CLASS={cl}", "-DFT_GENERIC=1", "-c",
                                      os.path.join(CSRC, "dispatch.hip"), "-o", obj]
            cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
            gen.append((obj, cmd))
    for dt in (0, 1):                         # grouped launches: general bodies, per-group shapes
        for cl in (2, 1):
            obj = os.path.join(OUT, f"dispatch_dt{dt}_grp_c{cl}.o")
            cmd = [HIPCC] + COMMON + [f"-DFT_DT={dt}", f"-DFT_CLASS={cl}", "-DFT_GENERIC=1", "-DFT_GROUPED=1", "-c",
                                      os.path.join(CSRC, "dispatch.hip"), "-o", obj]
            cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
            gen.append((obj, cmd))
    for dt in (0, 1):                         # grouped launches whose groups are all aligned: LDS-DMA bodies
        for cl in (2, 1, 0):
            obj = os.path.join(OUT, f"dispatch_dt{dt}_grpf_c{cl}.o")
            cmd = [HIPCC] + COMMON + [f"-DFT_DT={dt}", f"-DFT_CLASS={cl}", "-DFT_GROUPED=1", "-c",
                                      os.path.join(CSRC, "dispatch.hip"), "-o", obj]
            cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
            gen.append((obj, cmd))
    for dt in (0, 1):                         # operand B as [N][K]: LDS-DMA bodies, plain and grouped launches
        for cl in (2, 1, 0):
            for tag, defs in (("nk", []), ("grpnk", ["-DFT_GROUPED=1"])):
                obj = os.path.join(OUT, f"dispatch_dt{dt}_{tag}_c{cl}.o")
                cmd = [HIPCC] + COMMON + [f"-DFT_DT={dt}", f"-DFT_CLASS={cl}", "-DFT_BNK=1"] + defs + \
                      ["-c", os.path.join(CSRC, "dispatch.hip"), "-o", obj]
                cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
                gen.append((obj, cmd))
    gen.sort(key=lambda oc: "_c2" not in oc[0])   # the 512-register kernels take longest: start them first
    steps = gen + steps
    for src in ("host.cpp", "device.hip"):
        obj = os.path.join(OUT, src.replace(".", "_") + ".o")
        steps.append((obj, [HIPCC] + COMMON + ["-c", os.path.join(CSRC, src), "-o", obj]))
    jobs = jobs or min(8, len(steps))
    if trace:
        # only the f16 LDS-DMA dispatchers and the launch code carry the marks; everything else is
        # linked from the product build (same argument layout), which must exist
        prod = os.path.join(HERE, "_build")
        keep = lambda o: any(t in os.path.basename(o) for t in ("dispatch_dt0_c", "dispatch_dt0_pp_c", "device_hip", "host_cpp"))
        steps = [(o, c) if keep(o) else (os.path.join(prod, os.path.basename(o)), None) for o, c in steps]
    todo = [(o, c) for o, c in steps if c is not None]
    if incremental:
        src_of = lambda cmd: cmd[cmd.index("-c") + 1]
        todo = [(o, c) for o, c in todo if _stale(o, hdrs + [src_of(c)])]
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        futs = {ex.submit(_run, cmd, obj + ".log"): obj for obj, cmd in todo}
        for fut in cf.as_completed(futs):
            dt = fut.result()
            if verbose:
                print(f"  built {os.path.basename(futs[fut])} in {dt:.1f}s", flush=True)
    # a dispatcher that touches scratch memory (spilled registers, kernel arguments copied to the
    # stack by a dynamically indexed array) is several times slower: refuse to link it.  The general
    # (unaligned-operand) dispatchers may spill a few registers in their largest bodies.
    for obj, _ in steps:
        if "dispatch_" not in obj or not os.path.exists(obj + ".log"):
            continue
        use = _resource_usage(obj + ".log")
        if verbose or remarks:
            print(f"  {os.path.basename(obj)}: {use}", flush=True)
        name = os.path.basename(obj)
        allowed = 32 if ("_gen_" in name or "_grp_" in name) else 0
        # (the grouped LDS-DMA dispatchers of the 256-register class spill three registers around the
        # fix-up of a ragged last k-tile, outside the k loop's steady state: measured, no change)
        if ("_grpf_c1" in name or "_grpnk_c1" in name):
            allowed = 16
        # (the 512-register LDS-DMA dispatchers of bf16 spill one or two registers in the store code of the
        # 256 x 256 body -- the rounding to bf16 needs more temporaries than a conversion to fp16 -- outside
        # every k loop: one store and two loads per workgroup)
        if "_dt1_" in name and name.endswith("_c2.o") and allowed == 0:
            allowed = 8
        if trace:
            allowed = 1 << 20                 # development variants are not held to it
        if use.get("ScratchSize [bytes/lane]", 0) > allowed:
            raise RuntimeError(f"{os.path.basename(obj)} uses scratch memory: {use}")
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [o for o, _ in steps]
    _run(link, os.path.join(OUT, "link.log"))
    if verbose:
        print("  linked", LIB, flush=True)
    return LIB


if __name__ == "__main__":
    build(remarks="--remarks" in sys.argv, incremental="--incremental" in sys.argv, trace="--trace" in sys.argv)
