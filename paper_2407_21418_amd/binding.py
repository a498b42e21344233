"""ctypes binding of libftuner.so (see include/ftuner.h for the contract of every call).

Only marshals arguments.  The library must have been built (python -m
paper_2407_21418_amd.build, or __graft_entry__.build()); a missing library is an error,
there is no fallback path.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# FTUNER_LIB names another build of the same library (e.g. the development variant with timestamps)
LIB_PATH = os.environ.get("FTUNER_LIB") or os.path.join(_HERE, "libftuner.so")

FT_OK = 0
FT_ERR_INVALID_ARG, FT_ERR_UNSUPPORTED, FT_ERR_OUT_OF_RANGE = -1, -2, -3
FT_ERR_NO_COVER, FT_ERR_HIP, FT_ERR_OOM = -4, -5, -6
FT_OP_MATMUL, FT_OP_BMM, FT_OP_CONV2D = 0, 1, 2
FT_F16, FT_BF16 = 0, 1
FT_OUT_F32, FT_OUT_SAME = 0, 1
FT_EPI_NONE, FT_EPI_BIAS = 0, 1
FT_B_KN, FT_B_NK = 0, 1
FT_PLAN_PATCHWORK, FT_PLAN_PAD_BASELINE, FT_PLAN_FORCED, FT_PLAN_HOST_ONLY, FT_PLAN_TABLE_ORDER = 0, 1, 2, 16, 32
FT_SIA_LINEAR, FT_SIA_PRODUCT = 0, 1

u32, u64, u16 = C.c_uint32, C.c_uint64, C.c_uint16


class _S(C.Structure):
    def __init__(self, **kw):
        super().__init__()
        self.struct_size = C.sizeof(self)
        for k, v in kw.items():
            setattr(self, k, v)

    def as_dict(self):
        out = {}
        for name, _t in self._fields_:
            v = getattr(self, name)
            out[name] = list(v) if hasattr(v, "__len__") else v
        return out


class ft_hw_model(_S):
    _fields_ = [(n, u32) for n in (
        "struct_size", "num_cus", "simds_per_cu", "wave_size", "regs_per_lane", "max_waves_per_simd",
        "lds_bytes_per_cu", "clock_mhz", "mfma_flops_per_clk_per_cu", "bw_global_bytes_per_clk_per_cu",
        "bw_lds_bytes_per_clk_per_cu", "ktile_latency_clk", "solo_copy_exposed_pct", "hbm_gbytes_per_s", "num_xcds", "part_exchange_clk", "part_exchange_bytes_per_clk", "phase_latency_clk")]


class ft_tuning(_S):
    _fields_ = [(n, u32) for n in (
        "struct_size", "eps_min_pm", "eps_max_pm", "eps_step_pm", "lam_max_pm", "lam_min_pm", "lam_step_pm",
        "zeta", "rest_regs", "psi_num", "psi_den", "c0", "c1", "c2", "sia_form", "k_parts_max", "k_part_min_tiles", "second_axis_strips", "two_team_bodies")]


class ft_op_desc(_S):
    _fields_ = [(n, u32) for n in (
        "struct_size", "kind", "dtype", "m", "n", "k", "m_lo", "m_hi", "n_lo", "n_hi", "k_lo", "k_hi",
        "c_in", "c_out", "r", "s", "stride", "pad", "out_dtype", "epilogue", "batch_hi", "b_layout")]


class ft_ukernel_info(_S):
    _fields_ = [(n, u32) for n in (
        "struct_size", "id", "tm", "tn", "tk", "wm", "wn", "gm", "gn", "gk", "mfma", "stages", "lds_bytes",
        "acc_regs", "regs", "max_wg_per_cu", "reg_budget")] + [("cmr_q20", u64), ("cmr_shared_q20", u64)]


class ft_shape(_S):
    _fields_ = [(n, u32) for n in ("struct_size", "batch", "m", "n", "k", "img_n", "img_h", "img_w")]


class ft_forced_program(_S):
    _fields_ = [(n, u32) for n in ("struct_size", "k1", "count1", "k2", "count2", "k_parts")]


class ft_tile_desc(C.Structure):
    _fields_ = [("ukernel_id", u32), ("batch", u32), ("m0", u32), ("n0", u32),
                ("m_valid", u16), ("n_valid", u16), ("flags", u32)]


class ft_plan_stats(_S):
    _fields_ = [("struct_size", u32), ("tau", u32), ("batch", u32), ("m", u32), ("n", u32), ("k", u32),
                ("n_ukernels", u32), ("ukernel_id", u32 * 2), ("count_tau", u32 * 2), ("block_bound", u32),
                ("pool_size", u32), ("level", u32), ("pad_q20", u32), ("occ_q20", u32), ("cmr_q20", u32),
                ("lds_bytes", u32), ("kernel_class", u32), ("sia_q20", u64), ("n_tiles", u64),
                ("useful_elems", u64), ("covered_elems", u64), ("k_parts", u32), ("k_part_tiles", u32),
                ("workspace_bytes", u64), ("main_tiles", u32 * 2), ("strip_ukernel_id", u32 * 2), ("strip_tiles", u32 * 2), ("table_order", u32)]


class ft_pool_entry(C.Structure):
    _fields_ = [("k1", u32), ("count1", u32), ("k2", u32), ("count2", u32), ("pad_q20", u32),
                ("occ_q20", u32), ("cmr_q20", u32), ("flags", u32), ("sia_q20", u64), ("n_tiles", u64)]


class FtError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {ft_status_string(status)} ({status})")


_lib = None

# every symbol include/ftuner.h declares: name -> (restype, argtypes)
_P = C.c_void_p
SYMBOLS = {
    "ft_status_string": (C.c_char_p, [C.c_int32]),
    "ft_last_hip_error": (C.c_int32, []),
    "ft_hw_default_gfx950": (C.c_int32, [C.POINTER(ft_hw_model)]),
    "ft_hw_query": (C.c_int32, [C.c_int32, C.POINTER(ft_hw_model)]),
    "ft_tuning_default": (C.c_int32, [C.POINTER(ft_tuning)]),
    "ft_op_register": (C.c_int32, [C.POINTER(ft_op_desc), C.POINTER(_P)]),
    "ft_op_destroy": (None, [_P]),
    "ft_ukernels_derive": (C.c_int32, [_P, C.POINTER(ft_hw_model), C.POINTER(ft_tuning), C.POINTER(_P)]),
    "ft_ukset_size": (C.c_int32, [_P, C.POINTER(u32)]),
    "ft_ukset_get": (C.c_int32, [_P, u32, C.POINTER(ft_ukernel_info)]),
    "ft_ukset_destroy": (None, [_P]),
    "ft_plan_create": (C.c_int32, [_P, _P, C.POINTER(ft_shape), u32, C.POINTER(ft_forced_program), C.POINTER(_P)]),
    "ft_plan_create_grouped": (C.c_int32, [_P, _P, C.POINTER(ft_shape), u32, u32, C.POINTER(_P)]),
    "ft_plan_group_layout": (C.c_int32, [_P, u32, C.POINTER(u64), C.POINTER(u64), C.POINTER(u64)]),
    "ft_plan_cached": (C.c_int32, [_P, _P, C.POINTER(ft_shape), u32, C.POINTER(_P)]),
    "ft_plan_descriptors": (C.c_int32, [_P, C.POINTER(C.POINTER(ft_tile_desc)), C.POINTER(u64)]),
    "ft_plan_launch_order": (C.c_int32, [_P, C.POINTER(u32), u64, C.POINTER(u64)]),
    "ft_plan_stats_get": (C.c_int32, [_P, C.POINTER(ft_plan_stats)]),
    "ft_plan_destroy": (None, [_P]),
    "ft_plan_pool": (C.c_int32, [_P, _P, C.POINTER(ft_shape), C.POINTER(ft_pool_entry), u32, C.POINTER(u32)]),
    "ft_launch": (C.c_int32, [_P, _P, _P, _P, _P]),
    "ft_launch_epilogue": (C.c_int32, [_P, _P, _P, _P, _P, _P]),
    "ft_launch_noalloc": (C.c_int32, [_P, _P, _P, _P, _P, _P]),
    "ft_stream_rate": (C.c_int32, [_P, _P, u64, u32, _P, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float)]),
    "ft_launch_timed": (C.c_int32, [_P, C.POINTER(_P), C.POINTER(_P), C.POINTER(_P), u32, _P, u32,
                                    C.POINTER(C.c_float)]),
    "ft_launch_timed_graph": (C.c_int32, [_P, C.POINTER(_P), C.POINTER(_P), C.POINTER(_P), u32, _P, u32,
                                          C.POINTER(C.c_float)]),
}


def lib():
    """Load libftuner.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_21418_amd.build`")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SYMBOLS.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _check(status, what):
    if status != FT_OK:
        raise FtError(status, what)


def ft_status_string(status):
    return lib().ft_status_string(status).decode()


def ft_last_hip_error():
    return lib().ft_last_hip_error()


def ft_hw_default_gfx950():
    hw = ft_hw_model()
    _check(lib().ft_hw_default_gfx950(C.byref(hw)), "ft_hw_default_gfx950")
    return hw


def ft_hw_query(device=0):
    hw = ft_hw_model()
    _check(lib().ft_hw_query(device, C.byref(hw)), "ft_hw_query")
    return hw


def ft_tuning_default():
    t = ft_tuning()
    _check(lib().ft_tuning_default(C.byref(t)), "ft_tuning_default")
    return t


class _Handle:
    _destroy = None

    def __init__(self, ptr):
        self.ptr = ptr

    def close(self):
        if self.ptr:
            getattr(lib(), self._destroy)(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Op(_Handle):
    _destroy = "ft_op_destroy"


class UkSet(_Handle):
    _destroy = "ft_ukset_destroy"


class Plan(_Handle):
    _destroy = "ft_plan_destroy"


def ft_op_register(desc: ft_op_desc) -> Op:
    out = _P()
    _check(lib().ft_op_register(C.byref(desc), C.byref(out)), "ft_op_register")
    op = Op(out.value)
    op.desc = desc
    return op


def ft_ukernels_derive(op: Op, hw=None, tuning=None) -> UkSet:
    out = _P()
    _check(lib().ft_ukernels_derive(op.ptr, C.byref(hw) if hw is not None else None,
                                    C.byref(tuning) if tuning is not None else None, C.byref(out)),
           "ft_ukernels_derive")
    return UkSet(out.value)


def ft_ukset_size(s: UkSet) -> int:
    n = u32()
    _check(lib().ft_ukset_size(s.ptr, C.byref(n)), "ft_ukset_size")
    return n.value


def ft_ukset_get(s: UkSet, i: int) -> ft_ukernel_info:
    info = ft_ukernel_info()
    _check(lib().ft_ukset_get(s.ptr, i, C.byref(info)), "ft_ukset_get")
    return info


def ft_plan_create(op: Op, s: UkSet, shape: ft_shape, flags=FT_PLAN_PATCHWORK, forced=None) -> Plan:
    out = _P()
    _check(lib().ft_plan_create(op.ptr, s.ptr, C.byref(shape), flags,
                                C.byref(forced) if forced is not None else None, C.byref(out)),
           "ft_plan_create")
    return Plan(out.value)


def ft_plan_create_grouped(op: Op, s: UkSet, groups, flags=FT_PLAN_PATCHWORK) -> Plan:
    """groups: sequence of ft_shape, one per group (batch = matrices of that shape)."""
    arr = (ft_shape * max(1, len(groups)))(*groups)
    out = _P()
    _check(lib().ft_plan_create_grouped(op.ptr, s.ptr, arr, len(groups), flags, C.byref(out)), "ft_plan_create_grouped")
    return Plan(out.value)


def ft_plan_group_layout(p: Plan, group: int):
    """(off_a, off_b, off_c): element offsets of the group's first matrices in the packed buffers;
    group == number of groups gives the buffers' total element counts."""
    a, b, c = u64(), u64(), u64()
    _check(lib().ft_plan_group_layout(p.ptr, group, C.byref(a), C.byref(b), C.byref(c)), "ft_plan_group_layout")
    return a.value, b.value, c.value


def ft_plan_descriptors(p: Plan) -> bytes:
    """The descriptor table as raw bytes (24 bytes per tile, little endian)."""
    ptr = C.POINTER(ft_tile_desc)()
    n = u64()
    _check(lib().ft_plan_descriptors(p.ptr, C.byref(ptr), C.byref(n)), "ft_plan_descriptors")
    if n.value == 0:
        return b""
    return C.string_at(ptr, n.value * C.sizeof(ft_tile_desc))


class CachedPlan:
    """A plan owned by its uKernel set's cache: same .ptr interface as Plan, never destroyed here.
    Keeps the set alive."""

    def __init__(self, ptr, owner):
        self.ptr = ptr
        self._owner = owner


def ft_plan_cached(op: Op, s: UkSet, shape: ft_shape, flags: int = FT_PLAN_PATCHWORK) -> CachedPlan:
    out = _P()
    _check(lib().ft_plan_cached(op.ptr, s.ptr, C.byref(shape), flags, C.byref(out)), "ft_plan_cached")
    return CachedPlan(out.value, s)


def ft_plan_launch_order(p: Plan):
    """Descriptor index taken by each workgroup of the launch (a permutation of the table; for a
    plan walked in table order followed by 0xFFFFFFFF entries for the idle workgroups of the last round)."""
    n = u64()
    _check(lib().ft_plan_launch_order(p.ptr, None, 0, C.byref(n)), "ft_plan_launch_order")
    buf = (u32 * max(1, n.value))()
    _check(lib().ft_plan_launch_order(p.ptr, buf, n.value, C.byref(n)), "ft_plan_launch_order")
    return list(buf[:n.value])


def ft_plan_stats_get(p: Plan) -> ft_plan_stats:
    st = ft_plan_stats()
    _check(lib().ft_plan_stats_get(p.ptr, C.byref(st)), "ft_plan_stats_get")
    return st


def ft_plan_pool(op: Op, s: UkSet, shape: ft_shape):
    n = u32()
    _check(lib().ft_plan_pool(op.ptr, s.ptr, C.byref(shape), None, 0, C.byref(n)), "ft_plan_pool")
    arr = (ft_pool_entry * max(1, n.value))()
    _check(lib().ft_plan_pool(op.ptr, s.ptr, C.byref(shape), arr, n.value, C.byref(n)), "ft_plan_pool")
    return [arr[i] for i in range(n.value)]


def ft_launch(p: Plan, A: int, B: int, Cptr: int, stream: int = 0):
    """A, B, Cptr: device addresses (e.g. torch.Tensor.data_ptr()); stream: hipStream_t value."""
    _check(lib().ft_launch(p.ptr, A, B, Cptr, stream), "ft_launch")


def ft_launch_epilogue(p: Plan, A: int, B: int, Cptr: int, bias: int, stream: int = 0):
    """As ft_launch, with bias = device address of N fp32 values (0 / None for none)."""
    _check(lib().ft_launch_epilogue(p.ptr, A, B, Cptr, bias or None, stream), "ft_launch_epilogue")


def ft_launch_noalloc(p: Plan, A: int, B: int, Cptr: int, bias: int = 0, stream: int = 0):
    """As ft_launch_epilogue, with the workspace of a reduce-axis split in the library's own device array."""
    _check(lib().ft_launch_noalloc(p.ptr, A, B, Cptr, bias or None, stream), "ft_launch_noalloc")


def ft_stream_rate(src: int, dst: int, nbytes: int, iters: int, stream: int = 0):
    """(read, write, copy) GB/s of plain streaming kernels over nbytes at the device addresses src, dst."""
    r, w, c = C.c_float(), C.c_float(), C.c_float()
    _check(lib().ft_stream_rate(src, dst, nbytes, iters, stream, C.byref(r), C.byref(w), C.byref(c)), "ft_stream_rate")
    return r.value, w.value, c.value


def ft_launch_timed(p: Plan, A, B, Cs, stream: int, iters: int, graph: bool = False) -> float:
    """A, B, Cs: equally long lists of device addresses (rotating buffer sets).  graph=True times
    one replay of a HIP graph holding the `iters` launches (stream must not be the NULL stream)."""
    n = len(A)
    arr = lambda xs: (_P * n)(*xs)
    ms = C.c_float()
    fn = lib().ft_launch_timed_graph if graph else lib().ft_launch_timed
    _check(fn(p.ptr, arr(A), arr(B), arr(Cs), n, stream, iters, C.byref(ms)),
           "ft_launch_timed_graph" if graph else "ft_launch_timed")
    return ms.value
