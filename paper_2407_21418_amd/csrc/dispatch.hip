// One dispatcher kernel per (input dtype, register class).  Workgroup i takes tile descriptor
// remap(i) and runs the uKernel body the descriptor names, so a single launch executes a
// program made of one or two uKernel shapes (Sec. 5.1; Fig. 8 item 2).
// Compiled once per -DFT_DT={0,1} -DFT_CLASS={0,1,2} with the fast bodies (LDS-DMA ring, aligned
// operands) and per dtype with -DFT_GENERIC=1 -DFT_CLASS={1,2} for the general bodies (any alignment,
// ragged reduce axis, convolution gather): class 1 holds every body with at most 64 accumulator
// registers in a 256-register kernel (two workgroups per CU), class 2 all of them in 512 registers.
#include <mutex>

#include "gemm_fast.h"
#include "family.h"
#include "launch_iface.h"
#include "tile_order.h"

#ifndef FT_DT
#error "define FT_DT"
#endif
#define FT_MAX_DEVICES 64
#ifndef FT_CLASS
#error "define FT_CLASS"
#endif

// -DFT_BNK=1 (with the fast bodies only): operand B is [N][K]; the four-wave standard grids, no split-k
// wave grid (the host sends such a uKernel to its standard-grid twin)
#ifdef FT_BNK
#define FT_BNK_FLAG true
#else
#define FT_BNK_FLAG false
#endif

#ifdef FT_PP
// two-team workgroups: eight waves, two per SIMD; classes 0 (128 registers) and 1 (256 registers)
#define FT_THREADS 512
#define FT_TEAMS 2
#else
#define FT_THREADS 256
#define FT_TEAMS 1
#endif

#if FT_CLASS == 0
#define FT_MIN_WAVES 4
#define FT_ACC_MAX 32
#elif FT_CLASS == 1
#define FT_MIN_WAVES 2
#if defined(FT_GENERIC) || defined(FT_PP)
#define FT_ACC_MAX 64        // the general bodies also hold their staging registers; two teams: see family.h
#else
#define FT_ACC_MAX 128
#endif
#else
#define FT_MIN_WAVES 1
#define FT_ACC_MAX 256
#endif

namespace ftk {

__global__ __launch_bounds__(FT_THREADS, FT_MIN_WAVES) void FT_KERNEL_NAME(KArgs g) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    FT_MARK(g, 0);
    // The arguments span several cache lines and the compiler loads each field right before its
    // first use, so a cold scalar cache would be missed several times in a row (about half a
    // microsecond each, on the critical path of every workgroup).  Touch every line once, up front
    // and in parallel; the later loads hit.  Measured: +2.5 % on the sweep of small GEMMs (a few
    // hundred workgroups per launch, all in their first round).
    {
        const auto ka = __builtin_amdgcn_kernarg_segment_ptr();
        static_assert(sizeof(KArgs) > 0x100 && sizeof(KArgs) <= 0x140, "one load per 64-byte line of the arguments");
        uint32_t w0, w1, w2, w3, w4;
        asm volatile("s_load_dword %0, %5, 0x0\n\t"
                     "s_load_dword %1, %5, 0x40\n\t"
                     "s_load_dword %2, %5, 0x80\n\t"
                     "s_load_dword %3, %5, 0xc0\n\t"
                     "s_load_dword %4, %5, 0x100\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=s"(w0), "=s"(w1), "=s"(w2), "=s"(w3), "=s"(w4)
                     : "s"(ka)
                     : "memory");
    }
    LaunchOrder o;
    o.n[0] = g.slot_first[1] - g.slot_first[0];
    o.n[1] = g.n_tiles - g.slot_first[1];
    o.first[0] = g.slot_first[0]; o.first[1] = g.slot_first[1];
    o.rows[0] = g.slot_rows[0]; o.rows[1] = g.slot_rows[1];
    o.cols[0] = g.slot_cols[0]; o.cols[1] = g.slot_cols[1];
    o.group[0] = g.slot_group[0]; o.group[1] = g.slot_group[1];
    o.m_base[0] = g.slot_m0[0]; o.m_base[1] = g.slot_m0[1];
    o.n_base[0] = g.slot_n0[0]; o.n_base[1] = g.slot_n0[1];
    o.tm[0] = g.slot_tm[0]; o.tm[1] = g.slot_tm[1];
    o.tn[0] = g.slot_tn[0]; o.tn[1] = g.slot_tn[1];
    o.nx = g.num_xcds;
    // Reduce axis split over workgroups: the k_parts workgroups of a tile are k_parts consecutive
    // multiples of num_xcds apart, so they share an XCD (workgroup b runs on XCD b % num_xcds) and
    // their partial tiles meet in that XCD's L2.  The grid is rounded up to whole XCD rounds.
    uint32_t b = blockIdx.x, part = 0;
    if (g.k_parts > 1) {
        part = (b / o.nx) % g.k_parts;
        b = (b / (o.nx * g.k_parts)) * o.nx + b % o.nx;
        if (b >= (g.table_order ? table_grid(g.n_tiles, o.nx) : g.n_tiles)) return;
    }
    // A program of one or two uKernel shapes lays its tiles out as grids: the workgroup derives its
    // descriptor's contents in closed form and saves the dependent load from the table (about a
    // microsecond on the critical path of a launch whose workgroups all start at once; the host has
    // checked the closed form against the table).  A plan with second-axis strips has up to four
    // shapes and is walked in table order: its workgroups read their descriptor, whose uKernel id
    // names the slot (selects, no indexing: the arguments stay in SGPRs).
    uint32_t slot, t;
    TileDesc d;
#ifdef FT_GROUPED
    // Grouped launch: the table is the concatenation of the groups' programs, walked in table order.
    // A descriptor names its group (flags bits 12..31), its body (bits 1..7) and that body's LDS ring
    // depth (bits 8..11); the group's record replaces the launch-wide shape, pitches and operand
    // bases, read with scalar loads since the index is uniform.  The bodies see an ordinary batched
    // problem.  Compiled over the general bodies (any alignment) and over the LDS-DMA bodies (every
    // group aligned; the host decides per launch).
    t = table_index_of_workgroup(b, o.nx);
    if (t >= g.n_tiles) return;
    d = g.descs[t];
    const uint32_t dflags = __builtin_amdgcn_readfirstlane(d.flags);
    const GroupRec rec = g.groups[dflags >> 12];
    KArgs gl = g;
    gl.M = __builtin_amdgcn_readfirstlane(rec.m);
    gl.N = __builtin_amdgcn_readfirstlane(rec.n);
    gl.K = __builtin_amdgcn_readfirstlane(rec.k);
    gl.lda = gl.K; gl.ldb = FT_BNK_FLAG ? gl.K : gl.N; gl.ldc = gl.N;
    gl.strideA = (uint64_t)gl.M * gl.K;
    gl.strideB = (uint64_t)gl.K * gl.N;
    gl.strideC = (uint64_t)gl.M * gl.N;
    auto uniform64 = [](uint64_t x) -> uint64_t {
        return (uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)x) |
               ((uint64_t)__builtin_amdgcn_readfirstlane((uint32_t)(x >> 32)) << 32);
    };
    const uint64_t offA = uniform64(rec.offA), offB = uniform64(rec.offB), offC = uniform64(rec.offC);
    gl.A = g.A + offA;
    gl.B = g.B + offB;
    gl.C = g.out_kind == OUT_F32 ? static_cast<void *>(static_cast<float *>(g.C) + offC)
                                 : static_cast<void *>(static_cast<uint16_t *>(g.C) + offC);
    d.flags = dflags & 1u;
    d.batch = __builtin_amdgcn_readfirstlane(d.batch);
    d.m0 = __builtin_amdgcn_readfirstlane(d.m0);
    d.n0 = __builtin_amdgcn_readfirstlane(d.n0);
    t = __builtin_amdgcn_readfirstlane(t);
    slot = 0;
    (void)slot; (void)part;
    uint32_t gcode = (dflags >> 1) & 0x7fu;
#ifdef FT_GENERIC
    // the general path has no split-k wave grid: such a uKernel runs on its standard-grid twin
#define FT_X(CODE, TM, TN, TWIN) if (gcode == CODE) gcode = TWIN;
    FT_FAMILY_SPLITK(FT_X)
#undef FT_X
    switch (gcode) {
#define FT_X(CODE, WM, WN, GM, GN)                                              \
    case CODE:                                                                  \
        if constexpr ((WM) * (WN) / 64 <= FT_ACC_MAX)                           \
            UKernelBody<FT_DT, WM, WN, GM, GN, FT_TK>::run(gl, d, smem);        \
        break;
        FT_FAMILY(FT_X)
        FT_FAMILY_PARTIAL(FT_X)
#undef FT_X
    default: break;
    }
#else
    const uint32_t gstages = (dflags >> 8) & 0xfu;
    switch (gcode) {
#define FT_X(CODE, WM, WN, GM, GN)                                              \
    case CODE:                                                                  \
        if constexpr ((WM) * (WN) / 64 <= FT_ACC_MAX)                           \
            UKernelFast<FT_DT, WM, WN, GM, GN, 1, FT_BNK_FLAG>::run(gl, d, smem, gstages, t, 0u); \
        break;
        FT_FAMILY(FT_X)
#undef FT_X
#ifndef FT_BNK
#define FT_X(CODE, TM, TN, TWIN)                                                \
    case CODE:                                                                  \
        if constexpr ((TM) * (TN) / 64 <= FT_ACC_MAX)                           \
            UKernelSplitK<FT_DT, TM, TN>::run(gl, d, smem, gstages, t, 0u);     \
        break;
        FT_FAMILY_SPLITK(FT_X)
#undef FT_X
#endif
    default: break;
    }
#endif
    return;
#else
    if (g.table_order) {
        t = table_index_of_workgroup(b, o.nx);
        if (t >= g.n_tiles) return;             // the grid is rounded up to whole rounds of chunks
        d = g.descs[t];
        const uint32_t id = __builtin_amdgcn_readfirstlane(d.ukernel_id);       // uniform per workgroup
        slot = id == g.slot_ukernel[0] ? 0u : id == g.slot_ukernel[1] ? 1u : id == g.slot_ukernel[2] ? 2u : 3u;
    } else {
        const TileOfWorkgroup w = tile_of_workgroup(o, b);
        t = w.index;
        slot = w.slot;
        d.ukernel_id = 0; d.m_valid = 0; d.n_valid = 0; d.flags = 0;          // not used by the bodies
        d.batch = w.batch; d.m0 = w.m0; d.n0 = w.n0;
    }
    // Everything a body gets from here is the same for all lanes; say so.  Without it the
    // compiler's uniformity analysis gave up in the general dispatchers after small changes to
    // this prologue and built the buffer-store descriptors of every body in "waterfall" loops
    // (4 000 instead of 80 v_readfirstlane in the kernel, 10 more VGPRs): the store-bound attention
    // launches ran 10-30 % slower.
    d.batch = __builtin_amdgcn_readfirstlane(d.batch);
    d.m0 = __builtin_amdgcn_readfirstlane(d.m0);
    d.n0 = __builtin_amdgcn_readfirstlane(d.n0);
    slot = __builtin_amdgcn_readfirstlane(slot);
    t = __builtin_amdgcn_readfirstlane(t);
    const uint32_t code = slot == 0 ? g.slot_code[0] : slot == 1 ? g.slot_code[1] : slot == 2 ? g.slot_code[2] : g.slot_code[3];
    const uint32_t stages = slot == 0 ? g.slot_stages[0] : slot == 1 ? g.slot_stages[1] : slot == 2 ? g.slot_stages[2] : g.slot_stages[3];
    switch (code) {
#ifdef FT_GENERIC
#define FT_X(CODE, WM, WN, GM, GN)                                              \
    case CODE:                                                                  \
        if constexpr ((WM) * (WN) / 64 <= FT_ACC_MAX)                           \
            UKernelBody<FT_DT, WM, WN, GM, GN, FT_TK>::run(g, d, smem);         \
        break;
#elif defined(FT_PP)
#define FT_X(CODE, WM, WN, GM, GN)                                              \
    case CODE:                                                                  \
        if constexpr ((WM) * (WN) / 64 <= FT_ACC_MAX && ((GM) * (WM) + (GN) * (WN)) * FT_TK * 2 <= FT_PP_STAGE_MAX) \
            UKernelFast<FT_DT, WM, WN, GM, GN, 2>::run(g, d, smem, stages, t, part); \
        break;
#else
#define FT_X(CODE, WM, WN, GM, GN)                                              \
    case CODE:                                                                  \
        if constexpr ((WM) * (WN) / 64 <= FT_ACC_MAX)                           \
            UKernelFast<FT_DT, WM, WN, GM, GN, 1, FT_BNK_FLAG>::run(g, d, smem, stages, t, part); \
        break;
#endif
        FT_FAMILY(FT_X)
#ifdef FT_GENERIC
        FT_FAMILY_PARTIAL(FT_X)
#endif
#undef FT_X
#if defined(FT_PP) && FT_CLASS == 1
#define FT_X(CODE, WM, WN, GM, GN, TWIN)                                        \
    case CODE:                                                                  \
        UKernelFast<FT_DT, WM, WN, GM, GN, 1>::run(g, d, smem, stages, t, part); \
        break;
        FT_FAMILY_W8(FT_X)
#undef FT_X
#endif
#if !defined(FT_GENERIC) && !defined(FT_PP) && !defined(FT_BNK)
#define FT_X(CODE, TM, TN, TWIN)                                                \
    case CODE:                                                                  \
        if constexpr ((TM) * (TN) / 64 <= FT_ACC_MAX)                           \
            UKernelSplitK<FT_DT, TM, TN>::run(g, d, smem, stages, t, part);  \
        break;
        FT_FAMILY_SPLITK(FT_X)
#undef FT_X
#endif
    default: break;
    }
#endif
}

}  // namespace ftk

extern "C" int FT_LAUNCH_NAME(const ftk::KArgs *args, uint32_t lds_bytes, void *stream) {
    // the attribute is kept per device: set it once on each device this kernel is launched on
    static std::mutex attr_mu;
    static bool attr_done[FT_MAX_DEVICES] = {};
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return (int)e;
        if (dev < 0 || dev >= FT_MAX_DEVICES) return (int)hipErrorInvalidDevice;
        std::lock_guard<std::mutex> lock(attr_mu);
        if (!attr_done[dev]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ftk::FT_KERNEL_NAME),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 163840);
            if (e != hipSuccess) return (int)e;
            attr_done[dev] = true;
        }
    }
    const uint32_t nx = args->num_xcds ? args->num_xcds : 1;
    uint32_t grid = args->table_order ? ftk::table_grid(args->n_tiles, nx) : args->n_tiles;
    if (args->k_parts > 1) grid = (grid + nx - 1) / nx * nx * args->k_parts;
    hipLaunchKernelGGL(ftk::FT_KERNEL_NAME, dim3(grid), dim3(FT_THREADS), lds_bytes,
                       static_cast<hipStream_t>(stream), *args);
    return (int)hipGetLastError();
}
