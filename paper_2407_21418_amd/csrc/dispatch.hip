// One dispatcher kernel per (input dtype, register class).  Workgroup i takes tile descriptor
// remap(i) and runs the uKernel body the descriptor names, so a single launch executes a
// program made of one or two uKernel shapes (Sec. 5.1; Fig. 8 item 2).
// Compiled once per -DFT_DT={0,1} -DFT_CLASS={0,1,2} with the fast bodies (LDS-DMA ring, aligned
// operands) and once per dtype with -DFT_CLASS=2 -DFT_GENERIC=1 for the general bodies (any
// alignment, ragged reduce axis, convolution gather).
#include "gemm_fast.h"
#include "family.h"
#include "launch_iface.h"

#ifndef FT_DT
#error "define FT_DT"
#endif
#ifndef FT_CLASS
#error "define FT_CLASS"
#endif

#if FT_CLASS == 0
#define FT_MIN_WAVES 4
#define FT_ACC_MAX 32
#elif FT_CLASS == 1
#define FT_MIN_WAVES 2
#define FT_ACC_MAX 128
#else
#define FT_MIN_WAVES 1
#define FT_ACC_MAX 256
#endif

namespace ftk {

// Workgroups are handed to the 8 XCDs round-robin (workgroup b runs on XCD b % 8).  Give each
// XCD one contiguous slice of the descriptor table, so tiles that share an A row panel (and
// walk the same B columns) meet in the same per-XCD L2.
__device__ __forceinline__ uint32_t xcd_remap(uint32_t b, uint32_t n, uint32_t nx) {
    uint32_t x = b % nx, j = b / nx;
    uint32_t q = n / nx, r = n % nx;
    return x * q + (x < r ? x : r) + j;
}

// Inside a constituent's tile grid (rows x cols per batch entry, row-major in the table) the
// sequence is walked in groups of G tile rows, column by column, so the tiles an XCD runs at
// once form a compact 2-D block: they share few A row panels AND few B column panels, which is
// what the per-XCD L2 can keep (a 1-D strip of tiles makes every XCD fetch all of B).  The host
// picks G per constituent from the tile shape and the number of tiles an XCD holds at once.
__device__ __forceinline__ uint32_t grouped_index(uint32_t u, uint32_t rows, uint32_t cols, uint32_t G) {
    if (rows < 2 || cols < 2 || G < 2) return u;
    const uint32_t per = rows * cols;
    const uint32_t bidx = u / per, v = u % per;
    const uint32_t grp = v / (G * cols), w = v % (G * cols);
    const uint32_t first = grp * G;
    const uint32_t gr = rows - first < G ? rows - first : G;
    return bidx * per + (first + w % gr) * cols + w / gr;
}

__global__ __launch_bounds__(256, FT_MIN_WAVES) void FT_KERNEL_NAME(KArgs g) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const uint32_t seq = xcd_remap(blockIdx.x, g.n_tiles, g.num_xcds);
    const uint32_t slot = seq >= g.slot_first[1] ? 1u : 0u;
    const uint32_t t = g.slot_first[slot] + grouped_index(seq - g.slot_first[slot], g.slot_rows[slot], g.slot_cols[slot], g.slot_group[slot]);
    const TileDesc d = g.descs[t];
    const uint32_t code = g.slot_code[slot];
    switch (code) {
#ifdef FT_GENERIC
#define FT_X(CODE, WM, WN, GM, GN)                                              \
    case CODE:                                                                  \
        UKernelBody<FT_DT, WM, WN, GM, GN, FT_TK>::run(g, d, smem);             \
        break;
#else
#define FT_X(CODE, WM, WN, GM, GN)                                              \
    case CODE:                                                                  \
        if constexpr ((WM) * (WN) / 64 <= FT_ACC_MAX)                           \
            UKernelFast<FT_DT, WM, WN, GM, GN>::run(g, d, smem, g.slot_stages[slot]); \
        break;
#endif
        FT_FAMILY(FT_X)
#undef FT_X
#ifndef FT_GENERIC
#define FT_X(CODE, TM, TN, TWIN)                                                \
    case CODE:                                                                  \
        if constexpr ((TM) * (TN) / 64 <= FT_ACC_MAX)                           \
            UKernelSplitK<FT_DT, TM, TN>::run(g, d, smem, g.slot_stages[slot]);  \
        break;
        FT_FAMILY_SPLITK(FT_X)
#undef FT_X
#endif
    default: break;
    }
}

}  // namespace ftk

extern "C" int FT_LAUNCH_NAME(const ftk::KArgs *args, uint32_t lds_bytes, void *stream) {
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&ftk::FT_KERNEL_NAME),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 163840);
        if (e != hipSuccess) return (int)e;
        attr_done = true;
    }
    hipLaunchKernelGGL(ftk::FT_KERNEL_NAME, dim3(args->n_tiles), dim3(256), lds_bytes,
                       static_cast<hipStream_t>(stream), *args);
    return (int)hipGetLastError();
}
