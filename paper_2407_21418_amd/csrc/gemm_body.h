// uKernel bodies for gfx950: one workgroup (4 wave64, one per SIMD) computes one output tile
//   C[m0:m0+TM, n0:n0+TN] (+batch) = sum_k A * B          (Sec. 3: uKernel = thread block)
// with v_mfma_f32_32x32x16 / v_mfma_f32_16x16x32 (f16 or bf16 in, fp32 accumulate).
//
// The tiling hierarchy of Fig. 7: block-level tile (i.0, j.0) = one tile descriptor;
// LDS tile (i.1, j.1) = TM x TN x TK staged in LDS, double buffered along k; register tile
// (i.2, j.2) = the WM x WN fp32 accumulator block each wave keeps in VGPR/AGPR.
//
// LDS layout (16-byte chunks = 8 elements):
//   A tile  [TM rows][TK]  k-contiguous, row pitch 128 B, chunk position = kc ^ swzA(row)
//   B tile  [TK rows][TN]  n-contiguous as in memory (no transpose on the way in), row pitch
//           2*TN B, chunk position = nc ^ swzB(row).  The MFMA B operand wants 8 consecutive
//           k per lane; ds_read_b64_tr_b16 transposes 4 rows x 16 columns on the way out.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace ftk {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

struct TileDesc {            // mirrors the 24-byte descriptor of the C ABI
    uint32_t ukernel_id, batch, m0, n0;
    uint16_t m_valid, n_valid;
    uint32_t flags;
};

// One group of a grouped launch: `batch` matrices of one shape, densely packed; the offsets are in
// elements from the launch's A, B and C pointers.
struct GroupRec {
    uint32_t m, n, k, batch;
    uint64_t offA, offB, offC;
};

struct KArgs {
    const uint16_t *A;
    const uint16_t *B;
    void *C;                          // fp32, or the 16-bit input type (out_kind)
    const float *bias;                // one fp32 per output column, or NULL
    uint32_t out_kind;                // OUT_F32 / OUT_F16 / OUT_BF16
    const TileDesc *descs;
    uint32_t n_tiles;
    uint32_t M, N, K;                 // GEMM view
    uint32_t lda, ldb, ldc;           // row pitches in elements
    uint64_t strideA, strideB, strideC;   // per-batch strides in elements
    uint32_t is_conv;
    uint32_t H, W, Cin, P, Q, R, S, cstride, cpad;   // conv geometry (A = NHWC image)
    uint32_t slot_ukernel[4];         // uKernel ids of the plan's constituents: two parts, then their strips
    uint32_t slot_code[4];            // their body codes in the compiled family
    uint32_t slot_stages[4];          // LDS ring depth of each (fast path)
    uint32_t table_order;             // 1: workgroup b takes descriptor b and finds its slot by uKernel id
    uint32_t slot_first[2];           // first descriptor of each constituent's block of the table
    uint32_t slot_rows[2];            // its tile grid per batch entry: rows (m) x columns (n)
    uint32_t slot_cols[2];
    uint32_t slot_group[2];           // tile rows walked together in the launch order (XCD locality)
    uint32_t slot_m0[2], slot_n0[2];  // origin of its block of tiles in the GEMM view
    uint32_t slot_tm[2], slot_tn[2];  // its tile extents
    uint32_t num_xcds;
    // reduce axis split over workgroups (1 = off): tile t is computed by k_parts workgroups, part p
    // taking k-tiles [p * k_part_tiles, (p + 1) * k_part_tiles); partial tiles meet in ws
    uint32_t k_parts, k_part_tiles;
    uint32_t ws_tile_stride;          // floats between consecutive (tile, part) slabs of ws
    uint32_t c_stream;                // 1: C is stored with the non-temporal hint (see store_acc_as)
    float *ws;                        // [n_tiles][k_parts][ws_tile_stride] fp32 partial tiles
    uint32_t *arrive;                 // [n_tiles][4] arrival counters, zero between launches
    const GroupRec *groups;           // grouped launch: shape and operand offsets of each group, else NULL
    uint64_t *trace;                  // development builds (-DFT_TRACE): 16 timestamps per workgroup, else NULL
};

// Development aid, compiled only with -DFT_TRACE: workgroup b leaves the device-wide 100 MHz counter
// at up to 8 points of its life in trace[16 b ..], so a launch can be laid out on one time axis
// (trace_timeline.py reads it; marks inside the k loop would disturb the loop's own in-order counters).
#ifdef FT_TRACE
#define FT_MARK(g, i)                                                                              \
    do {                                                                                           \
        if ((g).trace != nullptr && threadIdx.x == 0) (g).trace[blockIdx.x * 16u + (i)] = wall_clock64(); \
    } while (0)
#else
#define FT_MARK(g, i) do { } while (0)
#endif

enum { DT_F16 = 0, DT_BF16 = 1 };

template <int DT> __device__ __forceinline__ f32x16 mfma32(uint4 a, uint4 b, f32x16 c) {
    if constexpr (DT == DT_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                       __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                        __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
template <int DT> __device__ __forceinline__ f32x4 mfma16(uint4 a, uint4 b, f32x4 c) {
    if constexpr (DT == DT_F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                       __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                        __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// XOR swizzles on the 16-byte chunk index.  A: 128-byte rows; 16 consecutive rows at one
// logical chunk land on 16 distinct bank quads whether the LDS resolves 8 or 16 lanes per
// cycle.  B: a transposing read moves 8 bytes per lane, so 32 lanes (two 16-lane groups of
// 4 rows x 32 bytes) share the 64 banks of one cycle.  The two groups are either the two column
// halves of a 32-wide block at the same 4 rows (32x32x16) or the same columns at rows r and r+8
// (16x16x32): the XOR puts rows r..r+3 and r+8..r+11 on 8 distinct 32-byte bank groups and never
// touches chunk bit 0 (the 32-byte pair a group reads stays contiguous).
__device__ __forceinline__ uint32_t swzA(uint32_t row) { return (row ^ ((row >> 3) & 1u)) & 7u; }
template <int TN> __device__ __forceinline__ uint32_t swzB(uint32_t row) {
    if constexpr (TN >= 128) return ((row & 3u) << 2) | (((row >> 3) & 1u) << 1);
    else if constexpr (TN == 64) return (((row >> 1) & 1u) << 2) | (((row >> 3) & 1u) << 1);
    else if constexpr (TN == 32) return ((row >> 3) & 1u) << 1;
    else return 0u;
}

__device__ __forceinline__ uint4 ld16(const uint16_t *p) {
    return *reinterpret_cast<const uint4 *>(p);      // global_load_dwordx4; any 2-byte alignment
}

// 8 elements starting at p, of which the first nvalid (0..8) exist; the rest read as zero.
// Element by element: only for rows shorter than one chunk.
__device__ __forceinline__ uint4 ld_partial(const uint16_t *p, int nvalid) {
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < nvalid) w[e >> 1] |= (uint32_t)p[e] << ((e & 1) * 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// The 128-bit value v moved down by s elements of 16 bits, zeros moving in (s >= 8: all zero).
// Selects only, so that no lane waits on another's branch.
__device__ __forceinline__ uint4 shift_down_elems(uint4 v, uint32_t s) {
    const bool s4 = s & 4u, s2 = s & 2u, s1 = s & 1u;
    v = s4 ? make_uint4(v.z, v.w, 0u, 0u) : v;
    v = s2 ? make_uint4(v.y, v.z, v.w, 0u) : v;
    v = s1 ? make_uint4((v.x >> 16) | (v.y << 16), (v.y >> 16) | (v.z << 16), (v.z >> 16) | (v.w << 16), v.w >> 16) : v;
    return s >= 8u ? make_uint4(0u, 0u, 0u, 0u) : v;
}

// The first n (0..8) of the 8 elements of v, the others zero.
__device__ __forceinline__ uint4 keep_low_elems(uint4 v, uint32_t n) {
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (uint32_t i = 0; i < 4; ++i) w[i] = n >= 2 * i + 2 ? w[i] : (n == 2 * i + 1 ? (w[i] & 0xffffu) : 0u);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// The chunk of 8 elements at position x of a row of len >= 8 elements, elements beyond the row's
// end reading as zero.  A chunk that straddles the end is fetched as the row's last 8 elements
// and moved down, one 16-byte load from inside the row whatever x is: every lane issues its
// load at once, where element-wise loads under a branch would queue one latency after another.
__device__ __forceinline__ uint4 ld_row_chunk(const uint16_t *row, uint32_t x, uint32_t len, bool row_exists) {
    const bool full = x + 8u <= len;
    const uint32_t over = full ? 0u : (x + 8u - len < 8u ? x + 8u - len : 8u);
    const uint4 v = ld16(row + (full ? x : len - 8u));
    return shift_down_elems(v, row_exists ? over : 8u);
}

// Output element kinds of the epilogue: fp32, or the accumulator (+ bias) rounded once, to nearest
// even, to the 16-bit type of the inputs.
enum { OUT_F32 = 0, OUT_F16 = 1, OUT_BF16 = 2 };

template <int OUT> struct OutElem { using type = uint16_t; };
template <> struct OutElem<OUT_F32> { using type = float; };

template <int OUT> __device__ __forceinline__ typename OutElem<OUT>::type out_cvt(float v) {
    if constexpr (OUT == OUT_F32) {
        return v;
    } else if constexpr (OUT == OUT_F16) {
        return __builtin_bit_cast(uint16_t, static_cast<_Float16>(v));       // v_cvt_f16_f32: nearest even
    } else {
        uint32_t u = __builtin_bit_cast(uint32_t, v);
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)0x7fc0u;      // NaN stays NaN
        u += 0x7fffu + ((u >> 16) & 1u);                                     // nearest, ties to even
        return (uint16_t)(u >> 16);
    }
}

// Store of one wave's accumulator blocks (rows m0w.., columns n0w.. of C), optionally plus a
// per-column bias, as fp32 or rounded to 16 bits.
// 32x32 block: acc[4*i + j] -> row 8*i + 4*(lane/32) + j, column lane % 32
// 16x16 block: acc[j]       -> row 4*(lane/16) + j,        column lane % 16
// A wave tile that lies wholly inside C (uniform test) is stored without predication from one
// per-lane pointer: one 64-bit add per row, the column blocks go into the instruction offsets.
// C is written once and never read by this kernel. With STREAM the stores carry the non-temporal
// hint and stream past the caches instead of evicting the operand panels (measured: +6 % on the
// bench sweep). The hint is only safe for speed when every store instruction fills whole 64-byte
// blocks: partial blocks written this way are not merged in the L2 and cost 2-3x the time of a plain
// store (measured on fp32 score matrices with odd row pitch), so the host sets it per launch.
// BI0..BI1 / BJ0..BJ1: the rows / columns of accumulator blocks this call stores (all by default; a
// workgroup of two teams stores half of a wave tile from each).
template <int OUT, bool INTERIOR_PATH, bool STREAM, bool M16, int BM, int BN, int BI0 = 0, int BI1 = BM, int BJ0 = 0,
          int BJ1 = BN, typename Acc>
__device__ __forceinline__ void store_acc_as(void *Cv, uint64_t coff, const float *__restrict__ bias, uint32_t ldc,
                                             uint32_t M, uint32_t N, uint32_t m0w, uint32_t n0w, uint32_t lane,
                                             const Acc (&acc)[BM][BN]) {
    using T = typename OutElem<OUT>::type;
    T *__restrict__ Cb = static_cast<T *>(Cv) + coff;
    constexpr int MB = M16 ? 16 : 32, NE = M16 ? 4 : 16;
    const uint32_t lrow = 4 * (lane / MB), lcol = lane % MB;
    float bv[BN];
#pragma unroll
    for (int bj = BJ0; bj < BJ1; ++bj) {
        const uint32_t col = n0w + bj * MB + lcol;
        bv[bj] = (bias != nullptr && col < N) ? bias[col] : 0.f;
    }
    if (INTERIOR_PATH && m0w + BM * MB <= M && n0w + BN * MB <= N) {
        T *lp = Cb + ((uint64_t)(m0w + lrow) * ldc + n0w + lcol);
#pragma unroll
        for (int bi = BI0; bi < BI1; ++bi)
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const uint32_t r = bi * MB + (M16 ? e : 8 * (e / 4) + (e % 4));
                T *rp = lp + (uint64_t)r * ldc;
#pragma unroll
                for (int bj = BJ0; bj < BJ1; ++bj) {
                    const T v = out_cvt<OUT>(acc[bi][bj][e] + bv[bj]);
                    if constexpr (STREAM) __builtin_nontemporal_store(v, &rp[bj * MB]);
                    else rp[bj * MB] = v;
                }
            }
        return;
    }
    // Edge tile: buffer stores through a descriptor that covers exactly the valid rows of this wave
    // tile, so the hardware drops what lies beyond the last valid row; a lane whose column is
    // beyond N gets an offset past the descriptor's range (offsets inside a wave tile stay below
    // 2^31: the host rejects operands with a row pitch of 2^20 elements or more).
    const uint32_t m0u = __builtin_amdgcn_readfirstlane(m0w), n0u = __builtin_amdgcn_readfirstlane(n0w);
    if (m0u >= M || n0u >= N) return;
    constexpr uint32_t ES = sizeof(T);
    const uint32_t rows_valid = M - m0u < (uint32_t)(BM * MB) ? M - m0u : (uint32_t)(BM * MB);
    const uint32_t cols_valid = N - n0u < (uint32_t)(BN * MB) ? N - n0u : (uint32_t)(BN * MB);
    const uint32_t num_records = ((rows_valid - 1) * ldc + cols_valid) * ES;
    T *tile = Cb + ((uint64_t)m0u * ldc + n0u);
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(tile, 0, (int)num_records, 0x00020000);
    constexpr int AUX_NT = STREAM ? 2 : 0;   // cache-policy bits of the buffer instruction: nt (streaming)
    uint32_t vb[BN];
#pragma unroll
    for (int bj = BJ0; bj < BJ1; ++bj)
        vb[bj] = (bj * MB + lcol < cols_valid) ? (lrow * ldc + bj * MB + lcol) * ES : 0x80000000u;
#pragma unroll
    for (int bi = BI0; bi < BI1; ++bi)
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            const uint32_t r = bi * MB + (M16 ? e : 8 * (e / 4) + (e % 4));
            const uint32_t roff = r * ldc * ES;                       // uniform
#pragma unroll
            for (int bj = BJ0; bj < BJ1; ++bj) {
                const T v = out_cvt<OUT>(acc[bi][bj][e] + bv[bj]);
                if constexpr (OUT == OUT_F32)
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), rsrc, (int)(vb[bj] + roff), 0, AUX_NT);
                else
                    __builtin_amdgcn_raw_buffer_store_b16(v, rsrc, (int)(vb[bj] + roff), 0, AUX_NT);
            }
        }
}

// The output kind is uniform per launch: fp32 or the 16-bit type of the inputs (DT).
// INTERIOR_PATH = false keeps only the predicated loops (general bodies: less code).
template <int DT, bool INTERIOR_PATH, bool M16, int BM, int BN, int BI0 = 0, int BI1 = BM, int BJ0 = 0, int BJ1 = BN,
          typename Acc>
__device__ __forceinline__ void store_acc(const KArgs &g, uint64_t coff, uint32_t m0w, uint32_t n0w, uint32_t lane,
                                          const Acc (&acc)[BM][BN]) {
    constexpr int OUT16 = DT == 0 ? OUT_F16 : OUT_BF16;
    if (g.out_kind == OUT_F32) {
        if (g.c_stream) store_acc_as<OUT_F32, INTERIOR_PATH, true, M16, BM, BN, BI0, BI1, BJ0, BJ1>(g.C, coff, g.bias, g.ldc, g.M, g.N, m0w, n0w, lane, acc);
        else store_acc_as<OUT_F32, INTERIOR_PATH, false, M16, BM, BN, BI0, BI1, BJ0, BJ1>(g.C, coff, g.bias, g.ldc, g.M, g.N, m0w, n0w, lane, acc);
    } else {
        // 16-bit outputs are always streamed (the host never clears c_stream for them)
        store_acc_as<OUT16, INTERIOR_PATH, true, M16, BM, BN, BI0, BI1, BJ0, BJ1>(g.C, coff, g.bias, g.ldc, g.M, g.N, m0w, n0w, lane, acc);
    }
}

template <int DT, int WM, int WN, int GM, int GN, int TK>
struct UKernelBody {
    static constexpr int TM = GM * WM, TN = GN * WN;
    static constexpr bool M16 = (WM == 16);
    static constexpr int MB = M16 ? 16 : 32;          // MFMA output block edge
    static constexpr int KSTEP = M16 ? 32 : 16;       // k per MFMA
    static constexpr int BM = WM / MB, BN = WN / MB;  // accumulator blocks per wave
    static constexpr int NTHREADS = 256;
    static constexpr int A_CHUNKS = TM * TK / 8, B_CHUNKS = TK * TN / 8;
    static constexpr int A_ITERS = (A_CHUNKS + NTHREADS - 1) / NTHREADS;
    static constexpr int B_ITERS = (B_CHUNKS + NTHREADS - 1) / NTHREADS;
    static constexpr int A_BYTES = TM * TK * 2, B_BYTES = TK * TN * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int KCH = TK / 8;                // chunks per A row
    static constexpr int NCH = TN / 8;                // chunks per B row
    static_assert(TK == 64, "A-tile swizzle assumes 128-byte rows");
    static_assert(GM * GN <= 4, "at most four computing waves per workgroup");
    static constexpr bool PARTIAL = GM * GN < 4;      // waves >= GM*GN only copy

    using Acc = typename std::conditional<M16, f32x4, f32x16>::type;

    __device__ static __forceinline__ void run(const KArgs &g, const TileDesc &d, unsigned char *smem) {
        const uint32_t tid = threadIdx.x;
        const uint32_t lane = tid & 63u, wave = tid >> 6;
        const uint32_t wave_m = wave / GN, wave_n = wave % GN;
        const uint32_t m0 = d.m0, n0 = d.n0;
        const uint32_t M = g.M, N = g.N, K = g.K;
        const uint16_t *__restrict__ Ab = g.A + (uint64_t)d.batch * g.strideA;
        const uint16_t *__restrict__ Bb = g.B + (uint64_t)d.batch * g.strideB;

        // ---- per-thread copy assignments (loop invariant) -------------------------------
        // A copy: iteration i moves chunk (row0 + 32*i, kc); 32 rows keep the swizzle phase.
        uint32_t a_off[A_ITERS];                      // element offset of the chunk at k = 0
        uint32_t a_pix[A_ITERS];                      // conv: packed (p, q) origin
        const bool a_on = (A_CHUNKS % NTHREADS == 0) || tid < (uint32_t)A_CHUNKS;
        const uint32_t a_row0 = (tid / KCH) % TM, a_kc = tid % KCH;
        const uint32_t a_lds0 = a_row0 * (TK * 2) + ((a_kc ^ swzA(a_row0)) << 4);
        constexpr int A_RSTEP = NTHREADS / KCH;       // 32 rows per iteration
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            const uint32_t kc = a_kc;
            uint32_t gm = m0 + a_row0 + i * A_RSTEP;
            if (gm >= M) gm = M - 1;                  // clamp: garbage rows are never stored
            if (!g.is_conv) {
                a_off[i] = gm * g.lda + kc * 8;
                a_pix[i] = 0;
            } else {
                uint32_t img = gm / (g.P * g.Q), rem = gm % (g.P * g.Q);
                uint32_t p = rem / g.Q, q = rem % g.Q;
                a_off[i] = img * g.H * g.W * g.Cin;   // image base
                a_pix[i] = (p * g.cstride) << 16 | (q * g.cstride);
            }
        }
        // B copy: iteration i moves chunk (krow0 + i*B_RSTEP, nc)
        constexpr int B_RSTEP = (NTHREADS / NCH) > 0 ? (NTHREADS / NCH) : 1;
        const bool b_on = (B_CHUNKS % NTHREADS == 0) || tid < (uint32_t)B_CHUNKS;
        const uint32_t b_krow0 = (tid / NCH) % TK, b_nc = tid % NCH;
        const uint32_t b_col = n0 + b_nc * 8;
        const uint32_t b_ccol = (b_col + 8 <= N) ? b_col : n0;   // clamp: garbage columns are never stored
        const uint32_t b_off0 = b_krow0 * g.ldb + b_ccol;
        const uint32_t b_rstep_ld = B_RSTEP * g.ldb;
        // every B chunk of this tile is wholly inside or wholly outside [0, N)
        const bool b_fast = (N % 8 == 0) || (n0 + TN <= N);
        const bool a_vec_conv = (g.Cin % 8 == 0);

        // ---- fragment read addresses (loop invariant apart from the k step) -------------
        // A operand: lane holds 8 consecutive k of one row.
        //   32x32x16: row = lane % 32, k chunk = 2*ks + lane / 32
        //   16x16x32: row = lane % 16, k chunk = 4*ks + lane / 16
        uint32_t fa_row[BM];
#pragma unroll
        for (int bi = 0; bi < BM; ++bi) fa_row[bi] = wave_m * WM + bi * MB + (lane % MB);
        const uint32_t fa_kc = lane / MB;
        // B operand through the transposing read: a 16-lane group fetches 4 k-rows x 16 columns;
        // lane j of the group supplies the address of row j/4, columns 4*(j%4)..+3 and receives
        // column j, rows 0..3.  Group -> (column half, k half) as the MFMA operand layout asks.
        const uint32_t j16 = lane & 15u;
        uint32_t fb_colgrp, fb_k8;                     // 16-column group inside the block; k offset / 8
        if constexpr (M16) { fb_colgrp = 0; fb_k8 = lane >> 4; }
        else { fb_colgrp = (lane >> 4) & 1u; fb_k8 = lane >> 5; }
        const uint32_t fb_rowin = j16 >> 2;            // row inside the 4-row group
        const uint32_t fb_cole = (j16 & 3u) * 4;       // element column inside the 16-col group

        Acc acc[BM][BN];
#pragma unroll
        for (int bi = 0; bi < BM; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj)
#pragma unroll
                for (int e = 0; e < (M16 ? 4 : 16); ++e) acc[bi][bj][e] = 0.f;

        uint4 ra[A_ITERS], rb[B_ITERS];

        auto load_a = [&](uint32_t k0, bool careful) {
            if (!a_on) return;
            const uint32_t kk = k0 + a_kc * 8;
#pragma unroll
            for (int i = 0; i < A_ITERS; ++i) {
                if (!g.is_conv) {
                    const uint16_t *p = Ab + a_off[i] + k0;
                    if (!careful) ra[i] = ld16(p);
                    else if (K >= 8u) ra[i] = ld_row_chunk(p - kk, kk, K, true);
                    else ra[i] = ld_partial(p, kk < K ? (int)(K - kk) : 0);
                } else {
                    // k = (r*S + s)*Cin + c ; input pixel (p*stride - pad + r, q*stride - pad + s)
                    uint32_t p0 = a_pix[i] >> 16, q0 = a_pix[i] & 0xffffu;
                    if (a_vec_conv) {
                        uint32_t tap = kk / g.Cin, ch = kk % g.Cin;
                        uint32_t r = tap / g.S, s = tap % g.S;
                        int h = (int)(p0 + r) - (int)g.cpad, w = (int)(q0 + s) - (int)g.cpad;
                        bool ok = kk < K && h >= 0 && h < (int)g.H && w >= 0 && w < (int)g.W;
                        ra[i] = ok ? ld16(Ab + a_off[i] + ((uint32_t)h * g.W + (uint32_t)w) * g.Cin + ch)
                                   : make_uint4(0, 0, 0, 0);
                    } else {
                        // channel count not a multiple of 8: the chunk's 8 elements come from up to 8
                        // (tap, channel) positions.  One division finds the first; the others follow by
                        // counting.  Every load is issued unconditionally (from the image's first element
                        // where the position is in the halo or beyond K) and masked afterwards, so the
                        // eight loads of a chunk, and those of the other chunks, are in flight together.
                        uint32_t tap = kk / g.Cin, ch = kk % g.Cin;
                        uint32_t r = tap / g.S, sx = tap % g.S;
                        uint32_t val[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int h = (int)(p0 + r) - (int)g.cpad, w = (int)(q0 + sx) - (int)g.cpad;
                            const bool ok = kk + e < K && h >= 0 && h < (int)g.H && w >= 0 && w < (int)g.W;
                            const uint32_t idx = ok ? ((uint32_t)h * g.W + (uint32_t)w) * g.Cin + ch : 0u;
                            const uint32_t x = Ab[a_off[i] + idx];
                            val[e] = ok ? x : 0u;
                            if (++ch == g.Cin) {
                                ch = 0;
                                if (++sx == g.S) { sx = 0; ++r; }
                            }
                        }
                        uint32_t wv[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) wv[e] = val[2 * e] | (val[2 * e + 1] << 16);
                        ra[i] = make_uint4(wv[0], wv[1], wv[2], wv[3]);
                    }
                }
            }
        };
        auto load_b = [&](uint32_t k0, bool careful) {
            if (!b_on) return;
            const uint16_t *pk = Bb + k0 * g.ldb;
#pragma unroll
            for (int i = 0; i < B_ITERS; ++i) {
                const uint16_t *p = pk + (b_off0 + i * b_rstep_ld);
                if (!careful) { rb[i] = ld16(p); continue; }
                uint32_t kr = k0 + b_krow0 + i * B_RSTEP;
                if (N >= 8u) {
                    rb[i] = ld_row_chunk(Bb + (kr < K ? kr : K - 1u) * g.ldb, b_col, N, kr < K);
                    continue;
                }
                if (kr >= K) rb[i] = make_uint4(0, 0, 0, 0);
                else if (b_col + 8 <= N) rb[i] = ld16(p);
                else if (b_col < N) rb[i] = ld_partial(Bb + (kr * g.ldb + b_col), (int)(N - b_col));
                else rb[i] = make_uint4(0, 0, 0, 0);
            }
        };
        auto store_lds = [&](uint32_t stage) {
            unsigned char *base = smem + stage * STAGE_BYTES;
            if (a_on) {
#pragma unroll
                for (int i = 0; i < A_ITERS; ++i)
                    *reinterpret_cast<uint4 *>(base + a_lds0 + i * (A_RSTEP * TK * 2)) = ra[i];
            }
            if (b_on) {
#pragma unroll
                for (int i = 0; i < B_ITERS; ++i) {
                    const uint32_t row = b_krow0 + i * B_RSTEP;
                    *reinterpret_cast<uint4 *>(base + A_BYTES + row * (TN * 2) + ((b_nc ^ swzB<TN>(row)) << 4)) = rb[i];
                }
            }
        };
        auto compute = [&](uint32_t stage) {
            const unsigned char *sa = smem + stage * STAGE_BYTES;
            const unsigned char *sb = sa + A_BYTES;
#pragma unroll
            for (int ks = 0; ks < TK / KSTEP; ++ks) {
                uint4 fa[BM], fb[BN];
#pragma unroll
                for (int bi = 0; bi < BM; ++bi) {
                    uint32_t kc = ks * (KSTEP / 8) + fa_kc;
                    fa[bi] = *reinterpret_cast<const uint4 *>(sa + fa_row[bi] * (TK * 2) +
                                                              ((kc ^ swzA(fa_row[bi])) << 4));
                }
#pragma unroll
                for (int bj = 0; bj < BN; ++bj) {
                    uint32_t col = wave_n * WN + bj * MB + fb_colgrp * 16 + fb_cole;
                    uint32_t nc = col >> 3, cin = (col & 7u) * 2;
                    s16x4 h[2];
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        uint32_t row = ks * KSTEP + fb_k8 * 8 + hh * 4 + fb_rowin;
                        uint32_t off = row * (TN * 2) + ((nc ^ swzB<TN>(row)) << 4) + cin;
                        h[hh] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(sb + off));
                    }
                    uint2 lo = __builtin_bit_cast(uint2, h[0]), hi = __builtin_bit_cast(uint2, h[1]);
                    fb[bj] = make_uint4(lo.x, lo.y, hi.x, hi.y);
                }
#pragma unroll
                for (int bi = 0; bi < BM; ++bi)
#pragma unroll
                    for (int bj = 0; bj < BN; ++bj) {
                        if constexpr (M16) acc[bi][bj] = mfma16<DT>(fa[bi], fb[bj], acc[bi][bj]);
                        else acc[bi][bj] = mfma32<DT>(fa[bi], fb[bj], acc[bi][bj]);
                    }
            }
        };

        // ---- main loop: double-buffered LDS, global loads of tile kt+1 overlap MFMA of kt ----
        const uint32_t nk = (K + TK - 1) / TK;
        const bool k_tail = (K % TK) != 0;
        if (nk > 0) {
            const bool tail0 = (nk == 1) && k_tail;
            load_a(0, tail0);
            load_b(0, tail0 || !b_fast);
            store_lds(0);
            __syncthreads();
            for (uint32_t kt = 0; kt < nk; ++kt) {
                const bool more = kt + 1 < nk;
                if (more) {
                    bool last = (kt + 2 == nk) && k_tail;
                    load_a((kt + 1) * TK, last);
                    load_b((kt + 1) * TK, last || !b_fast);
                }
                if (!PARTIAL || wave < (uint32_t)(GM * GN)) compute(kt & 1u);
                if (more) store_lds((kt + 1) & 1u);
                __syncthreads();
            }
        }

        // ---- epilogue: fp32 store, predicated only for tiles on the edge of C --------------
        if (!PARTIAL || wave < (uint32_t)(GM * GN))
            store_acc<DT, false, M16, BM, BN>(g, (uint64_t)d.batch * g.strideC, m0 + wave_m * WM, n0 + wave_n * WN, lane, acc);
    }
};

}  // namespace ftk
