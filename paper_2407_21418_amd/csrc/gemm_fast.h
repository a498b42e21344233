// Fast uKernel bodies for gfx950 (aligned Matmul / BMM operands).
//
// Same tiling hierarchy and LDS layout as gemm_body.h, but the copy global -> LDS never touches
// registers: global_load_lds_dwordx4 (one wave instruction = 64 lanes x 16 B = 1 KB of contiguous
// LDS, each lane fetching from its own global address) fills a ring of `stages` LDS buffers, so
// stages-1 k-tiles are in flight while the MFMAs consume the oldest one.  The XOR swizzles are
// applied on the *source* side: the lane that owns LDS chunk position p of a row fetches global
// chunk p ^ swz(row).
//
// The LDS reads of the MFMA fragments are issued as inline asm with hand-placed s_waitcnt, so the
// compiler's conservative "wait for every outstanding LDS-DMA before any LDS read" does not
// serialise the ring.  Register cost per lane: accumulators + two fragment sets + a few addresses.
//
// Preconditions (checked by the host before this path is chosen): A, B 16-byte aligned; row
// pitches lda, ldb and K, N multiples of 8 elements; for a convolution c_in a multiple of 64
// (a k-tile then lies inside one filter tap) and c_out a multiple of 8.
#pragma once
#include "family.h"
#include "gemm_body.h"

namespace ftk {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// 256 bytes of zeros: source of k-tail chunks (rows/columns of the reduce axis beyond K)
__device__ __attribute__((aligned(256))) uint32_t ft_zero_page[64];

// -DFT_NO_RAGGED: bodies without the code for rows that end inside a 16-byte chunk (see UKernelFast::run).
// The dispatchers of the plain launches are compiled both ways, so that the ones that run launches with
// whole chunks carry none of it (it costs them scalar registers and about one per cent).
// The dispatchers of grouped launches keep the general bookkeeping of the k loops (ring depth as planned, stage
// indices by division): with the leaner forms below their largest bodies no longer fit the register budget.
#ifdef FT_GROUPED
constexpr bool kLeanLoop = false;
#else
constexpr bool kLeanLoop = true;
#endif
// tiles a single-team body keeps in flight beyond the one it consumes, at most (measured: four are slower
// again than three)
#ifndef FT_DMAX
#define FT_DMAX 3
#endif
#ifdef FT_NO_RAGGED
constexpr bool kRaggedRows = false;
#else
constexpr bool kRaggedRows = true;
#endif

template <int OFF> __device__ __forceinline__ u32x4 lds_read_b128(uint32_t addr) {
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF> __device__ __forceinline__ u32x2 lds_read_b64(uint32_t addr) {
    u32x2 v;
    asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int OFF> __device__ __forceinline__ u32x2 lds_read_tr16_b64(uint32_t addr) {
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ void lds_dma16(const void *gptr, unsigned char *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gptr,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

// Reduce axis split over workgroups: the k_parts workgroups of one tile each leave their fp32
// partial in the workspace, one slab per (tile, part), laid out [register][lane] per wave so every
// store and load is one contiguous 256-byte line per wave.  Arrival is counted per (tile, wave):
// a wave writes its lines, waits until they are acknowledged, bumps the counter, and the wave that
// arrives last sums the k_parts slabs in part order (the result does not depend on who came last),
// resets the counter for the next launch and runs the normal epilogue.  Nobody waits for anybody.
//
// Coherence between the XCDs' L2 caches is kept per access, not per cache: the partials are written
// and read as relaxed agent-scope atomics (stores that write through, loads that do not trust a
// cached copy), so no whole-L2 write-back / invalidate is needed -- an agent-scope release/acquire
// fence pair here cost 40 us per launch, several times the GEMM itself.  Ordering: the wave's
// stores are complete when its vmcnt reaches zero, before the counter is touched; the loads of
// the last wave are issued after its counter increment has returned.
__device__ __forceinline__ bool k_part_arrive_last(const KArgs &g, uint32_t t, uint32_t wave) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    uint32_t *ctr = g.arrive + (t * 4u + wave);
    uint32_t old = 0;
    if ((threadIdx.x & 63u) == 0)
        old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    asm volatile("" ::: "memory");
    if (old + 1 != g.k_parts) return false;
    if ((threadIdx.x & 63u) == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return true;
}

// This wave's values <-> its lines of the slab of (tile t, part): floats [wave * NREGW + r][lane].
// get(r) / set(r, x) read and write value r in place (accumulator registers: a copy would double
// the register need of the largest tiles).
template <int NREGW, typename Get, typename Set>
__device__ __forceinline__ bool k_part_exchange(const KArgs &g, uint32_t t, uint32_t part, uint32_t wave,
                                                uint32_t lane, Get get, Set set) {
    const uint64_t tile0 = (uint64_t)t * g.k_parts * g.ws_tile_stride;
    const uint32_t in_slab = wave * (NREGW * 64) + lane;
    float *mine = g.ws + tile0 + (uint64_t)part * g.ws_tile_stride + in_slab;
#pragma unroll
    for (int r = 0; r < NREGW; ++r) __hip_atomic_store(mine + r * 64, get(r), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!k_part_arrive_last(g, t, wave)) return false;
    float *p = g.ws + tile0 + in_slab;
#pragma unroll
    for (int r = 0; r < NREGW; ++r) set(r, __hip_atomic_load(p + r * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    for (uint32_t q = 1; q < g.k_parts; ++q) {
        p += g.ws_tile_stride;
#pragma unroll
        for (int r = 0; r < NREGW; ++r) set(r, get(r) + __hip_atomic_load(p + r * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    return true;
}

// s_waitcnt vmcnt(0) that also "produces" the registers of one row of blocks: the loads into them
// are all issued above it and no use of them can be scheduled above it.
template <int BN, typename Blk>
__device__ __forceinline__ void landed(Blk (&row)[BN]) {
    static_assert(BN == 1 || BN == 2 || BN == 4 || BN == 8, "blocks per row of a wave tile");
    if constexpr (BN == 1) asm volatile("s_waitcnt vmcnt(0)" : "+v"(row[0]) :: "memory");
    else if constexpr (BN == 2) asm volatile("s_waitcnt vmcnt(0)" : "+v"(row[0]), "+v"(row[1]) :: "memory");
    else if constexpr (BN == 4)
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(row[0]), "+v"(row[1]), "+v"(row[2]), "+v"(row[3]) :: "memory");
    else
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(row[0]), "+v"(row[1]), "+v"(row[2]), "+v"(row[3]), "+v"(row[4]),
                     "+v"(row[5]), "+v"(row[6]), "+v"(row[7]) :: "memory");
}

// The exchange for a wave's accumulator blocks (register r = ((bi * BN) + bj) * NE + e, as the slab
// layout numbers them).  The loads of a slab are in flight together: into the accumulators themselves
// for the first slab, into temporaries for the others -- a whole tile of them where it has at most
// 64 registers, else one row of blocks at a time.  Written out this way because the compiler, left to
// itself, waits for each load of a 128-register tile before it issues the next (measured: 27 us per
// slab instead of 2).
template <bool M16, int BM, int BN, typename Acc>
__device__ __forceinline__ bool k_part_exchange_blocks(const KArgs &g, uint32_t t, uint32_t part, uint32_t wave,
                                                       uint32_t lane, Acc (&acc)[BM][BN]) {
    constexpr int NE = M16 ? 4 : 16, NREGW = BM * BN * NE;
    constexpr int RB = NREGW <= 64 ? BM : 1;          // rows of blocks per batch of loads
    const uint64_t tile0 = (uint64_t)t * g.k_parts * g.ws_tile_stride;
    const uint32_t in_slab = wave * (NREGW * 64) + lane;
    float *mine = g.ws + tile0 + (uint64_t)part * g.ws_tile_stride + in_slab;
#pragma unroll
    for (int bi = 0; bi < BM; ++bi)
#pragma unroll
        for (int bj = 0; bj < BN; ++bj)
#pragma unroll
            for (int e = 0; e < NE; ++e)
                __hip_atomic_store(mine + ((bi * BN + bj) * NE + e) * 64, acc[bi][bj][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!k_part_arrive_last(g, t, wave)) return false;
    const float *p = g.ws + tile0 + in_slab;
#pragma unroll
    for (int b0 = 0; b0 < BM; b0 += RB) {
#pragma unroll
        for (int bi = b0; bi < b0 + RB; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj)
#pragma unroll
                for (int e = 0; e < NE; ++e)
                    acc[bi][bj][e] = __hip_atomic_load(p + ((bi * BN + bj) * NE + e) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int bi = b0; bi < b0 + RB; ++bi) landed<BN>(acc[bi]);
    }
    for (uint32_t q = 1; q < g.k_parts; ++q) {
        p += g.ws_tile_stride;
#pragma unroll
        for (int b0 = 0; b0 < BM; b0 += RB) {
            Acc other[RB][BN];
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int bj = 0; bj < BN; ++bj)
#pragma unroll
                    for (int e = 0; e < NE; ++e)
                        other[i][bj][e] = __hip_atomic_load(p + (((b0 + i) * BN + bj) * NE + e) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int i = 0; i < RB; ++i) landed<BN>(other[i]);
#pragma unroll
            for (int i = 0; i < RB; ++i)
#pragma unroll
                for (int bj = 0; bj < BN; ++bj)
#pragma unroll
                    for (int e = 0; e < NE; ++e) acc[b0 + i][bj][e] += other[i][bj][e];
        }
    }
    return true;
}

// TEAMS = 2 ("ping-pong"): the workgroup has eight waves, two per SIMD, in two teams of four.  A team
// is a complete GM x GN wave grid with an LDS ring of its own; the teams take alternate k-tiles of the
// SAME output tile and add their partial sums through LDS at the end.  The workgroup moves in phases
// separated by s_barrier: while one team reads fragments and runs the MFMAs of its current k-tile, the
// other issues the LDS-DMA copies of a later one and waits for its next to land; then they swap.  A
// wave is held up while its copy instructions are accepted (measured: about as long as the MFMAs of a
// k-tile take), so with one wave per SIMD copy and MFMA time add up; with two teams the SIMD's other
// wave computes meanwhile.
// BNK: operand B is given as [N][K] (k contiguous, the layout of A; an attention's K matrix in Q K^T, a
// linear layer's weight as stored): its tile is copied and laid out in LDS exactly like A's, rows
// being output columns, and its fragments are read with plain reads instead of transposing ones.
template <int DT, int WM, int WN, int GM, int GN, int TEAMS = 1, bool BNK = false>
struct UKernelFast {
    static_assert(TEAMS == 1 || TEAMS == 2, "one team of four waves, or two");
    static_assert(!BNK || (TEAMS == 1 && GM * GN == 4), "the [N][K] layout is built for the four-wave grids");
    // A single team may also be a grid of EIGHT waves (GM * GN = 8, two per SIMD) that share every
    // k-tile: a 256 x 256 tile then costs a wave 128 accumulator registers instead of 256, and while
    // one wave of a SIMD is held up issuing copies or waiting for fragments the other runs MFMAs.
    static constexpr int NWT = GM * GN;               // waves of a team
    static_assert(NWT == 4 || (NWT == 8 && TEAMS == 1) || NWT == 1,
                  "four waves per team; eight in a single team (a 1 x 1 grid lends its fragment helpers to the split-k bodies)");
    static constexpr int TK = 64;
    static constexpr int TM = GM * WM, TN = GN * WN;
    static constexpr bool M16 = (WM == 16);
    static constexpr int MB = M16 ? 16 : 32;
    static constexpr int KSTEP = M16 ? 32 : 16;
    static constexpr int KS = TK / KSTEP;             // MFMA k-steps per tile
    static constexpr int BM = WM / MB, BN = WN / MB;
    static constexpr int A_BYTES = TM * TK * 2, B_BYTES = TK * TN * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    // wave-level copy instructions per stage: each wave of the team moves an equal share of A's rows
    // and of B's rows; a share smaller than 1 KB is moved by the low lanes only
    static constexpr int A_WAVE_BYTES = A_BYTES / (NWT == 1 ? 4 : NWT), B_WAVE_BYTES = B_BYTES / (NWT == 1 ? 4 : NWT);
    static constexpr int LA = (A_WAVE_BYTES + 1023) / 1024, LB = (B_WAVE_BYTES + 1023) / 1024;
    static constexpr int L = LA + LB;                 // vmcnt increments per stage per wave
    static constexpr int MAX_AHEAD = (63 / L) < 6 ? (63 / L) : 6;   // tiles in flight beyond the current
    static constexpr int NR = BM + 2 * BN;            // LDS read instructions per k-step
    static_assert(NR <= 15, "lgkmcnt is 4 bits");
    using Acc = typename std::conditional<M16, f32x4, f32x16>::type;
    // the lean bookkeeping of the k loop (see run): not for grouped launches and not for the bodies with
    // 256 accumulator registers (one wave per SIMD in a 512-register kernel), which measured 2-10 % slower
    // with it, most with the convolution gather in the loop
    static constexpr bool LEAN = kLeanLoop && WM * WN / 64 <= 128;

    // wait until at most `ahead` (LO..HI) whole stages of this wave's copies are outstanding: the count is
    // an immediate of the instruction, so a runtime `ahead` is a decision tree (three compares at most)
    template <int LO, int HI> __device__ static __forceinline__ void wait_tiles_in(uint32_t ahead) {
        if constexpr (LO == HI) wait_vmcnt<LO * L>();
        else {
            constexpr int MID = (LO + HI) / 2;
            if (ahead <= (uint32_t)MID) wait_tiles_in<LO, MID>(ahead);
            else wait_tiles_in<MID + 1, HI>(ahead);
        }
    }
    template <int T> __device__ static __forceinline__ void wait_tiles_chain(int ahead) {
        if constexpr (T >= MAX_AHEAD) wait_vmcnt<MAX_AHEAD * L>();
        else {
            if (ahead <= T) wait_vmcnt<T * L>();
            else wait_tiles_chain<T + 1>(ahead);
        }
    }
    __device__ static __forceinline__ void wait_tiles(uint32_t ahead) {
        if constexpr (LEAN) wait_tiles_in<0, MAX_AHEAD>(ahead > (uint32_t)MAX_AHEAD ? (uint32_t)MAX_AHEAD : ahead);
        else wait_tiles_chain<0>((int)ahead);
    }

    __device__ static __forceinline__ void run(const KArgs &g, const TileDesc &d, unsigned char *smem,
                                               uint32_t stages_in, uint32_t t, uint32_t part) {
        const uint32_t tid = threadIdx.x;
        const uint32_t lane = tid & 63u;
        const uint32_t wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
        const uint32_t team = TEAMS == 2 ? wave_all >> 2 : 0u;         // waves 0-3 / 4-7: one wave per SIMD each
        const uint32_t wave = TEAMS == 2 ? wave_all & 3u : wave_all;   // position in the team's wave grid
        const uint32_t wave_m = wave / GN, wave_n = wave % GN;
        const uint32_t m0 = d.m0, n0 = d.n0;
        const uint32_t M = g.M, N = g.N, K = g.K;
        const uint16_t *__restrict__ Ab = g.A + (uint64_t)d.batch * g.strideA;
        const uint16_t *__restrict__ Bb = g.B + (uint64_t)d.batch * g.strideB;
        // this workgroup's k-tiles: kt0 .. kt0 + nk - 1 of the nk_all of the reduce axis
        const uint32_t nk_all = (K + TK - 1) / TK;
        const uint32_t kt0 = part * g.k_part_tiles;
        const uint32_t nk = g.k_parts > 1 ? (nk_all - kt0 < g.k_part_tiles ? nk_all - kt0 : g.k_part_tiles) : nk_all;
        uint32_t S = stages_in < 2 ? 2u : stages_in;
        if (S > (uint32_t)MAX_AHEAD + 2) S = MAX_AHEAD + 2;
        unsigned char *const smem_all = smem;
        if constexpr (TEAMS == 2) smem += team * S * STAGE_BYTES;      // this team's ring

        // ---- copy assignments ---------------------------------------------------------------
        // A instruction i of this wave fills LDS bytes [wave*A_WAVE_BYTES + i*1024, +1024) of the
        // A tile: row = that offset / 128 (+ lane / 8), chunk position = lane % 8.
        // Convolution (implicit GEMM, c_in a multiple of the k-tile): row = output pixel (n,p,q); one
        // k-tile lies inside one filter tap (r,s), so the lane's source is pixel (p*stride-pad+r,
        // q*stride-pad+s) of its image, channels ch0 + 8*kc .. +7, or the zero page in the halo.
        // Source offsets are kept in BYTES relative to the (uniform) operand base, so a copy is
        // "scalar base of this k-tile + 32-bit lane offset": one instruction, no 64-bit vector math.
        uint32_t goff_a[LA];
        uint32_t a_pq[LA];                            // conv: (p*stride) << 16 | (q*stride)
        {
            uint32_t row0 = (wave * A_WAVE_BYTES) / 128 + lane / 8;
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                uint32_t row = row0 + i * 8;
                uint32_t kc = (lane & 7u) ^ swzA(row);
                uint32_t gm = m0 + row;
                if (gm >= M) gm = M - 1;              // clamp: garbage rows are never stored
                if (!g.is_conv) {
                    goff_a[i] = (gm * g.lda + kc * 8) * 2;
                    a_pq[i] = 0;
                } else {
                    uint32_t img = gm / (g.P * g.Q), rem = gm % (g.P * g.Q);
                    uint32_t pp = rem / g.Q, qq = rem % g.Q;
                    goff_a[i] = (img * g.H * g.W * g.Cin + kc * 8) * 2;
                    a_pq[i] = (pp * g.cstride) << 16 | (qq * g.cstride);
                }
            }
        }
        const bool a_lane_on = (A_WAVE_BYTES >= 1024) || lane < (uint32_t)(A_WAVE_BYTES / 16);
        // B instruction i fills bytes [wave*B_WAVE_BYTES + i*1024, +1024) of the B tile.
        uint32_t goff_b[LB];
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            if constexpr (!BNK) {
                uint32_t o = wave * B_WAVE_BYTES + i * 1024 + lane * 16;
                uint32_t krow = o / (TN * 2), p = (o % (TN * 2)) / 16;
                uint32_t nc = p ^ swzB<TN>(krow);
                uint32_t col = n0 + nc * 8;
                if (col >= N) col = n0;               // clamp: garbage columns are never stored
                goff_b[i] = (krow * g.ldb + col) * 2;
            } else {
                // as A: LDS row = output column of the tile, 128 bytes of k each
                uint32_t row = (wave * B_WAVE_BYTES + i * 1024) / 128 + lane / 8;
                uint32_t kc = (lane & 7u) ^ swzA(row);
                uint32_t gn = n0 + row;
                if (gn >= N) gn = N - 1;              // clamp: garbage columns are never stored
                goff_b[i] = (gn * g.ldb + kc * 8) * 2;
            }
        }
        const bool b_lane_on = (B_WAVE_BYTES >= 1024) || lane < (uint32_t)(B_WAVE_BYTES / 16);
        // Ragged edges (the copies take any 2-byte aligned source, so row pitches may be anything).
        // K % 8 != 0: the reduce extent ends inside a 16-byte chunk of A's rows (and of B's, stored [N][K]).
        // Such a chunk is fetched as the row's LAST 8 elements -- inside the row, so inside the operand --
        // and moved down in LDS once the tile has landed (fix_edges), zeros moving in: elements beyond K
        // multiply as zero whatever follows the row.  N % 8 != 0 with B stored [K][N]: what a lane reads
        // beyond N belongs to the next row and only reaches output columns that are never stored; only
        // the operand's last row (k = K - 1) must not be read past its end and is fetched the same way.
        // The host sends such launches here only for the single-team bodies, with N >= 8 where B is stored
        // [K][N], and with K >= 8 -- or, in a grouped launch, with a shorter reduce axis where 8 elements from
        // the start of a group's last row still lie inside the packed buffer: rows shorter than a chunk are
        // fetched as they lie and what follows them is cleared in LDS.
        // (Everything about them is computed where it is used, in the last k-tile: nothing more stays
        // live in scalar registers through the loop.)
        const bool k_tail = (K % TK) != 0 || (kRaggedRows && !BNK && !g.is_conv && (N % 8u) != 0);   // the last k-tile takes the checked copy code

        auto issue_impl = [&](uint32_t kt, uint32_t stage_off, auto tail_c) {
            constexpr bool tail = decltype(tail_c)::value;
            unsigned char *st = smem + stage_off;
            // (two teams: kt counts this team's k-tiles, every other one of the workgroup's)
            const uint32_t k0 = (TEAMS == 2 ? kt0 + team + 2 * kt : kt0 + kt) * TK;
            // byte offsets inside one batch entry fit 32 bits (the host rejects larger operands)
            const char *abase = reinterpret_cast<const char *>(Ab), *bbase = reinterpret_cast<const char *>(Bb);
            const uint32_t ka = k0 * 2, kb = k0 * g.ldb * 2;                                        // uniform
            // (the last k-tile's checks work on copies the compiler cannot see through: what they derive
            // from K, N and the pitch is then computed here, not kept in scalar registers through the loop)
            uint32_t Kt = K, Nt = N, ldbt = g.ldb;
            if constexpr (tail && kRaggedRows) asm volatile("" : "+s"(Kt), "+s"(Nt), "+s"(ldbt));
            if (!g.is_conv) {
#pragma unroll
                for (int i = 0; i < LA; ++i) {
                    const void *p = abase + (uint32_t)(goff_a[i] + ka);
                    if constexpr (tail) {
                        // logical chunk of this lane in instruction i (recomputed: tail tile only)
                        uint32_t row = (wave * A_WAVE_BYTES) / 128 + lane / 8 + i * 8;
                        uint32_t kc = (lane & 7u) ^ swzA(row);
                        if (k0 + kc * 8 >= Kt) p = ft_zero_page;
                        // the row's last 8 elements (a row shorter than that is fetched as it lies, with what follows
                        // it: the host has checked that this stays inside the operand buffer; fix_edges clears it)
                        else if (kRaggedRows && k0 + kc * 8 + 8 > Kt && Kt >= 8u) p = abase + (uint32_t)(goff_a[i] - kc * 16 + (Kt - 8u) * 2);
                    }
                    if (a_lane_on) lds_dma16(p, st + wave * A_WAVE_BYTES + i * 1024);
                }
            } else {
                const uint32_t tap = k0 / g.Cin, ch0 = k0 % g.Cin;       // uniform: c_in % 64 == 0
                const uint32_t r = tap / g.S, sx = tap % g.S;
#pragma unroll
                for (int i = 0; i < LA; ++i) {
                    const int h = (int)((a_pq[i] >> 16) + r) - (int)g.cpad;
                    const int w = (int)((a_pq[i] & 0xffffu) + sx) - (int)g.cpad;
                    // (one unsigned compare per coordinate, joined without short-circuit: written with && the
                    // compiler has at times turned the four tests of every copy into masked control flow,
                    // 10 % of a convolution's time)
                    const bool ok = ((uint32_t)h < g.H) & ((uint32_t)w < g.W);
                    // 32-bit byte offset first, one 64-bit add last (keeps the lane offsets in one register each)
                    const uint32_t off = goff_a[i] + (((uint32_t)h * g.W + (uint32_t)w) * g.Cin + ch0) * 2;
                    const void *p = ok ? static_cast<const void *>(abase + off) : static_cast<const void *>(ft_zero_page);
                    if (a_lane_on) lds_dma16(p, st + wave * A_WAVE_BYTES + i * 1024);
                }
            }
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                const void *p = bbase + (uint32_t)(goff_b[i] + (BNK ? ka : kb));
                if constexpr (tail) {
                    if constexpr (!BNK) {
                        uint32_t o = wave * B_WAVE_BYTES + i * 1024 + lane * 16;
                        uint32_t krow = o / (TN * 2);
                        if (k0 + krow >= Kt) p = ft_zero_page;
                        else if (kRaggedRows && k0 + krow + 1 == Kt && (Nt % 8u) != 0 && (goff_b[i] - krow * ldbt * 2) / 2 + 8 > Nt)
                            p = bbase + (uint32_t)(((Kt - 1u) * ldbt + Nt - 8u) * 2);     // the last row's last 8 (its ragged
                                                                                        // chunk, or the tile's first read in place of one beyond N)
                    } else {
                        uint32_t row = (wave * B_WAVE_BYTES + i * 1024) / 128 + lane / 8;
                        uint32_t kc = (lane & 7u) ^ swzA(row);
                        if (k0 + kc * 8 >= Kt) p = ft_zero_page;
                        else if (kRaggedRows && k0 + kc * 8 + 8 > Kt && Kt >= 8u) p = bbase + (uint32_t)(goff_b[i] - kc * 16 + (Kt - 8u) * 2);
                    }
                }
                if (b_lane_on) lds_dma16(p, st + A_BYTES + wave * B_WAVE_BYTES + i * 1024);
            }
        };
        // this part's (two teams: this team's) index of the operand's last k-tile, where that one takes the
        // checked copy code; none otherwise
        uint32_t tail_kt = 0xffffffffu;
        if (LEAN && k_tail) {
            if constexpr (TEAMS == 1) tail_kt = nk_all - 1u - kt0;
            else if (nk_all - 1u >= kt0 + team && ((nk_all - 1u - kt0 - team) & 1u) == 0) tail_kt = (nk_all - 1u - kt0 - team) >> 1;
        }
        auto is_tail = [&](uint32_t kt) -> bool {
            if constexpr (LEAN) return kt == tail_kt;
            else return k_tail && (TEAMS == 2 ? kt0 + team + 2 * kt : kt0 + kt) + 1 == nk_all;
        };
        auto issue_at = [&](uint32_t kt, uint32_t stage_off) {
#ifdef FT_DEBUG_NO_COPY          // development: only the first copies are issued (the loop then measures MFMA + LDS alone)
            if (kt >= 1) return;
#endif
            if (is_tail(kt)) issue_impl(kt, stage_off, std::true_type{});
            else issue_impl(kt, stage_off, std::false_type{});
        };

        // ---- fragment read addresses -----------------------------------------------------------
        const uint32_t sbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
        // A: row = wave_m*WM + bi*MB + lane%MB ; chunk = ks*(KSTEP/8) + lane/MB, position = chunk ^ swzA(row).
        // The ks term only touches bits the lane term leaves clear, so it is an XOR by a constant.
        const uint32_t fa_row = wave_m * WM + (lane % MB);
        const uint32_t fa_addr0 = sbase + fa_row * (TK * 2) + (((lane / MB) ^ swzA(fa_row)) << 4);
        // B through the transposing read (see gemm_body.h): lane j of a 16-lane group addresses row
        // j/4, columns 4*(j%4)..+3 of a 4 x 16 block and receives column j, rows 0..3.
        const uint32_t j16 = lane & 15u;
        uint32_t fb_colgrp, fb_k8;
        if constexpr (M16) { fb_colgrp = 0; fb_k8 = lane >> 4; }
        else { fb_colgrp = (lane >> 4) & 1u; fb_k8 = lane >> 5; }
        const uint32_t fb_row0 = fb_k8 * 8 + (j16 >> 2);
        uint32_t fb_addr[BN];
#pragma unroll
        for (int bj = 0; bj < BN; ++bj) {
            if constexpr (!BNK) {
                uint32_t col = wave_n * WN + bj * MB + fb_colgrp * 16 + (j16 & 3u) * 4;
                fb_addr[bj] = sbase + A_BYTES + fb_row0 * (TN * 2) + (((col >> 3) ^ swzB<TN>(fb_row0)) << 4) + (col & 7u) * 2;
            } else {
                // as A: row = output column wave_n*WN + bj*MB + lane%MB, chunk = lane/MB (+ the k-step's)
                const uint32_t row = wave_n * WN + bj * MB + (lane % MB);
                fb_addr[bj] = sbase + A_BYTES + row * (TK * 2) + (((lane / MB) ^ swzA(row)) << 4);
            }
        }

        Acc acc[BM][BN];
#pragma unroll
        for (int bi = 0; bi < BM; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj)
#pragma unroll
                for (int e = 0; e < (M16 ? 4 : 16); ++e) acc[bi][bj][e] = 0.f;

        if constexpr (TEAMS == 1) {
        if constexpr (LEAN) {
        // The loop's own bookkeeping is scalar code in front of every k-tile's first MFMA, on a wave that
        // issues in order: counters showed 70 scalar instructions per k-tile (the wait for a runtime
        // number of tiles in flight as a chain of compares, stage indices modulo a runtime ring depth,
        // the checks for the operand's last k-tile), as much issue time as the tile's MFMAs for the small
        // tiles.  So: at most three tiles are kept in flight beyond the one being consumed (deeper rings
        // measured slower again: what arrives is bound elsewhere), which leaves three possible waits;
        // stage offsets advance by add and wrap; the last k-tile is one compare.
        const uint32_t D = S - 1 < (uint32_t)FT_DMAX ? S - 1 : (uint32_t)FT_DMAX;   // tiles in flight beyond the current one
        const uint32_t ring_bytes = (D + 1) * STAGE_BYTES;    // stages in use: D + 1
        // ---- prologue: D tiles on their way -------------------------------------------------------
        FT_MARK(g, 1);
        for (uint32_t s = 0; s < D && s < nk; ++s) issue_at(s, s * STAGE_BYTES);
        FT_MARK(g, 2);
        uint32_t r_off = 0, w_off = D * STAGE_BYTES;          // stage being read; stage the next copy fills

        for (uint32_t kt = 0; kt < nk; ++kt) {
            // copies issued so far: tiles 0 .. min(kt + D - 1, nk - 1); tile kt must have landed
            {
                const uint32_t left = nk - 1 - kt;
                wait_tiles_in<0, FT_DMAX - 1>(left < D - 1 ? left : D - 1);
            }
            __builtin_amdgcn_s_barrier();      // tile kt visible to every wave; the stage of tile kt - 1 is free again
#ifdef FT_TRACE
            if (kt == 0) FT_MARK(g, 3);
            if (kt == nk / 2) FT_MARK(g, 4);
#endif
            if constexpr (kRaggedRows) if (is_tail(kt) && !g.is_conv) {   // uniform; the operand's last k-tile
                uint32_t Kf = K, Nf = N;
                asm volatile("" : "+s"(Kf), "+s"(Nf));        // (as in the copy code: nothing derived from them is hoisted)
                const uint32_t k_frac = Kf % 8u, n_frac = BNK ? 0u : Nf % 8u;
                if (k_frac | n_frac) {
                    fix_edges(smem + r_off, wave_all * 64u + lane, NWT * 64u, (kt0 + kt) * TK, Kf, Nf, n0, k_frac, n_frac);
                    // (a barrier alone does not wait for a wave's own LDS writes on this target)
                    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                }
            }
            if (kt + D < nk) {
                issue_at(kt + D, w_off);
                w_off = w_off + STAGE_BYTES == ring_bytes ? 0u : w_off + STAGE_BYTES;
            }

            const uint32_t a_addr = fa_addr0 + r_off;
            uint32_t b_addr[BN];
#pragma unroll
            for (int bj = 0; bj < BN; ++bj) b_addr[bj] = fb_addr[bj] + r_off;
            r_off = r_off + STAGE_BYTES == ring_bytes ? 0u : r_off + STAGE_BYTES;
            compute_tile(a_addr, b_addr, acc);
        }

        } else {
        // (grouped launches, 256-register tiles: the ring as deep as the plan says, stage indices by division)
        // ---- prologue: fill S-1 stages ------------------------------------------------------------
        FT_MARK(g, 1);
        for (uint32_t s = 0; s + 1 < S && s < nk; ++s) issue_at(s, s * STAGE_BYTES);
        FT_MARK(g, 2);

        for (uint32_t kt = 0; kt < nk; ++kt) {
            // copies issued so far: tiles 0 .. min(kt+S-2, nk-1); tile kt must have landed
            uint32_t newest = kt + S - 2 < nk - 1 ? kt + S - 2 : nk - 1;
            wait_tiles(newest - kt);
            __builtin_amdgcn_s_barrier();      // tile kt visible to every wave; stage (kt-1)%S is free again
#ifdef FT_TRACE
            if (kt == 0) FT_MARK(g, 3);
            if (kt == nk / 2) FT_MARK(g, 4);
#endif
            if constexpr (kRaggedRows) if (is_tail(kt) && !g.is_conv) {   // uniform; the operand's last k-tile
                uint32_t Kf = K, Nf = N;
                asm volatile("" : "+s"(Kf), "+s"(Nf));        // (as in the copy code: nothing derived from them is hoisted)
                const uint32_t k_frac = Kf % 8u, n_frac = BNK ? 0u : Nf % 8u;
                if (k_frac | n_frac) {
                    fix_edges(smem + (kt % S) * STAGE_BYTES, wave_all * 64u + lane, NWT * 64u, (kt0 + kt) * TK, Kf, Nf, n0, k_frac, n_frac);
                    // (a barrier alone does not wait for a wave's own LDS writes on this target)
                    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                }
            }
            if (kt + S - 1 < nk) issue_at(kt + S - 1, ((kt + S - 1) % S) * STAGE_BYTES);

            const uint32_t soff = (kt % S) * STAGE_BYTES;
            const uint32_t a_addr = fa_addr0 + soff;
            uint32_t b_addr[BN];
#pragma unroll
            for (int bj = 0; bj < BN; ++bj) b_addr[bj] = fb_addr[bj] + soff;

            u32x4 fa[2][BM];
            u32x2 fb[2][BN][2];
            read_step<0, 0>(a_addr, b_addr, fa, fb);
            step<0>(a_addr, b_addr, fa, fb, acc);
        }

        }
        // ---- epilogue ------------------------------------------------------------------------------
        FT_MARK(g, 5);
        // (bodies with more than 128 accumulator registers have no room for it: the host never splits them)
        if constexpr (WM * WN / 64 <= FT_KPART_ACC_MAX && NWT == 4) if (g.k_parts > 1) {
            if (!k_part_exchange_blocks<M16>(g, t, part, wave, lane, acc)) return;
        }
        FT_MARK(g, 6);
        store_acc<DT, true, M16, BM, BN>(g, (uint64_t)d.batch * g.strideC, m0 + wave_m * WM, n0 + wave_n * WN, lane, acc);
#ifdef FT_TRACE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        FT_MARK(g, 7);
#endif
        } else {
        // ---- two teams -------------------------------------------------------------------------------
        // Team T works on k-tiles T, T+2, ...: its j-th is copied in "load" phases and consumed in
        // "compute" phases that alternate, team 1 one phase behind team 0:
        //   phase p, team T, q = p - T:  q even -> L(q/2): issue the copies of tile q/2 + S-1 (into the stage
        //   that C(q/2 - 1) read in the phase before), then wait until tile q/2 has landed;
        //   q odd -> C(q/2): fragments + MFMAs of tile q/2.  One s_barrier ends every phase: it publishes
        //   the landed tile to the team and frees the stage just read.  Every wave runs every barrier.
        const uint32_t n_mine = nk > team ? (nk - team + 1) / 2 : 0u;
        const uint32_t n_team0 = (nk + 1) / 2;
        FT_MARK(g, 1);
        for (uint32_t s = 0; s + 1 < S && s < n_mine; ++s) issue_at(s, s * STAGE_BYTES);
        FT_MARK(g, 2);
        // (stage offsets advance by add and wrap: no division by the runtime ring depth per k-tile)
        const uint32_t ring_bytes = S * STAGE_BYTES;
        uint32_t r_off = 0, w_off = (S - 1) * STAGE_BYTES;
        // Written as a straight-line loop per team (the accumulators must not pass through a branch:
        // the compiler would keep two copies of them); team 1 starts one barrier late and the teams
        // run spare barriers at the end so that both execute 2 * n_team0 + 1 of them.
        if (team == 1) __builtin_amdgcn_s_barrier();
        for (uint32_t j = 0; j < n_mine; ++j) {
            if (j + S - 1 < n_mine) {
                issue_at(j + S - 1, w_off);
                w_off = w_off + STAGE_BYTES == ring_bytes ? 0u : w_off + STAGE_BYTES;
            }
            const uint32_t newest = j + S - 1 < n_mine - 1 ? j + S - 1 : n_mine - 1;
            wait_tiles(newest - j);
            __builtin_amdgcn_s_barrier();
#ifdef FT_TRACE
            if (j == 0) FT_MARK(g, 3);
            if (j == n_mine / 2) FT_MARK(g, 4);
#endif
            const uint32_t a_addr = fa_addr0 + r_off;
            uint32_t b_addr[BN];
#pragma unroll
            for (int bj = 0; bj < BN; ++bj) b_addr[bj] = fb_addr[bj] + r_off;
            r_off = r_off + STAGE_BYTES == ring_bytes ? 0u : r_off + STAGE_BYTES;
            compute_tile(a_addr, b_addr, acc);
            __builtin_amdgcn_s_barrier();
        }
        for (uint32_t x = (team == 1 ? 1u : 0u) + 2 * n_mine; x < 2 * n_team0 + 1; ++x) __builtin_amdgcn_s_barrier();
        FT_MARK(g, 5);
        // ---- sum of the two teams' partial tiles through LDS (the rings are idle now) ---------------
        // Wave w of one team and wave w of the other hold the same wave tile.  Each team finishes half of
        // its accumulator blocks (team 1 the upper half of the block rows, or of the block columns when
        // there is one row) and hands the other half over; a wave tile of a single block is finished by
        // team 0 alone.  Layout of a handed-over half: [wave][block][register][lane] floats.
        constexpr int NE = M16 ? 4 : 16;
        constexpr bool SPLIT_M = BM >= 2, SPLIT_N = !SPLIT_M && BN >= 2, SPLIT = SPLIT_M || SPLIT_N;
        constexpr int NB_GIVE = SPLIT ? BM * BN / 2 : BM * BN;       // blocks a wave hands over (team 0: none if !SPLIT)
        constexpr int XW = NB_GIVE * NE * 64;                        // floats per wave
        static_assert(8 * XW * 4 <= 2 * 2 * STAGE_BYTES, "the exchange fits the smallest pair of rings");
        float *const xmine = reinterpret_cast<float *>(smem_all) + (team * 4 + wave) * XW + lane;          // what I give
        const float *const xtheirs = reinterpret_cast<const float *>(smem_all) + ((1 - team) * 4 + wave) * XW + lane;
        auto owned_by_1 = [](int bi, int bj) { return SPLIT_M ? bi >= BM / 2 : (SPLIT_N ? bj >= BN / 2 : false); };
#pragma unroll
        for (int bi = 0; bi < BM; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj) {
                // a block changes hands when its owner is the other team (uniform per wave); the blocks a
                // team receives are numbered in (bi, bj) order
                const bool to1 = owned_by_1(bi, bj);
                if (to1 ? team == 0 : team == 1) {
                    const int slot = idx_of(bi, bj, to1);
#pragma unroll
                    for (int e = 0; e < NE; ++e) xmine[(slot * NE + e) * 64] = acc[bi][bj][e];
                }
            }
        __syncthreads();
#pragma unroll
        for (int bi = 0; bi < BM; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj) {
                const bool mine = owned_by_1(bi, bj) ? team == 1 : team == 0;
                if (mine) {
                    const int slot = idx_of(bi, bj, owned_by_1(bi, bj));
#pragma unroll
                    for (int e = 0; e < NE; ++e) acc[bi][bj][e] += xtheirs[(slot * NE + e) * 64];
                }
            }
        FT_MARK(g, 6);
        const uint64_t coff = (uint64_t)d.batch * g.strideC;
        const uint32_t m0w = m0 + wave_m * WM, n0w = n0 + wave_n * WN;
        if constexpr (SPLIT_M) {
            if (team == 0) store_acc<DT, true, M16, BM, BN, 0, BM / 2, 0, BN>(g, coff, m0w, n0w, lane, acc);
            else store_acc<DT, true, M16, BM, BN, BM / 2, BM, 0, BN>(g, coff, m0w, n0w, lane, acc);
        } else if constexpr (SPLIT_N) {
            if (team == 0) store_acc<DT, true, M16, BM, BN, 0, BM, 0, BN / 2>(g, coff, m0w, n0w, lane, acc);
            else store_acc<DT, true, M16, BM, BN, 0, BM, BN / 2, BN>(g, coff, m0w, n0w, lane, acc);
        } else {
            if (team == 0) store_acc<DT, true, M16, BM, BN>(g, coff, m0w, n0w, lane, acc);
        }
#ifdef FT_TRACE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        FT_MARK(g, 7);
#endif
        }
    }

    // Position of block (bi, bj) among the blocks its receiving team gets, in (bi, bj) order: blocks owned
    // by team 1 (to_team1) count from the first such block, the others likewise.
    static constexpr int idx_of(int bi, int bj, bool to_team1) {
        constexpr bool SM = BM >= 2, SN = !SM && BN >= 2;
        if (SM) return to_team1 ? (bi - BM / 2) * BN + bj : bi * BN + bj;
        if (SN) return to_team1 ? bj - BN / 2 : bj;
        return bi * BN + bj;
    }

    // The chunks of the last k-tile that were fetched as "the row's last 8 elements" (see run): moved
    // down so that the row's element k0 + 8c sits at position 0 of chunk c, zeros behind the row's end.
    // tid of nt: the threads that share the work (a workgroup; one wave for a split-k body's private ring).
    __device__ static __forceinline__ void fix_edges(unsigned char *st, uint32_t tid, uint32_t nt, uint32_t k0, uint32_t K,
                                                     uint32_t N, uint32_t n0, uint32_t k_frac, uint32_t n_frac) {
        const uint32_t NT = nt;
        if (k_frac) {
            const uint32_t c = (K - 1u - k0) / 8u;               // the chunk the reduce axis ends in
            for (uint32_t r = tid; r < (uint32_t)(BNK ? TM + TN : TM); r += NT) {
                // rows of A, then (B stored [N][K]) rows of B: same 128-byte rows, same swizzle
                const uint32_t row = r < (uint32_t)TM ? r : r - TM;
                uint4 *q = reinterpret_cast<uint4 *>(st + (r < (uint32_t)TM ? 0 : A_BYTES) + row * (TK * 2) + ((c ^ swzA(row)) << 4));
                // (rows of at least 8 elements were fetched as their last 8; shorter ones as they lie)
                *q = K >= 8u ? shift_down_elems(*q, 8u - k_frac) : keep_low_elems(*q, k_frac);
            }
        }
        if constexpr (!BNK) {
            // the operand's last row, where it ends inside this tile's columns
            if (n_frac && N > n0 && N - n0 < (uint32_t)TN && tid == 0) {
                const uint32_t krow = K - 1u - k0, nc = (N - 1u - n0) / 8u;
                uint4 *q = reinterpret_cast<uint4 *>(st + A_BYTES + krow * (TN * 2) + ((nc ^ swzB<TN>(krow)) << 4));
                *q = shift_down_elems(*q, 8u - n_frac);
            }
        }
    }

    // LDS reads of the A and B fragments of k-step ks into fragment set buf.  Row offsets of the
    // accumulator blocks and the k-step offset of B go into the instructions' offset fields.
    template <int ks, int buf, int bi = 0>
    __device__ static __forceinline__ void read_a(uint32_t aa, u32x4 (&fa)[2][BM]) {
        fa[buf][bi] = lds_read_b128<bi * MB * TK * 2>(aa);
        if constexpr (bi + 1 < BM) read_a<ks, buf, bi + 1>(aa, fa);
    }
    template <int ks, int buf, int bj = 0>
    __device__ static __forceinline__ void read_b(const uint32_t (&b_addr)[BN], u32x2 (&fb)[2][BN][2]) {
        if constexpr (!BNK) {
            fb[buf][bj][0] = lds_read_tr16_b64<(ks * KSTEP) * TN * 2>(b_addr[bj]);
            fb[buf][bj][1] = lds_read_tr16_b64<(ks * KSTEP + 4) * TN * 2>(b_addr[bj]);
        } else {
            // the lane's 8 consecutive k of its column: two halves of one 16-byte chunk
            const uint32_t bb = b_addr[bj] ^ (uint32_t)(ks * (KSTEP / 8) * 16);
            fb[buf][bj][0] = lds_read_b64<0>(bb);
            fb[buf][bj][1] = lds_read_b64<8>(bb);
        }
        if constexpr (bj + 1 < BN) read_b<ks, buf, bj + 1>(b_addr, fb);
    }
    template <int ks, int buf>
    __device__ static __forceinline__ void read_step(uint32_t a_addr, const uint32_t (&b_addr)[BN],
                                                     u32x4 (&fa)[2][BM], u32x2 (&fb)[2][BN][2]) {
        read_a<ks, buf>(a_addr ^ (uint32_t)(ks * (KSTEP / 8) * 16), fa);
        read_b<ks, buf>(b_addr, fb);
    }

    // k-steps of one tile, software pipelined: the reads of step ks+1 are in flight during the MFMAs of ks
    template <int ks>
    __device__ static __forceinline__ void step(uint32_t a_addr, const uint32_t (&b_addr)[BN], u32x4 (&fa)[2][BM],
                                                u32x2 (&fb)[2][BN][2], Acc (&acc)[BM][BN]) {
        constexpr int buf = ks & 1;
#ifdef FT_DEBUG_NO_MFMA          // development: copies and barriers only
        if constexpr (ks == 0) wait_frag<0>(fa[0], fb[0]);
        return;
#endif
        if constexpr (ks + 1 < KS) {
            read_step<ks + 1, buf ^ 1>(a_addr, b_addr, fa, fb);
            wait_frag<NR>(fa[buf], fb[buf]);
        } else {
            wait_frag<0>(fa[buf], fb[buf]);
        }
#pragma unroll
        for (int bi = 0; bi < BM; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj) {
                uint4 a = __builtin_bit_cast(uint4, fa[buf][bi]);
                uint4 b = make_uint4(fb[buf][bj][0][0], fb[buf][bj][0][1], fb[buf][bj][1][0], fb[buf][bj][1][1]);
                if constexpr (M16) acc[bi][bj] = mfma16<DT>(a, b, acc[bi][bj]);
                else acc[bi][bj] = mfma32<DT>(a, b, acc[bi][bj]);
            }
        if constexpr (ks + 1 < KS) step<ks + 1>(a_addr, b_addr, fa, fb, acc);
    }

    // s_waitcnt lgkmcnt(N) that also "produces" the fragment registers, so no consumer can be
    // scheduled above it
    template <int N>
    __device__ static __forceinline__ void wait_frag(u32x4 (&a)[BM], u32x2 (&b)[BN][2]) {
        if constexpr (BM == 1 && BN == 1)
            asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a[0]), "+v"(b[0][0]), "+v"(b[0][1]) : "n"(N));
        else if constexpr (BM == 1 && BN == 2)
            asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(a[0]), "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]) : "n"(N));
        else if constexpr (BM == 1 && BN == 4)
            asm volatile("s_waitcnt lgkmcnt(%9)" : "+v"(a[0]), "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]),
                         "+v"(b[2][0]), "+v"(b[2][1]), "+v"(b[3][0]), "+v"(b[3][1]) : "n"(N));
        else if constexpr (BM == 2 && BN == 1)
            asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a[0]), "+v"(a[1]), "+v"(b[0][0]), "+v"(b[0][1]) : "n"(N));
        else if constexpr (BM == 2 && BN == 2)
            asm volatile("s_waitcnt lgkmcnt(%6)" : "+v"(a[0]), "+v"(a[1]), "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]) : "n"(N));
        else if constexpr (BM == 2 && BN == 4)
            asm volatile("s_waitcnt lgkmcnt(%10)" : "+v"(a[0]), "+v"(a[1]), "+v"(b[0][0]), "+v"(b[0][1]), "+v"(b[1][0]), "+v"(b[1][1]),
                         "+v"(b[2][0]), "+v"(b[2][1]), "+v"(b[3][0]), "+v"(b[3][1]) : "n"(N));
        else if constexpr (BM == 4 && BN == 2)
            asm volatile("s_waitcnt lgkmcnt(%8)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0][0]), "+v"(b[0][1]),
                         "+v"(b[1][0]), "+v"(b[1][1]) : "n"(N));
        else if constexpr (BM == 4 && BN == 4)
            asm volatile("s_waitcnt lgkmcnt(%12)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0][0]), "+v"(b[0][1]),
                         "+v"(b[1][0]), "+v"(b[1][1]), "+v"(b[2][0]), "+v"(b[2][1]), "+v"(b[3][0]), "+v"(b[3][1]) : "n"(N));
        else
            static_assert(BM == 0, "unsupported fragment shape");
    }

    // Fragments and MFMAs of one k-tile.  Wave tiles of few MFMAs per k-step (two for 64 x 32) cannot hide
    // an LDS round trip behind the step before: with the reads only one step ahead every step waited for
    // its fragments (measured: 740 clocks per k-tile for 256 clocks of MFMAs).  Where four k-steps' worth
    // of reads fit the counter of outstanding LDS operations two at a time, every step has a fragment set
    // of its own and the reads run two steps ahead: one exposed round trip per k-tile instead of four.
    static constexpr bool LOOKAHEAD2 = kLeanLoop && KS == 4 && 2 * NR <= 15;
    template <int ks>
    __device__ static __forceinline__ void read_set(uint32_t a_addr, const uint32_t (&b_addr)[BN], u32x4 (&a)[BM], u32x2 (&b)[BN][2]) {
        const uint32_t aa = a_addr ^ (uint32_t)(ks * (KSTEP / 8) * 16);
        read_set_a<0>(aa, a);
#pragma unroll
        for (int bj = 0; bj < BN; ++bj) {
            if constexpr (!BNK) {
                b[bj][0] = lds_read_tr16_b64<(ks * KSTEP) * TN * 2>(b_addr[bj]);
                b[bj][1] = lds_read_tr16_b64<(ks * KSTEP + 4) * TN * 2>(b_addr[bj]);
            } else {
                const uint32_t bb = b_addr[bj] ^ (uint32_t)(ks * (KSTEP / 8) * 16);
                b[bj][0] = lds_read_b64<0>(bb);
                b[bj][1] = lds_read_b64<8>(bb);
            }
        }
    }
    template <int bi>
    __device__ static __forceinline__ void read_set_a(uint32_t aa, u32x4 (&a)[BM]) {
        a[bi] = lds_read_b128<bi * MB * TK * 2>(aa);
        if constexpr (bi + 1 < BM) read_set_a<bi + 1>(aa, a);
    }
    __device__ static __forceinline__ void mfma_set(const u32x4 (&fa)[BM], const u32x2 (&fb)[BN][2], Acc (&acc)[BM][BN]) {
#pragma unroll
        for (int bi = 0; bi < BM; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj) {
                uint4 a = __builtin_bit_cast(uint4, fa[bi]);
                uint4 b = make_uint4(fb[bj][0][0], fb[bj][0][1], fb[bj][1][0], fb[bj][1][1]);
                if constexpr (M16) acc[bi][bj] = mfma16<DT>(a, b, acc[bi][bj]);
                else acc[bi][bj] = mfma32<DT>(a, b, acc[bi][bj]);
            }
    }
    __device__ static __forceinline__ void compute_tile(uint32_t a_addr, const uint32_t (&b_addr)[BN], Acc (&acc)[BM][BN]) {
        if constexpr (LOOKAHEAD2) {
#ifdef FT_DEBUG_NO_MFMA
            u32x4 a0[BM]; u32x2 b0[BN][2];
            read_set<0>(a_addr, b_addr, a0, b0);
            wait_frag<0>(a0, b0);
#else
            u32x4 a0[BM], a1[BM], a2[BM], a3[BM];
            u32x2 b0[BN][2], b1[BN][2], b2[BN][2], b3[BN][2];
            // (at most two sets' reads are outstanding at any time: the counter has four bits)
            read_set<0>(a_addr, b_addr, a0, b0);
            read_set<1>(a_addr, b_addr, a1, b1);
            wait_frag<NR>(a0, b0);
            read_set<2>(a_addr, b_addr, a2, b2);
            mfma_set(a0, b0, acc);
            wait_frag<NR>(a1, b1);
            read_set<3>(a_addr, b_addr, a3, b3);
            mfma_set(a1, b1, acc);
            wait_frag<NR>(a2, b2);
            mfma_set(a2, b2, acc);
            wait_frag<0>(a3, b3);
            mfma_set(a3, b3, acc);
#endif
        } else {
            u32x4 fa[2][BM];
            u32x2 fb[2][BN][2];
            read_step<0, 0>(a_addr, b_addr, fa, fb);
            step<0>(a_addr, b_addr, fa, fb, acc);
        }
    }
};


// ---------------------------------------------------------------------------------------------
// Split-k wave grid (1 x 1 x 4): every wave owns the whole TM x TN output tile and a quarter of the
// reduce axis (k-tiles w, w+4, w+8, ...), with a private LDS ring filled by its own LDS-DMA copies.
// No workgroup barrier in the main loop; the four partial tiles are summed through LDS at the end.
// For shapes with few tiles and a long reduce axis the barrier-per-k-tile loop above is bound by
// its own latency chain; here each SIMD runs an independent, deeply prefetched stream.
// ---------------------------------------------------------------------------------------------
template <int DT, int TM, int TN>
struct UKernelSplitK {
    static constexpr int TK = 64;
    static constexpr bool M16 = (TM == 16);
    static constexpr int MB = M16 ? 16 : 32;
    static constexpr int KSTEP = M16 ? 32 : 16;
    static constexpr int KS = TK / KSTEP;
    static constexpr int BM = TM / MB, BN = TN / MB;
    static constexpr int A_BYTES = TM * TK * 2, B_BYTES = TK * TN * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LA = A_BYTES / 1024, LB = B_BYTES / 1024;
    static constexpr int L = LA + LB;
    static constexpr int MAX_AHEAD = (63 / L) < 6 ? (63 / L) : 6;
    static constexpr int NR = BM + 2 * BN;
    static constexpr int NREG = TM * TN / 64;          // accumulator registers per lane
    static_assert(NR <= 15 && LA >= 1 && LB >= 1 && NREG % 4 == 0, "unsupported split-k tile");
    using Acc = typename std::conditional<M16, f32x4, f32x16>::type;
    using Std = UKernelFast<DT, TM, TN, 1, 1>;         // fragment helpers only (same layouts)

    // (as in UKernelFast: a decision tree over the immediate wait counts)
    template <int LO, int HI> __device__ static __forceinline__ void wait_tiles_in(uint32_t ahead) {
        if constexpr (LO == HI) wait_vmcnt<LO * L>();
        else {
            constexpr int MID = (LO + HI) / 2;
            if (ahead <= (uint32_t)MID) wait_tiles_in<LO, MID>(ahead);
            else wait_tiles_in<MID + 1, HI>(ahead);
        }
    }
    template <int T> __device__ static __forceinline__ void wait_tiles_chain(int ahead) {
        if constexpr (T >= MAX_AHEAD) wait_vmcnt<MAX_AHEAD * L>();
        else {
            if (ahead <= T) wait_vmcnt<T * L>();
            else wait_tiles_chain<T + 1>(ahead);
        }
    }
    __device__ static __forceinline__ void wait_tiles(uint32_t ahead) {
        if constexpr (kLeanLoop) wait_tiles_in<0, MAX_AHEAD>(ahead > (uint32_t)MAX_AHEAD ? (uint32_t)MAX_AHEAD : ahead);
        else wait_tiles_chain<0>((int)ahead);
    }

    __device__ static __forceinline__ void run(const KArgs &g, const TileDesc &d, unsigned char *smem,
                                               uint32_t stages_in, uint32_t t, uint32_t part) {
        const uint32_t tid = threadIdx.x;
        const uint32_t lane = tid & 63u;
        const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const uint32_t m0 = d.m0, n0 = d.n0;
        const uint32_t M = g.M, N = g.N, K = g.K;
        const uint16_t *__restrict__ Ab = g.A + (uint64_t)d.batch * g.strideA;
        const uint16_t *__restrict__ Bb = g.B + (uint64_t)d.batch * g.strideB;
        // this workgroup's k-tiles: kt0 .. kt0 + nk - 1 of the nk_all of the reduce axis
        const uint32_t nk_all = (K + TK - 1) / TK;
        const uint32_t kt0 = part * g.k_part_tiles;
        const uint32_t nk = g.k_parts > 1 ? (nk_all - kt0 < g.k_part_tiles ? nk_all - kt0 : g.k_part_tiles) : nk_all;
        const uint32_t nkw = nk > wave ? (nk - wave + 3) / 4 : 0;     // k-tiles of this wave
        uint32_t S = stages_in < 2 ? 2u : stages_in;
        if (S > (uint32_t)MAX_AHEAD + 2) S = MAX_AHEAD + 2;
        unsigned char *ring = smem + wave * S * STAGE_BYTES;          // this wave's private ring

        uint32_t goff_a[LA], goff_b[LB];
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            uint32_t row = i * 8 + lane / 8;
            uint32_t kc = (lane & 7u) ^ swzA(row);
            uint32_t gm = m0 + row;
            if (gm >= M) gm = M - 1;
            goff_a[i] = (gm * g.lda + kc * 8) * 2;          // bytes from the operand base
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            uint32_t o = i * 1024 + lane * 16;
            uint32_t krow = o / (TN * 2), p = (o % (TN * 2)) / 16;
            uint32_t nc = p ^ swzB<TN>(krow);
            uint32_t col = n0 + nc * 8;
            if (col >= N) col = n0;
            goff_b[i] = (krow * g.ldb + col) * 2;
        }
        // ragged rows (K or N not a multiple of 8) as in UKernelFast: the chunk a row ends in is fetched
        // as the 8 elements that end with the row and moved down in LDS by the wave that owns the k-tile.
        // Only the two narrowest tiles carry that code: the others have a four-wave standard grid of the
        // same tile, which the host sends ragged launches to.
        constexpr bool RAGGED = kRaggedRows && TM * TN <= 16 * 32;
        const bool k_tail = (K % TK) != 0 || (RAGGED && (N % 8u) != 0);

        auto issue_impl = [&](uint32_t j, uint32_t stage_off, auto tail_c) {
            constexpr bool tail = decltype(tail_c)::value;
            unsigned char *st = ring + stage_off;
            const uint32_t k0 = (kt0 + wave + 4 * j) * TK;
            // byte offsets inside one batch entry fit 32 bits (the host rejects larger operands)
            const char *abase = reinterpret_cast<const char *>(Ab), *bbase = reinterpret_cast<const char *>(Bb);
            const uint32_t ka = k0 * 2, kb = k0 * g.ldb * 2;                                        // uniform
            uint32_t Kt = K, Nt = N, ldbt = g.ldb;
            if constexpr (tail && RAGGED) asm volatile("" : "+s"(Kt), "+s"(Nt), "+s"(ldbt));   // (see UKernelFast)
#pragma unroll
            for (int i = 0; i < LA; ++i) {
                const void *p = abase + (uint32_t)(goff_a[i] + ka);
                if constexpr (tail) {
                    uint32_t row = i * 8 + lane / 8;
                    uint32_t kc = (lane & 7u) ^ swzA(row);
                    if (k0 + kc * 8 >= Kt) p = ft_zero_page;
                    else if (RAGGED && k0 + kc * 8 + 8 > Kt && Kt >= 8u) p = abase + (uint32_t)(goff_a[i] - kc * 16 + (Kt - 8u) * 2);
                }
                lds_dma16(p, st + i * 1024);
            }
#pragma unroll
            for (int i = 0; i < LB; ++i) {
                const void *p = bbase + (uint32_t)(goff_b[i] + kb);
                if constexpr (tail) {
                    uint32_t krow = (i * 1024 + lane * 16) / (TN * 2);
                    if (k0 + krow >= Kt) p = ft_zero_page;
                    else if (RAGGED && k0 + krow + 1 == Kt && (Nt % 8u) != 0 && (goff_b[i] - krow * ldbt * 2) / 2 + 8 > Nt)
                        p = bbase + (uint32_t)(((Kt - 1u) * ldbt + Nt - 8u) * 2);
                }
                lds_dma16(p, st + A_BYTES + i * 1024);
            }
        };
        // this wave's index of the operand's last k-tile where that one takes the checked copy code; none otherwise
        uint32_t tail_j = 0xffffffffu;
        if (kLeanLoop && k_tail && nk_all - 1u >= kt0 + wave && ((nk_all - 1u - kt0 - wave) & 3u) == 0) tail_j = (nk_all - 1u - kt0 - wave) >> 2;
        auto is_tail = [&](uint32_t j) -> bool {
            if constexpr (kLeanLoop) return j == tail_j;
            else return k_tail && kt0 + wave + 4 * j + 1 == nk_all;
        };
        auto issue_at = [&](uint32_t j, uint32_t stage_off) {
            if (is_tail(j)) issue_impl(j, stage_off, std::true_type{});
            else issue_impl(j, stage_off, std::false_type{});
        };

        const uint32_t sbase = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem +
                               wave * S * STAGE_BYTES;
        const uint32_t fa_row = lane % MB;
        const uint32_t fa_addr0 = sbase + fa_row * (TK * 2) + (((lane / MB) ^ swzA(fa_row)) << 4);
        const uint32_t j16 = lane & 15u;
        uint32_t fb_colgrp, fb_k8;
        if constexpr (M16) { fb_colgrp = 0; fb_k8 = lane >> 4; }
        else { fb_colgrp = (lane >> 4) & 1u; fb_k8 = lane >> 5; }
        const uint32_t fb_row0 = fb_k8 * 8 + (j16 >> 2);
        uint32_t fb_addr[BN];
#pragma unroll
        for (int bj = 0; bj < BN; ++bj) {
            uint32_t col = bj * MB + fb_colgrp * 16 + (j16 & 3u) * 4;
            fb_addr[bj] = sbase + A_BYTES + fb_row0 * (TN * 2) + (((col >> 3) ^ swzB<TN>(fb_row0)) << 4) + (col & 7u) * 2;
        }

        Acc acc[BM][BN];
#pragma unroll
        for (int bi = 0; bi < BM; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj)
#pragma unroll
                for (int e = 0; e < (M16 ? 4 : 16); ++e) acc[bi][bj][e] = 0.f;

        FT_MARK(g, 1);
        for (uint32_t s = 0; s + 1 < S && s < nkw; ++s) issue_at(s, s * STAGE_BYTES);
        FT_MARK(g, 2);
        // (stage offsets advance by add and wrap: no division by the runtime ring depth per k-tile)
        const uint32_t ring_bytes = S * STAGE_BYTES;
        uint32_t r_off = 0, w_off = (S - 1) * STAGE_BYTES;
        for (uint32_t j = 0; j < nkw; ++j) {
            uint32_t newest = j + S - 2 < nkw - 1 ? j + S - 2 : nkw - 1;
            wait_tiles(newest - j);
#ifdef FT_TRACE
            if (j == 0) FT_MARK(g, 3);
            if (j == nkw / 2) FT_MARK(g, 4);
#endif
            if constexpr (RAGGED) if (is_tail(j)) {   // this wave holds the operand's last k-tile
                uint32_t Kf = K, Nf = N;
                asm volatile("" : "+s"(Kf), "+s"(Nf));
                const uint32_t k_frac = Kf % 8u, n_frac = Nf % 8u;
                if (k_frac | n_frac) {
                    // the wave's own ring: its 64 lanes do what a workgroup does in UKernelFast; the reads below
                    // are the same wave's, in order behind these writes
                    Std::fix_edges(ring + r_off, lane, 64u, (kt0 + wave + 4 * j) * TK, Kf, Nf, n0, k_frac, n_frac);
                    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
                }
            }
            // stage (j-1)%S was fully read by this wave (its last k-step waited lgkmcnt(0))
            if (j + S - 1 < nkw) {
                if constexpr (kLeanLoop) {
                    issue_at(j + S - 1, w_off);
                    w_off = w_off + STAGE_BYTES == ring_bytes ? 0u : w_off + STAGE_BYTES;
                } else issue_at(j + S - 1, ((j + S - 1) % S) * STAGE_BYTES);
            }
            const uint32_t a_addr = fa_addr0 + r_off;
            uint32_t b_addr[BN];
#pragma unroll
            for (int bj = 0; bj < BN; ++bj) b_addr[bj] = fb_addr[bj] + r_off;
            if constexpr (kLeanLoop) r_off = r_off + STAGE_BYTES == ring_bytes ? 0u : r_off + STAGE_BYTES;
            else r_off = ((j + 1) % S) * STAGE_BYTES;
            Std::compute_tile(a_addr, b_addr, acc);
        }

        FT_MARK(g, 5);
        // ---- sum the four partial tiles: partials go to the wave's own (now idle) ring as
        // [register][lane] floats, then wave w adds up and stores registers w*NREG/4 .. +NREG/4
        constexpr int PER = NREG / 4;
        constexpr int RPB = M16 ? 4 : 16;               // registers per accumulator block
        float fin[PER];
        if constexpr (PER % 4 == 0) {
            // four registers per LDS access (register r of the tile at float4 (r / 4) * 64 + lane, component r % 4):
            // a quarter of the LDS instructions of the scalar form below, same sums in the same order
            float4 *own4 = reinterpret_cast<float4 *>(ring);
#pragma unroll
            for (int bi = 0; bi < BM; ++bi)
#pragma unroll
                for (int bj = 0; bj < BN; ++bj)
#pragma unroll
                    for (int e = 0; e < RPB; e += 4)
                        own4[(((bi * BN + bj) * RPB + e) / 4) * 64 + lane] =
                            make_float4(acc[bi][bj][e], acc[bi][bj][e + 1], acc[bi][bj][e + 2], acc[bi][bj][e + 3]);
            __syncthreads();
#pragma unroll
            for (int q = 0; q < PER; q += 4) {
                float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float4 x = reinterpret_cast<const float4 *>(smem + w * S * STAGE_BYTES)[(wave * (PER / 4) + q / 4) * 64 + lane];
                    sum.x += x.x; sum.y += x.y; sum.z += x.z; sum.w += x.w;
                }
                fin[q] = sum.x; fin[q + 1] = sum.y; fin[q + 2] = sum.z; fin[q + 3] = sum.w;
            }
        } else {
        float *own = reinterpret_cast<float *>(ring);
#pragma unroll
        for (int bi = 0; bi < BM; ++bi)
#pragma unroll
            for (int bj = 0; bj < BN; ++bj)
#pragma unroll
                for (int e = 0; e < RPB; ++e)
                    own[((bi * BN + bj) * RPB + e) * 64 + lane] = acc[bi][bj][e];
        __syncthreads();
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                sum += reinterpret_cast<const float *>(smem + w * S * STAGE_BYTES)[(wave * PER + q) * 64 + lane];
            fin[q] = sum;
        }
        }
        if (g.k_parts > 1 && !k_part_exchange<PER>(g, t, part, wave, lane, [&](int r) -> float { return fin[r]; },
                                                  [&](int r, float x) { fin[r] = x; })) return;
        FT_MARK(g, 6);
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const uint32_t r = wave * PER + q;          // uniform: register r of the tile's accumulator layout
            const uint32_t e = r % RPB, bj = (r / RPB) % BN, bi = r / (RPB * BN);
            float sum = fin[q];
            uint32_t col = n0 + bj * MB + (lane % MB);
            uint32_t row = m0 + bi * MB + (M16 ? 4 * (lane / 16) + e : 8 * (e / 4) + 4 * (lane / 32) + (e % 4));
            if (row < M && col < N) {
                if (g.bias != nullptr) sum += g.bias[col];
                const uint64_t o = (uint64_t)d.batch * g.strideC + (uint64_t)row * g.ldc + col;
                if (g.out_kind == OUT_F32) __builtin_nontemporal_store(sum, static_cast<float *>(g.C) + o);
                else __builtin_nontemporal_store(out_cvt<DT == 0 ? OUT_F16 : OUT_BF16>(sum), static_cast<uint16_t *>(g.C) + o);
            }
        }
#ifdef FT_TRACE
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        FT_MARK(g, 7);
#endif
    }
};

}  // namespace ftk
