/*
 * ftuner.h -- C ABI of the MI355X (gfx950) dynamic-shape contraction library.
 *
 * The library runs dense contractions whose shape is known only at run time -- Matmul,
 * batched Matmul and NHWC Conv2d as implicit GEMM -- as a patchwork of differently sized
 * uKernel tiles (Sec. 3; Fig. 4(c)): each workgroup computes one tile of the output with
 * fp16/bf16 MFMA and fp32 accumulation, and the tiles of one or two uKernel shapes cover
 * the output exactly once with no padding on the main axis beyond the 16-row MFMA granule.
 *
 * The four stages follow the paper's problem statement:
 *   (a) ft_op_register      operator template + every possible shape        (Sec. 3, Sec. 4)
 *   (b) ft_ukernels_derive  uKernel set from the hardware model             (Sec. 4, Alg. 1)
 *   (c) ft_plan             uKernel-based program for one runtime shape     (Sec. 5, Alg. 2, Eq. 1)
 *   (d) ft_launch           one launch over the tile-descriptor table       (Sec. 3: uKernel = thread block)
 *
 * Conventions
 *   - Plain C, no exceptions cross the boundary; every call returns ft_status (0 = FT_OK).
 *   - Every struct starts with struct_size, which the caller sets to sizeof(the struct).
 *   - "host pointer" / "device pointer" is stated per argument.  The caller owns A, B, C and
 *     the HIP stream; the library owns its handles and the descriptor tables.
 *   - Everything except ft_hw_query, ft_launch and the device half of ft_plan works in a
 *     process without a GPU.
 *   - Handles are not thread-safe against concurrent mutation; distinct handles may be used
 *     from distinct threads.
 */
#ifndef FTUNER_H
#define FTUNER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t ft_status;
enum {
    FT_OK = 0,
    FT_ERR_INVALID_ARG = -1,   /* null pointer, wrong struct_size, inconsistent fields      */
    FT_ERR_UNSUPPORTED = -2,   /* valid request the library has no kernel for               */
    FT_ERR_OUT_OF_RANGE = -3,  /* runtime extent outside the registered dynamic range       */
    FT_ERR_NO_COVER = -4,      /* uKernel set empty / no program covers the shape           */
    FT_ERR_HIP = -5,           /* a HIP runtime call failed (see ft_last_hip_error)         */
    FT_ERR_OOM = -6            /* host or device allocation failed                          */
};

/* Static string for a status code (never NULL). */
const char *ft_status_string(ft_status s);
/* hipError_t value of the last failing HIP call made by this library on this thread. */
int32_t ft_last_hip_error(void);

/* ---------------------------------------------------------------------------------------
 * Hardware description (Sec. 8: bandwidth per memory level, core clock, core count), in
 * gfx950 terms.  All fields are integers so that every derived metric is an exact rational.
 * ------------------------------------------------------------------------------------- */
typedef struct ft_hw_model {
    uint32_t struct_size;
    uint32_t num_cus;                        /* NumCores: compute units (256)                */
    uint32_t simds_per_cu;                   /* 4                                            */
    uint32_t wave_size;                      /* 64                                           */
    uint32_t regs_per_lane;                  /* unified VGPR+AGPR per lane per SIMD (512)    */
    uint32_t max_waves_per_simd;             /* 8                                            */
    uint32_t lds_bytes_per_cu;               /* 163840                                       */
    uint32_t clock_mhz;                      /* 2400                                         */
    uint32_t mfma_flops_per_clk_per_cu;      /* FLOPS of Eq. 6 for dense 16-bit MFMA (4096)  */
    uint32_t bw_global_bytes_per_clk_per_cu; /* bw_G of Eq. 7: L2 -> CU path (64)            */
    uint32_t bw_lds_bytes_per_clk_per_cu;    /* bw_S of Eq. 7 (256, measured 227..256)       */
    uint32_t ktile_latency_clk;              /* latency of one k-tile step of the k loop (400)*/
    uint32_t solo_copy_exposed_pct;          /* share of the global->LDS copy time a workgroup
                                                alone on its CU cannot hide behind MFMA (50)  */
    uint32_t hbm_gbytes_per_s;               /* 8000; used for rooflines only                */
    uint32_t num_xcds;                       /* 8                                            */
    uint32_t part_exchange_clk;              /* reduce-axis split: latency of handing a partial
                                                tile to the workgroup that sums them (2000)   */
    uint32_t part_exchange_bytes_per_clk;    /* rate at which that workgroup reads the k_parts
                                                fp32 partial tiles (16); 0: not counted       */
    uint32_t phase_latency_clk;              /* two-team bodies: cost of the barrier that ends each
                                                k-tile phase (150)                            */
} ft_hw_model;

/* gfx950 defaults; host only. out: host pointer. */
ft_status ft_hw_default_gfx950(ft_hw_model *out);
/* Defaults overridden by what hipGetDeviceProperties reports for hip_device (CU count,
 * clock, LDS size, wave size).  Needs a GPU. out: host pointer. */
ft_status ft_hw_query(int32_t hip_device, ft_hw_model *out);

/* ---------------------------------------------------------------------------------------
 * Hyper-parameters (Sec. 4.2: epsilon/lambda sweep and zeta; Sec. 4.3: psi; Sec. 5.2: SIA
 * coefficients).  Fractions are per-mille or num/den pairs.
 * ------------------------------------------------------------------------------------- */
typedef struct ft_tuning {
    uint32_t struct_size;
    uint32_t eps_min_pm, eps_max_pm, eps_step_pm;   /* 500, 950, 10                         */
    uint32_t lam_max_pm, lam_min_pm, lam_step_pm;   /* 950, 900, 1                          */
    uint32_t zeta;                                  /* default active workgroups per CU: 2  */
    uint32_t rest_regs;                             /* RestRegs of Eq. 4: 72                */
    uint32_t psi_num, psi_den;                      /* threshold of Eq. 6: 1/64             */
    uint32_t c0, c1, c2;                            /* Eq. 1 coefficients: 1, 1, 1          */
    uint32_t sia_form;                              /* FT_SIA_LINEAR: c0*CMR + c1*Pad + c2*Occ of
                                                       the program, as printed; FT_SIA_PRODUCT
                                                       (default): mean over the program's uKernels
                                                       of CMR^c0 * Pad^c1 * Occ^c2, each on its own
                                                       sub-workload (c0..c2 <= 4)               */
    /* Occupancy rescue for shapes whose tiles do not fill the device (the weakness Sec. 6.2
     * reports for short sequences): Matmul programs are also scored with the reduce axis of
     * every tile split over 2, 3, 4, 6 or 8 workgroups (Occ and block.bound count workgroups,
     * compute_eff is taken on one part), as long as all workgroups are resident at once.      */
    uint32_t k_parts_max;                           /* most parts per tile; 1 = never split: 8    */
    uint32_t k_part_min_tiles;                      /* fewest k-tiles (of tk) a part may get: 8   */
    /* Operators with two dynamic space axes (Fig. 4(d)): programs are also scored with a second,
     * narrower uKernel covering what the part's own tiles leave of the other axis (up to four
     * uKernel shapes per launch).                                                                */
    uint32_t second_axis_strips;                    /* 0: off (default: measured slower on gfx950,
                                                       where the fp32 score matrix is bound by its
                                                       own write), 1: on                           */
    /* Two-team bodies (Sec. 3: a uKernel is one thread block; Fig. 7: its thread-level tiling): the
     * standard wave grids again with EIGHT waves, two teams of four that take alternate k-tiles of
     * the same tile, so that one team's copies overlap the other's MFMAs (gk = 2 in
     * ft_ukernel_info).  Matmul and Conv2d.  The same switch derives the eight-wave GRIDS (gm*gn = 8,
     * gk = 1: tiles of 256x256, 128x256 and 256x128 whose eight waves share every k-tile), Matmul only.
     * Against block.bound an eight-wave grid counts twice: one workgroup puts two waves on each SIMD. */
    uint32_t two_team_bodies;                       /* 1: derive them (default), 0: four-wave bodies only */
} ft_tuning;
enum { FT_SIA_LINEAR = 0, FT_SIA_PRODUCT = 1 };

ft_status ft_tuning_default(ft_tuning *out);        /* out: host pointer */

/* ---------------------------------------------------------------------------------------
 * (a) Operator template.
 * ------------------------------------------------------------------------------------- */
enum { FT_OP_MATMUL = 0, FT_OP_BMM = 1, FT_OP_CONV2D = 2 };
enum { FT_F16 = 0, FT_BF16 = 1 };
/* Output element type: fp32 (the default), or the accumulator rounded once, to nearest even, to
 * the 16-bit type of the inputs.  Epilogue: none, or C[.., j] += bias[j] before that rounding
 * (the fused Dense + bias-add of the paper's BERT evaluation, Sec. 6.2). */
enum { FT_OUT_F32 = 0, FT_OUT_SAME = 1 };
enum { FT_EPI_NONE = 0, FT_EPI_BIAS = 1 };
/* Layout of operand B (Matmul and BMM; the GEMM view itself, Sec. 4.1 / Fig. 12 caption, does not
 * change): FT_B_KN, B[b,k,j] with j contiguous (row pitch N); FT_B_NK, the same matrix stored
 * transposed, B[b,j,k] with k contiguous (row pitch K): the K matrix of an attention's Q K^T, a
 * linear layer's weight as frameworks keep it.  With FT_B_NK the operator derives the four-wave
 * standard grids only, and a launch needs operands the LDS-DMA bodies accept: a reduce extent of
 * at least 8 (any alignment, any N); otherwise ft_launch returns FT_ERR_UNSUPPORTED (the general
 * bodies have no such variant).                                                                  */
enum { FT_B_KN = 0, FT_B_NK = 1 };

typedef struct ft_op_desc {
    uint32_t struct_size;
    uint32_t kind;                 /* FT_OP_*                                                */
    uint32_t dtype;                /* FT_F16 / FT_BF16 inputs; accumulation is fp32          */
    /* GEMM view C[b,i,j] = sum_k A[b,i,k] B[b,k,j].  An extent > 0 is static; 0 means dynamic
     * with the inclusive range [lo, hi] below (lo may be 0: empty inputs are legal).  Matmul
     * and BMM use these directly (Matmul has batch 1; the BMM batch count is always a runtime
     * value).  For Conv2d they are ignored except m_lo/m_hi, the range of n*P*Q.            */
    uint32_t m, n, k;
    uint32_t m_lo, m_hi, n_lo, n_hi, k_lo, k_hi;
    /* Conv2d (NHWC input, RSCK weights, NHWC fp32 output): space axes (n,p,q,k), reduce axes
     * (r,s,c) (Fig. 7 caption).  GEMM view: M = n*P*Q, N = c_out, K = r*s*c_in.            */
    uint32_t c_in, c_out, r, s, stride, pad;
    uint32_t out_dtype;            /* FT_OUT_*: element type of C                            */
    uint32_t epilogue;             /* FT_EPI_*                                               */
    uint32_t batch_hi;             /* BMM: largest batch count of the workload (the batch of a
                                      launch is a runtime value); 0 = unknown: the workload
                                      filters (CrossPick, Eq. 5) are skipped for this operator */
    uint32_t b_layout;             /* FT_B_*: Matmul and BMM; Conv2d takes FT_B_KN (RSCK weights) */
} ft_op_desc;

typedef struct ft_op ft_op;
/* desc: host pointer, copied.  *out: new handle, released with ft_op_destroy. */
ft_status ft_op_register(const ft_op_desc *desc, ft_op **out);
void ft_op_destroy(ft_op *op);

/* ---------------------------------------------------------------------------------------
 * (b) uKernel set: HardwareAlign, then IsOverflow, Eq. 4 (one workgroup per CU), Eq. 6, and
 * CrossPick + Eq. 5 (Alg. 1, Sec. 4.3) evaluated over the workload = every shape of the
 * registered dynamic ranges (sampled at the range ends and at multiples of 16); canonical
 * order = larger smem_tile area first.  If nothing survives the workload filters they are
 * skipped.  SetBound (block.bound of the shape at hand) is applied by ft_plan_create.
 * ------------------------------------------------------------------------------------- */
typedef struct ft_ukernel_info {
    uint32_t struct_size;
    uint32_t id;                   /* index in the set                                       */
    uint32_t tm, tn, tk;           /* smem_tile: workgroup tile staged in LDS                */
    uint32_t wm, wn;               /* reg_tile: per-wave fp32 accumulator tile               */
    uint32_t gm, gn, gk;           /* wave grid over rows, columns, reduce axis: gm*gn*gk = 4 waves, or
                                      gk = 2 with gm*gn = 4: two teams of four waves (eight in all), or
                                      gm*gn = 8 with gk = 1: eight waves on the same k-tiles          */
    uint32_t mfma;                 /* 0: 32x32x16, 1: 16x16x32                               */
    uint32_t stages;               /* LDS ring depth: k-tiles resident at once (2..8), per wave for
                                      gk = 4 and per team for gk = 2                          */
    uint32_t lds_bytes;            /* gk*stages*(tm+tn)*tk*2                                 */
    uint32_t acc_regs;             /* wm*wn/64 per lane                                      */
    uint32_t regs;                 /* acc_regs + RestRegs                                    */
    uint32_t max_wg_per_cu;        /* resident workgroups per CU allowed by LDS and registers*/
    uint32_t reg_budget;           /* registers per lane granted to the body: 128, 256 or 512*/
    uint64_t cmr_q20;              /* compute_eff (Eq. 6) alone on its CU, floor(x * 2^20)   */
    uint64_t cmr_shared_q20;       /* compute_eff when two or more workgroups share the CU   */
} ft_ukernel_info;

typedef struct ft_ukset ft_ukset;
/* hw, tuning: host pointers or NULL for the defaults; copied.  The set keeps a reference to
 * nothing in op after the call except the copied descriptor. */
ft_status ft_ukernels_derive(const ft_op *op, const ft_hw_model *hw, const ft_tuning *tuning,
                             ft_ukset **out);
ft_status ft_ukset_size(const ft_ukset *set, uint32_t *n);
ft_status ft_ukset_get(const ft_ukset *set, uint32_t i, ft_ukernel_info *out);
void ft_ukset_destroy(ft_ukset *set);

/* ---------------------------------------------------------------------------------------
 * (c) Plan.
 * ------------------------------------------------------------------------------------- */
typedef struct ft_shape {
    uint32_t struct_size;
    uint32_t batch;                /* BMM batch count; ignored for Matmul / Conv2d           */
    uint32_t m, n, k;              /* dynamic GEMM extents (static ones: 0 or the same value);
                                      every operand of one batch entry must stay below 2^31
                                      elements and N below 2^20, else FT_ERR_UNSUPPORTED      */
    uint32_t img_n, img_h, img_w;  /* Conv2d input: images, height, width                    */
} ft_shape;

enum {
    FT_PLAN_PATCHWORK = 0u,        /* Alg. 2 pool + SIA Top-1                                */
    FT_PLAN_PAD_BASELINE = 1u,     /* pad every dynamic axis to the largest uKernel (Fig. 2) */
    FT_PLAN_FORCED = 2u,           /* take the program given in ft_forced_program            */
    FT_PLAN_MODE_MASK = 3u,
    FT_PLAN_HOST_ONLY = 16u,       /* no device table; the plan cannot be launched           */
    FT_PLAN_TABLE_ORDER = 32u      /* workgroups read their descriptors from the table even where
                                      the closed form of the tile grids would do (ft_plan_stats.
                                      table_order); same results, for debugging and comparison  */
};

/* Program to build when the mode is FT_PLAN_FORCED (used to measure every program of the
 * pool against its SIA score, Sec. 6.3): count1 tiles of uKernel k1 along the main axis,
 * then count2 of k2 (count2 = 0: single uKernel).  The counts must cover the granule-rounded
 * main-axis extent exactly. */
typedef struct ft_forced_program {
    uint32_t struct_size;
    uint32_t k1, count1, k2, count2;
    uint32_t k_parts;              /* workgroups per tile along the reduce axis (0 or 1: none); cut
                                      down to the k-tiles there are; ignored (1) when a constituent
                                      has more than 128 accumulator registers per lane          */
} ft_forced_program;

/* Tile descriptor: one workgroup's work.  24 bytes, little endian, compared byte for byte
 * with the planner oracle.  Order in the table: ukernel_id, batch, m0, n0 ascending. */
typedef struct ft_tile_desc {
    uint32_t ukernel_id;           /* index into the uKernel set                             */
    uint32_t batch;
    uint32_t m0, n0;               /* tile origin in the GEMM view                           */
    uint16_t m_valid, n_valid;     /* min(tm, M - m0), min(tn, N - n0)                       */
    uint32_t flags;                /* bit 0: edge tile (some rows/columns predicated off)    */
} ft_tile_desc;

typedef struct ft_plan_stats {
    uint32_t struct_size;
    uint32_t tau;                  /* main axis: 0 rows (M), 1 columns (N)                   */
    uint32_t batch, m, n, k;       /* resolved GEMM view                                     */
    uint32_t n_ukernels;           /* 0 (empty plan), 1 or 2                                 */
    uint32_t ukernel_id[2];        /* ascending                                              */
    uint32_t count_tau[2];         /* Num1, Num2 of Alg. 2 in the same order                 */
    uint32_t block_bound;          /* min(K.wkl.block, zeta)                                 */
    uint32_t pool_size;            /* programs in uProg                                      */
    uint32_t level;                /* 0: Top-1 among programs within block.bound, 1: none was      */
    uint32_t pad_q20, occ_q20, cmr_q20;   /* Eq. 2, Eq. 3, normalised Eq. 6; floor(x * 2^20) */
    uint32_t lds_bytes;            /* dynamic LDS of the launch                              */
    uint32_t kernel_class;         /* which dispatcher kernel runs the plan                  */
    uint64_t sia_q20;              /* Eq. 1                                                  */
    uint64_t n_tiles;
    uint64_t useful_elems;         /* batch*M*N                                              */
    uint64_t covered_elems;        /* sum of tm*tn over all tiles                            */
    uint32_t k_parts;              /* workgroups per tile along the reduce axis (1 = no split)*/
    uint32_t k_part_tiles;         /* k-tiles (of tk) per part; the last part may get fewer  */
    uint64_t workspace_bytes;      /* device memory the plan owns for the partial tiles      */
    /* Second-axis strips (operators with two dynamic space axes, Fig. 4(d)): part i places
     * main_tiles[i] tiles of its own uKernel across the other axis and, if strip_ukernel_id[i] is not
     * UINT32_MAX, strip_tiles[i] tiles of that narrower uKernel (same extent along tau) after them. */
    uint32_t main_tiles[2];
    uint32_t strip_ukernel_id[2];
    uint32_t strip_tiles[2];
    uint32_t table_order;          /* 0: the tiles of each uKernel shape form a grid and a workgroup
                                      derives its descriptor's contents in closed form (checked against
                                      the table when the plan is made); 1: workgroups read the table
                                      (plans with strips)                                          */
} ft_plan_stats;

typedef struct ft_plan ft_plan;
/* op, set, shape: host pointers.  forced: host pointer, read only in mode FT_PLAN_FORCED, else
 * may be NULL.  Unless FT_PLAN_HOST_ONLY is set the descriptor table is also copied to the
 * current HIP device (one hipMalloc + one synchronous hipMemcpy).  Plans are immutable and may
 * be launched any number of times.  A plan with k_parts > 1 also owns workspace_bytes of device
 * memory for the fp32 partial tiles plus 16 bytes of counters per tile: launches of one such plan
 * must be ordered (same stream, or otherwise not overlapping), every launch leaves the counters
 * at zero, and the sum over the parts is taken in part order, so results are reproducible.
 * The split and the eight-wave uKernels run in the bodies that copy 16-byte chunks straight into LDS
 * and have no code for rows that end inside a chunk: shapes whose K or N is not a multiple of 8 are
 * never scored with a split, and a program of eight-wave uKernels runs its four-wave twins there.
 * Pointer alignment does not matter (2-byte aligned operands are copied the same way). */
ft_status ft_plan_create(const ft_op *op, const ft_ukset *set, const ft_shape *shape, uint32_t flags,
                         const ft_forced_program *forced, ft_plan **out);
/* The same plan through the set's per-shape cache (Sec. 5: the runtime stage is paid once per shape;
 * with kernels of a few microseconds a plan must not be rebuilt per call): returns the plan made
 * earlier for the same shape and flags, or makes it (as ft_plan_create would, on the current HIP
 * device unless FT_PLAN_HOST_ONLY) and keeps it.  *out stays owned by the set: valid until
 * ft_ukset_destroy, never passed to ft_plan_destroy.  Safe to call from several threads; mode
 * FT_PLAN_FORCED is not cached (FT_ERR_INVALID_ARG).  A set keeps at most 65536 plans (each owns a
 * descriptor table on the device); beyond that the call returns FT_ERR_OOM and ft_plan_create, whose
 * plans the caller destroys, is the way. */
ft_status ft_plan_cached(const ft_op *op, ft_ukset *set, const ft_shape *shape, uint32_t flags,
                         const ft_plan **out);
/* Grouped plan: n_groups batched Matmul problems of DIFFERENT shapes run by ONE launch -- a batch
 * of sequences of different lengths without padding them to the longest (the paper's motivation,
 * Sec. 1 / Fig. 1(b): padded batches waste most of their work).  op must be a batched Matmul; groups[g]
 * is a runtime shape of it (batch = number of equally shaped matrices of the group, e.g. the heads of
 * one sequence; a group with an empty extent contributes nothing).  Each group gets the program the
 * planner picks for its shape at the batch of the whole launch (Sec. 5; the groups share the device:
 * batch = the sum of the groups' batches rounded up to a power of two, at most batch_hi; the set
 * caches the program per (shape, that batch), so later launches only copy tiles); the descriptor table is the
 * concatenation of the groups' own entries, the groups with the longest reduce axis first (then the
 * largest outputs: the workgroups with the most work start first), operands stay in group
 * order, and descriptor flags carry the group in bits 12..31, the body in bits 1..7 and its LDS ring
 * depth in bits 8..11 (bit 0 as before).  Operands are packed group after group, each group's matrices densely packed as for a
 * plain batched launch; ft_plan_group_layout reports where a group starts.  Launch with ft_launch /
 * ft_launch_epilogue on the packed buffers.  Any alignment and any row length works; the launch
 * takes the faster LDS-DMA bodies when every group's rows hold at least 8 elements (k >= 8 and, with B
 * stored [K][N], n >= 8), else the general ones.  The reduce axis is never split.  flags: FT_PLAN_PATCHWORK or FT_PLAN_PAD_BASELINE, optionally
 * FT_PLAN_HOST_ONLY.  groups: host pointer, read during the call only.  n_groups < 2^20. */
ft_status ft_plan_create_grouped(const ft_op *op, ft_ukset *set, const ft_shape *groups, uint32_t n_groups,
                                 uint32_t flags, ft_plan **out);
/* Element offsets of group `group`'s first matrices in the packed A, B and C buffers, and the
 * buffers' total element counts for group == number of groups.  Host pointers. */
ft_status ft_plan_group_layout(const ft_plan *plan, uint32_t group, uint64_t *off_a, uint64_t *off_b, uint64_t *off_c);

/* *descs: host pointer to library-owned memory, valid until ft_plan_destroy. */
ft_status ft_plan_descriptors(const ft_plan *plan, const ft_tile_desc **descs, uint64_t *n);
/* Which descriptor each workgroup of the launch takes (Sec. 3: one uKernel = one thread block):
 * order[b] = index into the descriptor table of workgroup b, for b < min(*n, cap); *n receives
 * the number of workgroups (= tiles).  The order is a permutation of the table: every XCD (a
 * group of CUs with its own L2; workgroup b runs on XCD b % num_xcds) takes a contiguous slice of
 * each constituent's tiles, walked in 2-D groups.  order: host pointer, caller-owned.
 * A plan with second-axis strips (up to four uKernel shapes) is walked in table order, dealt to the
 * XCDs in chunks of 16 consecutive descriptors; its grid is rounded up to whole rounds of chunks, so
 * *n may exceed the tile count and order[b] = UINT32_MAX marks a workgroup with nothing to do.
 * With k_parts = P > 1 every entry of this order is worked on by P workgroups of the same XCD:
 * workgroup b takes entry (b / (P*X))*X + b % X and part (b / X) % P, X = num_xcds. */
ft_status ft_plan_launch_order(const ft_plan *plan, uint32_t *order, uint64_t cap, uint64_t *n);
ft_status ft_plan_stats_get(const ft_plan *plan, ft_plan_stats *out);
void ft_plan_destroy(ft_plan *plan);

/* Scores of every program of the pool for one shape (Sec. 5.1 pool, Sec. 5.2 evaluation):
 * fills up to cap entries of out (host pointer) and stores the pool size in *n. */
typedef struct ft_pool_entry {
    uint32_t k1, count1, k2, count2;       /* k2 = UINT32_MAX for a single-uKernel program   */
    uint32_t pad_q20, occ_q20, cmr_q20;
    uint32_t flags;                        /* bit0 in_bound, bit1 CrossPick, bit2 Eq. 5      */
    uint64_t sia_q20;
    uint64_t n_tiles;
} ft_pool_entry;
ft_status ft_plan_pool(const ft_op *op, const ft_ukset *set, const ft_shape *shape,
                       ft_pool_entry *out, uint32_t cap, uint32_t *n);

/* ---------------------------------------------------------------------------------------
 * (d) Launch: ONE kernel launch; workgroup i runs the uKernel body named by descriptor i.
 *   Matmul: A [M,K], B [K,N] row-major 16-bit; C [M,N] row-major fp32 (or 16-bit, see out_dtype).
 *   BMM:    A [batch,M,K], B [batch,K,N], C [batch,M,N], densely packed.
 *   Conv2d: A = X [n,H,W,c_in], B = W [r,s,c_in,c_out], C = Y [n,P,Q,c_out] fp32.
 * A, B, C: device pointers owned by the caller (A, B at least 2-byte aligned, C 4-byte
 * aligned; rows of at least 8 elements -- K >= 8 and, with B stored [K][N], N >= 8 -- take the
 * LDS-DMA bodies whatever their length and alignment, shorter ones the general bodies; any N is correct, rows of C that start on 64-byte blocks are written fastest, since
 * neighbouring tiles then share no block of memory).  hip_stream: a hipStream_t (NULL = default stream).  Asynchronous; allocates
 * nothing and does not synchronise.  An empty plan launches nothing.  The current HIP device must
 * be the one the plan was created on (else FT_ERR_INVALID_ARG).
 * ------------------------------------------------------------------------------------- */
ft_status ft_launch(const ft_plan *plan, const void *A, const void *B, void *C, void *hip_stream);

/* The same launch for operators registered with an epilogue (Sec. 6.2: Dense + bias-add as one
 * fused operator): C[.., j] = sum_k A B + bias[j].  bias: device pointer to N (= c_out for a
 * convolution) fp32 values, 4-byte aligned, owned by the caller; must be non-NULL exactly when
 * the operator has FT_EPI_BIAS (else FT_ERR_INVALID_ARG).  C has the operator's out_dtype
 * (fp32, or the inputs' 16-bit type: 2-byte aligned, same row-major layout).  ft_launch is this
 * call with bias = NULL. */
ft_status ft_launch_epilogue(const ft_plan *plan, const void *A, const void *B, void *C, const float *bias,
                             void *hip_stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: ft_launch_epilogue (bias may be NULL exactly as there) with
 * nothing allocated anywhere on the way.  The partial tiles and arrival counters of a reduce-axis
 * split, which ft_plan_create otherwise allocates per plan, live in one array that is part of the
 * library's device code (32 MiB of partial tiles + 64 KiB of counters per GPU, held until the process
 * ends), and a plan made with FT_PLAN_HOST_ONLY -- no device table, so no allocation at plan time
 * either -- is accepted as long as its workgroups derive their tiles in closed form
 * (ft_plan_stats.table_order == 0: every plan without second-axis strips; grouped plans and
 * table-order plans without a device table: FT_ERR_UNSUPPORTED).  A plan whose split needs more than
 * the array holds (n_tiles * k_parts * largest tile * 4 bytes > 32 MiB, or more than 4096 tiles) is
 * refused with FT_ERR_UNSUPPORTED; nothing is launched then.  The call clears the counters it will use
 * with a small kernel on hip_stream, then launches; it calls no allocating routine and does not
 * synchronise.  All calls on one GPU share the array: calls that may overlap in time (different
 * streams, different threads) race on it and must be ordered by the caller; ft_launch / ft_launch_epilogue
 * with plans that own their workspace do not touch it.  Same results as ft_launch_epilogue, bit for bit. */
ft_status ft_launch_noalloc(const ft_plan *plan, const void *A, const void *B, void *C, const float *bias,
                            void *hip_stream);

/* Timing helper for benchmarks: launches the plan `iters` times back to back on hip_stream,
 * launch i using buffer set i % n_sets (A, B, C: host arrays of n_sets device pointers; rotating
 * over many sets keeps operands out of the caches), between two HIP events recorded on that same
 * stream; waits for the second event and stores the mean milliseconds per launch in
 * *ms_per_launch (host pointer). */
ft_status ft_launch_timed(const ft_plan *plan, const void *const *A, const void *const *B, void *const *C,
                          uint32_t n_sets, void *hip_stream, uint32_t iters, float *ms_per_launch);

/* Attainable memory rates of the device, for the figure reported beside the 8 TB/s roofline: streams
 * `bytes` (>= 1 MiB; use far more than the 256 MB Infinity Cache) from src, to dst, and from src to dst
 * with plain 16-byte-per-lane kernels, `iters` timed launches each after one untimed, between two HIP
 * events on hip_stream, and stores GB/s (10^9 bytes; the copy counts bytes read + bytes written).
 * src, dst: device pointers to `bytes` each, 16-byte aligned, caller-owned; dst is overwritten.
 * The three results are host pointers.  Allocates nothing. */
ft_status ft_stream_rate(const void *src, void *dst, uint64_t bytes, uint32_t iters, void *hip_stream, float *read_gbs,
                         float *write_gbs, float *copy_gbs);

/* Same measurement with the `iters` launches captured once into a HIP graph (stream capture of
 * ft_launch on hip_stream, which must not be the NULL stream) and replayed: one untimed replay,
 * then one replay between the two events.  Removes the host's per-launch cost from the timed
 * region; the kernels and their order are the same. */
ft_status ft_launch_timed_graph(const ft_plan *plan, const void *const *A, const void *const *B, void *const *C,
                                uint32_t n_sets, void *hip_stream, uint32_t iters, float *ms_per_launch);

#ifdef __cplusplus
}
#endif
#endif /* FTUNER_H */
