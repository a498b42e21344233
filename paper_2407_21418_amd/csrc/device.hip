// HIP-facing half of the library: device query, descriptor-table upload and the launch.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "family.h"
#include "ft_internal.h"
#include "gemm_body.h"
#include "launch_iface.h"

// Workspace of ft_launch_noalloc: the fp32 partial tiles and arrival counters of a reduce-axis split,
// which ft_plan_create otherwise allocates per plan.  One copy per GPU, held until the process ends and
// shared by every call on that GPU.  The name is a host-side handle only: its device address comes from
// hipGetSymbolAddress (noalloc_scratch_of below) and that pointer is what the kernels are given.
#define FT_NOALLOC_COUNTER_BYTES (64u << 10)
#define FT_NOALLOC_PARTIAL_BYTES (32u << 20)
static __device__ __align__(256) unsigned char scratch[FT_NOALLOC_COUNTER_BYTES + FT_NOALLOC_PARTIAL_BYTES];

namespace ftk {
// zeroes n 32-bit words (a kernel, not a memset node: the call may be captured into a HIP graph)
__global__ void ft_clear_words(uint32_t *p, uint32_t n) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}
}  // namespace ftk

namespace ftk {
// Streaming kernels for the attainable-bandwidth figure beside the roofline: every lane moves 16
// bytes per step, a workgroup walks its own contiguous segment in 4 KB rows, eight rows in flight.
typedef uint32_t stream_u32x4 __attribute__((ext_vector_type(4)));
template <int MODE>   // 0: read, 1: write, 2: copy
__global__ __launch_bounds__(256) void ft_stream(const stream_u32x4 *__restrict__ src, stream_u32x4 *__restrict__ dst, uint64_t n16,
                                                 uint32_t *sink) {
    // every workgroup streams one contiguous segment of the buffer
    const uint64_t seg = (n16 + gridDim.x - 1) / gridDim.x;
    const uint64_t end = (blockIdx.x + 1) * seg < n16 ? (blockIdx.x + 1) * seg : n16;
    n16 = end;
    const uint64_t stride = 256u;
    stream_u32x4 acc = {0u, 0u, 0u, 0u};
    uint64_t i = (uint64_t)blockIdx.x * seg + threadIdx.x;
    constexpr int U = 8;                                   // 16-byte accesses in flight per lane
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        stream_u32x4 v[U];
        if (MODE != 1) {
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = src[i + u * stride];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (MODE == 0) acc += v[u];
            else if (MODE == 1) { const stream_u32x4 w = {(uint32_t)i, 1u, 2u, 3u}; dst[i + u * stride] = w; }
            else dst[i + u * stride] = v[u];
        }
    }
    for (; i < n16; i += stride) {
        if (MODE == 1) { const stream_u32x4 w = {(uint32_t)i, 1u, 2u, 3u}; dst[i] = w; }
        else if (MODE == 0) acc += src[i];
        else dst[i] = src[i];
    }
    if (MODE == 0 && (acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = acc[0];   // keeps the loads alive
}
}  // namespace ftk

namespace {

typedef int (*launch_fn)(const ftk::KArgs *, uint32_t, void *);
const launch_fn kLaunch[2][FT_NUM_CLASSES] = {
    {ft_launch_dt0_c0, ft_launch_dt0_c1, ft_launch_dt0_c2},
    {ft_launch_dt1_c0, ft_launch_dt1_c1, ft_launch_dt1_c2},
};

// the same bodies with the code for rows that end inside a 16-byte chunk (the ones above have none)
const launch_fn kLaunchRagged[2][FT_NUM_CLASSES] = {
    {ft_launch_dt0_rg_c0, ft_launch_dt0_rg_c1, ft_launch_dt0_rg_c2},
    {ft_launch_dt1_rg_c0, ft_launch_dt1_rg_c1, ft_launch_dt1_rg_c2},
};
// two-team bodies (eight waves): classes 0 and 1
const launch_fn kLaunchTwoTeams[2][2] = {{ft_launch_dt0_pp_c0, ft_launch_dt0_pp_c1}, {ft_launch_dt1_pp_c0, ft_launch_dt1_pp_c1}};
// general bodies: [dtype][0] = bodies with <= 64 accumulator registers (256-register kernel),
// [dtype][1] = all bodies (512-register kernel)
const launch_fn kLaunchGeneric[2][2] = {{ft_launch_dt0_gen_c1, ft_launch_dt0_gen_c2},
                                        {ft_launch_dt1_gen_c1, ft_launch_dt1_gen_c2}};
// grouped launches: the general bodies behind a dispatcher that reads each group's shape
const launch_fn kLaunchGrouped[2][2] = {{ft_launch_dt0_grp_c1, ft_launch_dt0_grp_c2},
                                        {ft_launch_dt1_grp_c1, ft_launch_dt1_grp_c2}};
const launch_fn kLaunchGroupedFast[2][3] = {{ft_launch_dt0_grpf_c0, ft_launch_dt0_grpf_c1, ft_launch_dt0_grpf_c2},
                                            {ft_launch_dt1_grpf_c0, ft_launch_dt1_grpf_c1, ft_launch_dt1_grpf_c2}};
// operand B as [N][K]: LDS-DMA bodies of the four-wave standard grids, plain and grouped
const launch_fn kLaunchNK[2][3] = {{ft_launch_dt0_nk_c0, ft_launch_dt0_nk_c1, ft_launch_dt0_nk_c2},
                                   {ft_launch_dt1_nk_c0, ft_launch_dt1_nk_c1, ft_launch_dt1_nk_c2}};
const launch_fn kLaunchGroupedNK[2][3] = {{ft_launch_dt0_grpnk_c0, ft_launch_dt0_grpnk_c1, ft_launch_dt0_grpnk_c2},
                                          {ft_launch_dt1_grpnk_c0, ft_launch_dt1_grpnk_c1, ft_launch_dt1_grpnk_c2}};
static_assert(sizeof(ftk::GroupRec) == sizeof(ft_group_rec) && sizeof(ft_group_rec) == 40,
              "the kernels read the host's group records as they are");

static_assert(sizeof(ftk::TileDesc) == sizeof(ft_tile_desc) && sizeof(ft_tile_desc) == 24,
              "descriptor layout is part of the ABI");

#ifdef FT_TRACE
uint64_t *g_trace = nullptr;      // development builds: where the next launches leave their timestamps
#endif

ft_status hip_fail(hipError_t e) {
    ftd_set_hip_error((int)e);
    return FT_ERR_HIP;
}

// Device address of `scratch` on the current device: looked up once per device, with that device
// current, and kept (every GPU holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
ft_status noalloc_scratch_of(int dev, unsigned char **out) {
    static std::mutex mu;
    static unsigned char *ptr_of[kMaxDevices] = {};
    if (dev < 0 || dev >= kMaxDevices) return FT_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr_of[dev]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!p) return FT_ERR_HIP;
        ptr_of[dev] = static_cast<unsigned char *>(p);
    }
    *out = ptr_of[dev];
    return FT_OK;
}

void fill_args(const ft_plan *p, const void *A, const void *B, void *C, const float *bias, ftk::KArgs *a) {
    std::memset(a, 0, sizeof(*a));
    const ft_plan_stats &s = p->st;
    a->A = static_cast<const uint16_t *>(A);
    a->B = static_cast<const uint16_t *>(B);
    a->C = C;
    a->bias = bias;
    a->out_kind = p->op.out_dtype == FT_OUT_SAME ? (p->op.dtype == FT_F16 ? ftk::OUT_F16 : ftk::OUT_BF16) : ftk::OUT_F32;
    a->descs = static_cast<const ftk::TileDesc *>(p->d_descs);
    a->n_tiles = (uint32_t)s.n_tiles;
    a->M = s.m; a->N = s.n; a->K = s.k;
    a->lda = s.k; a->ldb = p->op.b_layout == FT_B_NK ? s.k : s.n; a->ldc = s.n;
    a->strideA = (uint64_t)s.m * s.k;
    a->strideB = (uint64_t)s.k * s.n;
    a->strideC = (uint64_t)s.m * s.n;
    a->is_conv = p->op.kind == FT_OP_CONV2D;
    if (a->is_conv) {
        a->H = p->img_h; a->W = p->img_w; a->Cin = p->op.c_in;
        a->P = p->out_p; a->Q = p->out_q; a->R = p->op.r; a->S = p->op.s;
        a->cstride = p->op.stride; a->cpad = p->op.pad;
        a->lda = 0; a->strideA = 0;
    }
    for (int i = 0; i < 4; ++i) {
        a->slot_ukernel[i] = p->slot_id[i];
        a->slot_code[i] = p->slot_code[i];
        a->slot_stages[i] = p->slot_stages[i];
    }
    a->table_order = p->table_order ? 1u : 0u;
    for (int i = 0; i < 2; ++i) {
        a->slot_first[i] = p->slot_first[i];
        a->slot_rows[i] = p->slot_rows[i];
        a->slot_cols[i] = p->slot_cols[i];
        a->slot_group[i] = p->slot_group[i];
        a->slot_m0[i] = p->slot_m0[i]; a->slot_n0[i] = p->slot_n0[i];
        a->slot_tm[i] = p->slot_tm[i]; a->slot_tn[i] = p->slot_tn[i];
    }
    a->num_xcds = p->num_xcds;
    a->k_parts = s.k_parts > 1 && p->d_ws ? s.k_parts : 1;
    a->k_part_tiles = s.k_part_tiles;
    a->ws_tile_stride = p->ws_tile_stride;
    a->ws = static_cast<float *>(p->d_ws);
    a->arrive = static_cast<uint32_t *>(p->d_arrive);
#ifdef FT_TRACE
    a->trace = g_trace;
#endif
    // Non-temporal stores stream past the L2, which keeps the operand panels resident.  A store
    // instruction writes 128-byte row segments; where rows of C do not start on 64-byte blocks the
    // segments of neighbouring tiles share blocks, a streamed partial block goes to memory as it is
    // and a plain one waits in the L2 for its other half (the launch order keeps a batch entry's
    // tiles on one XCD).  Measured on fp32 score matrices: with rows on 64-byte blocks streamed
    // stores win (L = 240: 45 vs 58 us); otherwise plain stores win by 10-20 % when the reduce axis is
    // a single k-tile (the launch is one long store stream), streamed ones win or tie with more
    // k-tiles and with 16-bit outputs.
    const uint64_t es = a->out_kind == ftk::OUT_F32 ? 4 : 2;
    const bool lines = reinterpret_cast<uintptr_t>(C) % 64 == 0 && (a->ldc * es) % 64 == 0 &&
                       (a->strideC * es) % 64 == 0;
    a->c_stream = (lines || es == 2 || a->K > 64) ? 1u : 0u;
}

}  // namespace

ft_status ftd_upload(ft_plan *p) {
    if (p->descs.empty()) return FT_OK;
    hipError_t e = hipGetDevice(&p->device);
    if (e != hipSuccess) return hip_fail(e);
    size_t bytes = p->descs.size() * sizeof(ft_tile_desc);
    e = hipMalloc(&p->d_descs, bytes);
    if (e != hipSuccess) { p->d_descs = nullptr; return e == hipErrorOutOfMemory ? FT_ERR_OOM : hip_fail(e); }
    e = hipMemcpy(p->d_descs, p->descs.data(), bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) { ftd_release(p); return hip_fail(e); }
    if (!p->groups.empty()) {
        const size_t gbytes = p->groups.size() * sizeof(ft_group_rec);
        e = hipMalloc(&p->d_groups, gbytes);
        if (e != hipSuccess) { p->d_groups = nullptr; ftd_release(p); return e == hipErrorOutOfMemory ? FT_ERR_OOM : hip_fail(e); }
        e = hipMemcpy(p->d_groups, p->groups.data(), gbytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) { ftd_release(p); return hip_fail(e); }
    }
    if (p->st.k_parts > 1) {
        const size_t ctr_bytes = p->descs.size() * 4 * sizeof(uint32_t);
        e = hipMalloc(&p->d_ws, (size_t)p->st.workspace_bytes);
        if (e != hipSuccess) { p->d_ws = nullptr; ftd_release(p); return e == hipErrorOutOfMemory ? FT_ERR_OOM : hip_fail(e); }
        e = hipMalloc(&p->d_arrive, ctr_bytes);
        if (e != hipSuccess) { p->d_arrive = nullptr; ftd_release(p); return e == hipErrorOutOfMemory ? FT_ERR_OOM : hip_fail(e); }
        e = hipMemset(p->d_arrive, 0, ctr_bytes);        // once: every launch leaves the counters at zero
        if (e == hipSuccess) e = hipStreamSynchronize(nullptr);
        if (e != hipSuccess) { ftd_release(p); return hip_fail(e); }
    }
    return FT_OK;
}

void ftd_release(ft_plan *p) {
    if (p->d_descs) { (void)hipFree(p->d_descs); p->d_descs = nullptr; }
    if (p->d_ws) { (void)hipFree(p->d_ws); p->d_ws = nullptr; }
    if (p->d_arrive) { (void)hipFree(p->d_arrive); p->d_arrive = nullptr; }
    if (p->d_groups) { (void)hipFree(p->d_groups); p->d_groups = nullptr; }
}

static ft_status launch_common(const ft_plan *plan, const void *A, const void *B, void *C, const float *bias,
                               void *hip_stream, bool static_ws);

extern "C" {

#ifdef FT_TRACE
// development builds only: device buffer of 8 x (workgroups of the largest launch) uint64, or NULL
void ft_debug_set_trace(void *dev_buf) { g_trace = static_cast<uint64_t *>(dev_buf); }
#endif

ft_status ft_hw_query(int32_t hip_device, ft_hw_model *out) {
    if (!out) return FT_ERR_INVALID_ARG;
    ft_status st = ft_hw_default_gfx950(out);
    if (st != FT_OK) return st;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, hip_device);
    if (e != hipSuccess) return hip_fail(e);
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return FT_ERR_UNSUPPORTED;
    out->num_cus = (uint32_t)prop.multiProcessorCount;
    out->wave_size = (uint32_t)prop.warpSize;
    out->clock_mhz = (uint32_t)(prop.clockRate / 1000);
    out->lds_bytes_per_cu = (uint32_t)prop.sharedMemPerBlock;   // a workgroup may own the whole CU's LDS
    return FT_OK;
}

ft_status ft_launch(const ft_plan *plan, const void *A, const void *B, void *C, void *hip_stream) {
    return ft_launch_epilogue(plan, A, B, C, nullptr, hip_stream);
}

ft_status ft_launch_epilogue(const ft_plan *plan, const void *A, const void *B, void *C, const float *bias,
                             void *hip_stream) {
    return launch_common(plan, A, B, C, bias, hip_stream, false);
}

ft_status ft_launch_noalloc(const ft_plan *plan, const void *A, const void *B, void *C, const float *bias,
                            void *hip_stream) {
    return launch_common(plan, A, B, C, bias, hip_stream, true);
}

}  // extern "C"

// static_ws: the call is ft_launch_noalloc -- partial tiles and counters live in `scratch`, a plan
// without a device table is accepted where the kernels derive their tiles in closed form
static ft_status launch_common(const ft_plan *plan, const void *A, const void *B, void *C, const float *bias,
                               void *hip_stream, bool static_ws) {
    if (!plan) return FT_ERR_INVALID_ARG;
    if ((plan->op.epilogue == FT_EPI_BIAS) != (bias != nullptr)) return FT_ERR_INVALID_ARG;
    if (plan->st.n_tiles == 0) return FT_OK;
    if (!A || !B || !C) return FT_ERR_INVALID_ARG;
    if (!static_ws && !plan->d_descs) return FT_ERR_INVALID_ARG;   // host-only plan (found out without touching the GPU)
    int dev = -1;
    {
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return hip_fail(e);
    }
    if (!static_ws) {
        if (dev != plan->device) return FT_ERR_INVALID_ARG;     // the plan's tables live on one device
    } else {
        if (!plan->groups.empty()) return FT_ERR_UNSUPPORTED;   // grouped plans read their tables
        if (plan->d_descs ? dev != plan->device : plan->table_order) return plan->d_descs ? FT_ERR_INVALID_ARG : FT_ERR_UNSUPPORTED;
    }
    if (plan->st.kernel_class >= FT_NUM_CLASSES || plan->op.dtype > 1) return FT_ERR_UNSUPPORTED;
    ftk::KArgs a;
    fill_args(plan, A, B, C, bias, &a);
    if (static_ws && plan->st.k_parts > 1) {
        const uint64_t ctr_bytes = plan->st.n_tiles * 4 * sizeof(uint32_t);
        const uint64_t ws_bytes = plan->st.n_tiles * plan->st.k_parts * (uint64_t)plan->ws_tile_stride * sizeof(float);
        if (ctr_bytes > FT_NOALLOC_COUNTER_BYTES || ws_bytes > FT_NOALLOC_PARTIAL_BYTES) return FT_ERR_UNSUPPORTED;
        unsigned char *base = nullptr;
        ft_status st = noalloc_scratch_of(dev, &base);
        if (st != FT_OK) return st;
        a.k_parts = plan->st.k_parts;
        a.arrive = reinterpret_cast<uint32_t *>(base);
        a.ws = reinterpret_cast<float *>(base + FT_NOALLOC_COUNTER_BYTES);
    }
    if (!plan->groups.empty()) {
        // grouped launch: the dispatcher takes shape, pitches and operand bases from the group records
        if (!plan->d_groups) return FT_ERR_INVALID_ARG;
        a.groups = static_cast<const ftk::GroupRec *>(plan->d_groups);
        a.table_order = 1;
        a.k_parts = 1;
        const bool out16 = a.out_kind != ftk::OUT_F32;
        const bool on_blocks = plan->grp_rows_on_blocks && reinterpret_cast<uintptr_t>(C) % 64 == 0;
        a.c_stream = (on_blocks || out16 || plan->grp_k_min > 64) ? 1u : 0u;     // as for a plain launch
        // every group aligned and the buffers too: the LDS-DMA bodies; else the general ones
        // (the LDS-DMA bodies take any 2-byte aligned operand; grp_aligned: every group's rows hold a chunk)
        const bool fast = plan->grp_aligned && reinterpret_cast<uintptr_t>(A) % 2 == 0 && reinterpret_cast<uintptr_t>(B) % 2 == 0;
        if (plan->op.b_layout == FT_B_NK) {
            if (!fast) return FT_ERR_UNSUPPORTED;       // no general bodies for this layout
            const int rc = kLaunchGroupedNK[plan->op.dtype][ft_class_of_acc((int)plan->grp_fast_acc)](&a, plan->grp_fast_lds, hip_stream);
            if (rc != 0) return hip_fail((hipError_t)rc);
            return FT_OK;
        }
        const int rc = fast ? kLaunchGroupedFast[plan->op.dtype][ft_class_of_acc((int)plan->grp_fast_acc)](&a, plan->grp_fast_lds, hip_stream)
                            : kLaunchGrouped[plan->op.dtype][plan->grp_acc <= 64 ? 0 : 1](&a, 2 * plan->grp_stage_bytes, hip_stream);
        if (rc != 0) return hip_fail((hipError_t)rc);
        return FT_OK;
    }
    // The LDS-DMA copies take any 2-byte aligned source (measured on gfx950 with an in-bounds probe), so
    // the LDS-DMA bodies run whatever the row pitches are.  Where a row ends inside a 16-byte chunk
    // (K, or N with B stored [K][N], not a multiple of 8: "ragged") the single-team bodies fetch that
    // chunk from inside the row and fix it up in LDS (gemm_fast.h); that needs rows of at least one chunk.  Convolution: c_in a multiple of 64, c_out of 8, 16-byte aligned operands.  Everything
    // else takes the general bodies.
    const bool aligned = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (reinterpret_cast<uintptr_t>(B) % 16 == 0);
    const bool even = (reinterpret_cast<uintptr_t>(A) % 2 == 0) && (reinterpret_cast<uintptr_t>(B) % 2 == 0);
    const bool nk = plan->op.b_layout == FT_B_NK;
    const bool ragged = !a.is_conv && (a.K % 8 != 0 || (!nk && a.N % 8 != 0));
    bool fast = a.is_conv ? (aligned && a.Cin % 64 == 0 && a.N % 8 == 0)
                          : (even && a.K >= 8 && (nk || a.N >= 8) && !(ragged && plan->two_teams));
    // (no general bodies for B stored [N][K])
    if (nk && !fast) return FT_ERR_UNSUPPORTED;
    if (fast && ragged) {
        // ragged rows: the single-team bodies (and the two narrowest split-k ones) fix them up
        for (int i = 0; i < 4; ++i) a.slot_code[i] = (uint32_t)ft_ragged_code((int)a.slot_code[i]);
        a.k_parts = 1;                 // (the planner never splits such a shape; a forced split is not taken)
    }
    if (!fast || a.is_conv) {          // no split-k variant of the gather or of the general bodies: use the twin
        for (int i = 0; i < 4; ++i) {
            // (the planner derives no eight-wave grid for a convolution: its twin would run in the wrong kernel)
            if (a.is_conv && ft_is_w8_code((int)a.slot_code[i])) return FT_ERR_UNSUPPORTED;
            a.slot_code[i] = (uint32_t)ft_general_code((int)a.slot_code[i]);
            // the twins of the narrowest tiles exist in the general dispatcher only
            if (ft_is_partial_code((int)a.slot_code[i])) fast = false;
        }
        if (nk && !fast) return FT_ERR_UNSUPPORTED;
        a.k_parts = 1;                 // these bodies walk the whole reduce axis in one workgroup
    }
    if (static_ws && a.k_parts > 1) {
        // the array keeps what the last call on this GPU left in it: the counters this launch uses start at zero
        const uint32_t words = (uint32_t)plan->st.n_tiles * 4u;
        hipLaunchKernelGGL(ftk::ft_clear_words, dim3((words + 255u) / 256u), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                           a.arrive, words);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e);
    }
    int rc;
    if (plan->op.b_layout == FT_B_NK) {
        if (plan->two_teams) return FT_ERR_UNSUPPORTED;      // (such an operator derives none)
        rc = kLaunchNK[plan->op.dtype][plan->st.kernel_class](&a, plan->st.lds_bytes, hip_stream);
    } else if (fast && plan->two_teams) {
        if (plan->st.kernel_class > 1) return FT_ERR_UNSUPPORTED;
        rc = kLaunchTwoTeams[plan->op.dtype][plan->st.kernel_class](&a, plan->st.lds_bytes, hip_stream);
    } else if (fast) {
        rc = (ragged ? kLaunchRagged : kLaunch)[plan->op.dtype][plan->st.kernel_class](&a, plan->st.lds_bytes, hip_stream);
    } else {
        // the general bodies stage through registers into two LDS stages, whatever ring depth the
        // uKernel has on the LDS-DMA path
        uint32_t stage = 0;
        int acc = 0;
        for (int i = 0; i < 4; ++i) {
            stage = std::max(stage, ft_stage_bytes_of_code((int)a.slot_code[i]));
            acc = std::max(acc, ft_acc_of_code((int)a.slot_code[i]));
        }
        const uint32_t lds = 2 * stage;
        rc = kLaunchGeneric[plan->op.dtype][acc <= 64 ? 0 : 1](&a, lds, hip_stream);
    }
    if (rc != 0) return hip_fail((hipError_t)rc);
    return FT_OK;
}

extern "C" {

ft_status ft_launch_timed(const ft_plan *plan, const void *const *A, const void *const *B, void *const *C,
                          uint32_t n_sets, void *hip_stream, uint32_t iters, float *ms_per_launch) {
    if (!plan || !A || !B || !C || !n_sets || !iters || !ms_per_launch) return FT_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return hip_fail(e);
    e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(e); }
    ft_status st = FT_OK;
    e = hipEventRecord(e0, s);
    for (uint32_t i = 0; i < iters && st == FT_OK && e == hipSuccess; ++i)
        st = ft_launch(plan, A[i % n_sets], B[i % n_sets], C[i % n_sets], hip_stream);
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != FT_OK) return st;
    if (e != hipSuccess) return hip_fail(e);
    *ms_per_launch = ms / (float)iters;
    return FT_OK;
}

ft_status ft_stream_rate(const void *src, void *dst, uint64_t bytes, uint32_t iters, void *hip_stream, float *read_gbs,
                         float *write_gbs, float *copy_gbs) {
    if (!src || !dst || bytes < (1u << 20) || !iters || !read_gbs || !write_gbs || !copy_gbs) return FT_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16) return FT_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipDeviceProp_t prop;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return hip_fail(e);
    const uint64_t n16 = bytes / 16;
    const dim3 grid((unsigned)prop.multiProcessorCount * 8u), block(256);
    const auto *sp = static_cast<const ftk::stream_u32x4 *>(src);
    auto *dp = static_cast<ftk::stream_u32x4 *>(dst);
    uint32_t *sink = static_cast<uint32_t *>(dst);             // written only if a checksum matches a constant
    hipEvent_t e0, e1;
    e = hipEventCreate(&e0);
    if (e != hipSuccess) return hip_fail(e);
    e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(e); }
    float *outs[3] = {read_gbs, write_gbs, copy_gbs};
    for (int mode = 0; mode < 3 && e == hipSuccess; ++mode) {
        for (uint32_t i = 0; i <= iters && e == hipSuccess; ++i) {      // one untimed launch first
            if (i == 1) e = hipEventRecord(e0, s);
            if (mode == 0) hipLaunchKernelGGL(ftk::ft_stream<0>, grid, block, 0, s, sp, dp, n16, sink);
            else if (mode == 1) hipLaunchKernelGGL(ftk::ft_stream<1>, grid, block, 0, s, sp, dp, n16, sink);
            else hipLaunchKernelGGL(ftk::ft_stream<2>, grid, block, 0, s, sp, dp, n16, sink);
        }
        if (e == hipSuccess) e = hipEventRecord(e1, s);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess) *outs[mode] = (float)((mode == 2 ? 2.0 : 1.0) * (double)(n16 * 16) * iters / (ms * 1e6));
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return hip_fail(e);
    return FT_OK;
}

ft_status ft_launch_timed_graph(const ft_plan *plan, const void *const *A, const void *const *B, void *const *C,
                                uint32_t n_sets, void *hip_stream, uint32_t iters, float *ms_per_launch) {
    if (!plan || !A || !B || !C || !n_sets || !iters || !ms_per_launch || !hip_stream) return FT_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ft_status st = FT_OK;
    hipError_t e = hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) return hip_fail(e);
    for (uint32_t i = 0; i < iters && st == FT_OK; ++i)
        st = ft_launch(plan, A[i % n_sets], B[i % n_sets], C[i % n_sets], hip_stream);
    e = hipStreamEndCapture(s, &graph);          // always end the capture, also after a failed launch
    if (st == FT_OK && e == hipSuccess) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (st == FT_OK && e == hipSuccess) e = hipEventCreate(&e0);
    if (st == FT_OK && e == hipSuccess) e = hipEventCreate(&e1);
    if (st == FT_OK && e == hipSuccess) e = hipGraphLaunch(exec, s);             // untimed replay
    if (st == FT_OK && e == hipSuccess) e = hipStreamSynchronize(s);
    if (st == FT_OK && e == hipSuccess) e = hipEventRecord(e0, s);
    if (st == FT_OK && e == hipSuccess) e = hipGraphLaunch(exec, s);
    if (st == FT_OK && e == hipSuccess) e = hipEventRecord(e1, s);
    if (st == FT_OK && e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (st == FT_OK && e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (exec) (void)hipGraphExecDestroy(exec);
    if (graph) (void)hipGraphDestroy(graph);
    if (st != FT_OK) return st;
    if (e != hipSuccess) return hip_fail(e);
    *ms_per_launch = ms / (float)iters;
    return FT_OK;
}

}  // extern "C"
