// Internal types shared by the host logic (host.cpp) and the HIP-facing code (device.hip).
#pragma once
#include <stdint.h>
#include <map>
#include <mutex>
#include <vector>

#include "ftuner.h"

struct ft_op {
    ft_op_desc d;
};

struct ft_ukset {
    ft_op_desc op;
    ft_hw_model hw;
    ft_tuning t;
    std::vector<ft_ukernel_info> uk;   // canonical order
    uint64_t cap_q;                    // best compute_eff of the set (normaliser of Eq. 1's CMR term)
    // per-shape plan cache (ft_plan_cached): key = (flags, batch, m, n, k, img_n, img_h, img_w); the
    // set owns the plans
    std::mutex cache_mu;
    std::map<std::vector<uint32_t>, ft_plan *> cache;
};

// shape and operand offsets (in elements) of one group of a grouped launch; the kernels read it
struct ft_group_rec {
    uint32_t m, n, k, batch;
    uint64_t off_a, off_b, off_c;
};

struct ft_plan {
    ft_op_desc op;
    ft_plan_stats st;
    std::vector<ft_tile_desc> descs;
    // launch parameters
    uint32_t slot_id[4];                                   // uKernels of the plan (2 parts + their strips)
    uint32_t slot_code[4];
    uint32_t slot_stages[4];
    uint32_t n_slots;
    bool table_order;                                      // workgroup b takes descriptor b (plans with strips)
    bool two_teams;                                        // the plan's uKernels are two-team bodies (eight waves)
    uint32_t slot_first[2], slot_rows[2], slot_cols[2];   // tile grid of each constituent in the table
    uint32_t slot_group[2];                                // tile rows per group of the launch order
    uint32_t slot_m0[2], slot_n0[2], slot_tm[2], slot_tn[2];   // closed form of each constituent's descriptors
    uint32_t num_xcds;
    uint32_t img_h, img_w, out_p, out_q;   // conv geometry
    void *d_descs;                          // device copy of descs (NULL for host-only / empty plans)
    // reduce axis split over workgroups (st.k_parts > 1): fp32 partial tiles and arrival counters
    uint32_t ws_tile_stride;                // floats per (tile, part) slab: largest tm*tn of the plan
    void *d_ws;                             // [n_tiles][k_parts][ws_tile_stride] floats
    void *d_arrive;                         // [n_tiles][4] counters, zero between launches
    int device;
    // grouped launch (ft_plan_create_grouped): one record per group, device copy, launch parameters
    std::vector<ft_group_rec> groups;
    void *d_groups;
    uint32_t grp_stage_bytes;               // largest LDS stage of the bodies the groups use
    uint32_t grp_acc;                       // most accumulator registers of those bodies
    uint32_t grp_k_min;                     // shortest reduce axis of the groups that have tiles
    bool grp_rows_on_blocks;                // every group's rows of C start on 64-byte blocks (given such a C)
    bool grp_aligned;                       // every group fits the LDS-DMA bodies (given 16-byte aligned A, B)
    uint32_t grp_fast_lds, grp_fast_acc;    // LDS bytes and accumulator registers the LDS-DMA bodies need
};

// device.hip
ft_status ftd_upload(ft_plan *p);
void ftd_release(ft_plan *p);
void ftd_set_hip_error(int e);
