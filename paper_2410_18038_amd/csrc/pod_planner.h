// Host-side plan: how one hybrid batch is cut into prefill items, decode units and combine
// groups, and where each table lives in the device workspace.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/pod_attn.h"
#include "pod_common.h"

namespace pod {

struct Plan {
    pod_attn_params prm;
    int n_cus = 256;
    int group = 1;
    std::vector<int32_t> meta;              // host copy of seq_meta
    bool heavy_advised = false;             // see pod_attn_plan_info.prefill_heavy_advised
    std::vector<PrefillItem> pitems;
    // The same items in the order the stand-alone prefill kernels take them by workgroup index: the
    // hardware deals workgroups to the XCDs round-robin, so workgroup b gets an item of queue b % 8.
    std::vector<PrefillItem> pitems_by_wg;
    std::vector<DecodeUnit> dunits;
    std::vector<CombineEntry> centries;
    std::vector<int32_t> crows;             // (entry, row) pairs, prefill entries first
    int n_crows_prefill = 0;
    int64_t n_prefill_rows = 0;
    int64_t n_partial_rows = 0;
    int p_ratio = 1, d_ratio = 1;
    int decode_chunk = 0;
    int max_psplits = 1, max_dsplits = 1;
    int pq_begin[kXcdQueues + 1] = {0};     // per-XCD prefill queues inside pitems
    int dq_begin[16] = {0};                 // per-XCD decode queues inside dunits (entries 0..8 used)
    int n_static_seats = 0;                 // decode seats whose first four units are fixed
    int n_dwgs = 0;                         // decode workers: workgroups of the stand-alone decode kernel, decode seats of the fused one
    int fused_grid = 0;                     // workgroups of the fused kernel
    // byte offsets inside the workspace (each 256-byte aligned)
    size_t off_pitems = 0, off_pitems_by_wg = 0, off_dunits = 0, off_centries = 0, off_crows = 0, off_dq = 0, off_part_o = 0, off_part_ml = 0;
    size_t ws_bytes = 0;
    // events of the two-kernel modes (fork, two joins), created on first use
    void *events[3] = {nullptr, nullptr, nullptr};
    void *trace = nullptr;                  // device buffer for TraceRecords, or null
    size_t trace_bytes = 0;
    void *evlog = nullptr;                  // device buffer for the event log, or null
    size_t evlog_bytes = 0;
};

// Validates and fills `plan`; returns POD_OK or an error code with a message in `err`.
pod_status build_plan(const pod_attn_params &prm, const int32_t *seq_meta, int n_cus, Plan &plan,
                      std::string &err);

// Reduce a (prefill workgroups : decode workgroups) count to the small role ratio of Section 4.1.
void role_ratio(int policy, int n_prefill_wgs, int n_decode_wgs, int &p, int &d);

}  // namespace pod
