// C ABI of the library (see include/pod_attn.h).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/pod_attn.h"
#include "pod_common.h"
#include "pod_launch.h"
#include "pod_planner.h"

struct pod_attn_plan {
    pod::Plan p;
    uint64_t serial = 0;                    // unique per plan object of this process, never reused
};

namespace {

thread_local std::string g_last_error;
std::atomic<uint64_t> g_next_plan_serial{1};

// Which plan's work tables each GPU's static scratch holds (0 = none), for pod_attn_forward_static.
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
uint64_t g_static_owner[kMaxDevices] = {0};

pod_status fail(pod_status code, const std::string &msg)
{
    g_last_error = msg;
    return code;
}

pod_status fail_hip(hipError_t e, const char *what)
{
    return fail(POD_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

int device_cu_count()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return 256; }
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return 256;
    }
    return n;
}

pod::KernelArgs make_args(const pod::Plan &p, const void *prefill_q, const void *decode_q,
                          const void *k_cache, const void *v_cache, const int32_t *seq_meta,
                          const int32_t *block_table, void *out, void *workspace)
{
    pod::KernelArgs a;
    std::memset(&a, 0, sizeof a);
    unsigned char *ws = (unsigned char *)workspace;
    a.prefill_q = prefill_q; a.decode_q = decode_q; a.k_cache = k_cache; a.v_cache = v_cache;
    a.seq_meta = seq_meta; a.block_table = block_table; a.out = out;
    a.hdr = (pod::WsHeader *)ws;
    a.pitems = (const pod::PrefillItem *)(ws + p.off_pitems);
    a.pitems_by_wg = (const pod::PrefillItem *)(ws + p.off_pitems_by_wg);
    a.dunits = (const pod::DecodeUnit *)(ws + p.off_dunits);
    a.centries = (const pod::CombineEntry *)(ws + p.off_centries);
    a.crows = (const int32_t *)(ws + p.off_crows);
    a.n_crows = (int)(p.crows.size() / 2);
    a.part_o = (float *)(ws + p.off_part_o);
    a.part_ml = (float *)(ws + p.off_part_ml);
    a.kv_seq_stride = p.prm.kv_seq_stride;
    {
        const int64_t d = p.prm.head_dim, hkv = p.prm.n_kv_heads, bs = p.prm.block_size;
        a.block_elems = bs * hkv * d;
        if (p.prm.kv_order == POD_KV_HEAD_MAJOR) {
            a.tok_stride = (int32_t)d;
            a.head_stride = bs > 0 ? bs * d : p.prm.kv_seq_stride / (hkv * d) * d;
        } else {
            a.tok_stride = (int32_t)(hkv * d);
            a.head_stride = d;
        }
    }
    a.n_prefill = p.prm.n_prefill;
    a.n_q_heads = p.prm.n_q_heads;
    a.n_kv_heads = p.prm.n_kv_heads;
    a.group = p.group;
    a.block_size = p.prm.block_size;
    a.max_blocks_per_seq = p.prm.max_blocks_per_seq;
    a.bs_shift = -1;
    if (p.prm.block_size > 0 && (p.prm.block_size & (p.prm.block_size - 1)) == 0) {
        int s = 0;
        while ((1 << s) < p.prm.block_size) ++s;
        a.bs_shift = s;
    }
    a.n_pitems = (int)p.pitems.size();
    a.n_dunits = (int)p.dunits.size();
    a.n_dwgs = p.n_dwgs;
    a.fused_grid = p.fused_grid;
    for (int q = 0; q <= pod::kXcdQueues; ++q) a.pq_begin[q] = p.pq_begin[q];
    // Every workgroup of a launch with decode work asks for a decode seat sooner or later and the
    // grid is never smaller than the number of seats, so all fixed units are run whatever
    // operation the workgroups start with.
    a.dq_begin = (const int32_t *)(ws + p.off_dq);
    a.n_static_seats = p.n_static_seats;
    a.n_dctas = ((int)p.dunits.size() + pod::kWavesPerWg - 1) / pod::kWavesPerWg;
    a.single_unit = 0;
    a.n_combine = (int)p.centries.size();
    a.n_prefill_rows = (int)p.n_prefill_rows;
    a.p_ratio = p.p_ratio;
    a.d_ratio = p.d_ratio;
    a.scale_log2 = p.prm.softmax_scale * 1.4426950408889634f;
    a.trace = (pod::TraceRecord *)p.trace;
    a.evlog = (uint32_t *)p.evlog;
    a.evlog_cap = p.evlog ? (uint32_t)((p.evlog_bytes - 16) / sizeof(pod::EventRecord)) : 0u;
    return a;
}

// The two streams the two-kernel modes run their kernels on: one pair per GPU, created at the
// first such call on that GPU and kept until the process ends.  (A pair per plan would be spread
// over the few hardware queues a process has in creation order, and a later plan's pair can land
// on one queue, where its two kernels run one after the other.)
pod_status side_streams(hipStream_t *s0, hipStream_t *s1)
{
    static std::mutex mu;
    static hipStream_t pair[kMaxDevices][2] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "asking for the current device");
    if (dev < 0 || dev >= kMaxDevices) return fail(POD_ERR_UNSUPPORTED, "device index beyond what the library tracks");
    std::lock_guard<std::mutex> lock(mu);
    for (hipStream_t &st : pair[dev])
        if (!st) {
            e = hipStreamCreateWithFlags(&st, hipStreamNonBlocking);
            if (e != hipSuccess) { st = nullptr; return fail_hip(e, "creating side stream"); }
        }
    *s0 = pair[dev][0];
    *s1 = pair[dev][1];
    return POD_OK;
}

// Clear the counters at the head of `workspace` (with a kernel, not a memset) and copy the plan's
// work tables behind them; returns when the copies have completed.
pod_status upload_tables(const pod::Plan &p, void *workspace, hipStream_t s)
{
    unsigned char *ws = (unsigned char *)workspace;
    hipError_t e = pod::clear_header((pod::WsHeader *)ws, s);
    if (e != hipSuccess) return fail_hip(e, "clearing workspace counters");
    struct Part { size_t off; const void *src; size_t bytes; };
    const Part parts[6] = {
        {p.off_pitems_by_wg, p.pitems_by_wg.data(), p.pitems_by_wg.size() * sizeof(pod::PrefillItem)},
        {p.off_dq, p.dq_begin, sizeof p.dq_begin},
        {p.off_pitems, p.pitems.data(), p.pitems.size() * sizeof(pod::PrefillItem)},
        {p.off_dunits, p.dunits.data(), p.dunits.size() * sizeof(pod::DecodeUnit)},
        {p.off_centries, p.centries.data(), p.centries.size() * sizeof(pod::CombineEntry)},
        {p.off_crows, p.crows.data(), p.crows.size() * sizeof(int32_t)}};
    for (const Part &part : parts) {
        if (part.bytes == 0) continue;
        e = hipMemcpyAsync(ws + part.off, part.src, part.bytes, hipMemcpyHostToDevice, s);
        if (e != hipSuccess) return fail_hip(e, "copying plan tables");
    }
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return fail_hip(e, "waiting for plan upload");
    return POD_OK;
}

}  // namespace

extern "C" {

const char *pod_attn_last_error(void) { return g_last_error.c_str(); }
const char *pod_attn_version(void) { return "pod_attn 0.1 (gfx950)"; }

pod_status pod_attn_plan_create(const pod_attn_params *params, const int32_t *seq_meta_host,
                                pod_attn_plan **plan)
{
    if (!params || !plan) return fail(POD_ERR_INVALID_ARG, "params or plan is null");
    *plan = nullptr;
    const int n_cus = params->n_compute_units > 0 ? params->n_compute_units : device_cu_count();
    pod_attn_plan *obj = new (std::nothrow) pod_attn_plan();
    if (!obj) return fail(POD_ERR_INVALID_ARG, "out of host memory");
    std::string err;
    pod_status st;
    try {
        st = pod::build_plan(*params, seq_meta_host, n_cus, obj->p, err);
    } catch (const std::bad_alloc &) {
        st = POD_ERR_INVALID_ARG;
        err = "out of host memory";
    }
    if (st != POD_OK) {
        delete obj;
        return fail(st, err);
    }
    obj->serial = g_next_plan_serial.fetch_add(1);
    *plan = obj;
    return POD_OK;
}

void pod_attn_plan_destroy(pod_attn_plan *plan)
{
    if (!plan) return;
    for (void *&e : plan->p.events)
        if (e) { (void)hipEventDestroy((hipEvent_t)e); e = nullptr; }
    delete plan;
}

pod_status pod_attn_plan_info_get(const pod_attn_plan *plan, pod_attn_plan_info *info)
{
    if (!plan || !info) return fail(POD_ERR_INVALID_ARG, "plan or info is null");
    const pod::Plan &p = plan->p;
    info->n_prefill_items = (int32_t)p.pitems.size();
    info->n_decode_units = (int32_t)p.dunits.size();
    info->n_combine = (int32_t)p.centries.size();
    info->max_prefill_splits = p.max_psplits;
    info->max_decode_splits = p.max_dsplits;
    info->decode_chunk = p.decode_chunk;
    info->prefill_ratio = p.p_ratio;
    info->decode_ratio = p.d_ratio;
    info->fused_grid = p.fused_grid;
    info->n_compute_units = p.n_cus;
    info->n_prefill_rows = p.n_prefill_rows;
    info->n_partial_rows = p.n_partial_rows;
    info->workspace_bytes = (int64_t)p.ws_bytes;
    info->prefill_heavy_advised = p.heavy_advised ? 1 : 0;
    info->reserved0 = 0;
    return POD_OK;
}

pod_status pod_attn_plan_set_trace(pod_attn_plan *plan, void *trace, size_t trace_bytes)
{
    if (!plan) return fail(POD_ERR_INVALID_ARG, "plan is null");
    // one record per workgroup of the largest launch: the two stand-alone kernels together, or the fused round
    const size_t n_dctas = (plan->p.dunits.size() + pod::kWavesPerWg - 1) / pod::kWavesPerWg;
    const size_t n_records = std::max(plan->p.pitems.size() + n_dctas, (size_t)plan->p.fused_grid);
    const size_t need = n_records * sizeof(pod::TraceRecord);
    if (trace && trace_bytes < need) return fail(POD_ERR_WORKSPACE, "trace buffer too small");
    plan->p.trace = trace;
    plan->p.trace_bytes = trace ? trace_bytes : 0;
    return POD_OK;
}

pod_status pod_attn_plan_set_event_log(pod_attn_plan *plan, void *log, size_t log_bytes)
{
    if (!plan) return fail(POD_ERR_INVALID_ARG, "plan is null");
    if (log && log_bytes < 16 + sizeof(pod::EventRecord)) return fail(POD_ERR_WORKSPACE, "event log too small");
    if (log && ((uintptr_t)log & 15)) return fail(POD_ERR_INVALID_ARG, "event log must be 16-byte aligned");
    plan->p.evlog = log;
    plan->p.evlog_bytes = log ? log_bytes : 0;
    return POD_OK;
}

size_t pod_attn_workspace_size(const pod_attn_plan *plan) { return plan ? plan->p.ws_bytes : 0; }

pod_status pod_attn_plan_prefill_item(const pod_attn_plan *plan, int32_t index, int32_t out[8])
{
    if (!plan || !out || index < 0 || index >= (int32_t)plan->p.pitems.size())
        return fail(POD_ERR_INVALID_ARG, "prefill item index out of range");
    const pod::PrefillItem &it = plan->p.pitems[(size_t)index];
    const int32_t v[8] = {it.req, it.kv_head, it.row0, it.n_rows, it.kv_begin, it.kv_end, it.prow0, it.split};
    std::memcpy(out, v, sizeof v);
    return POD_OK;
}

pod_status pod_attn_plan_prefill_item_of_workgroup(const pod_attn_plan *plan, int32_t workgroup, int32_t out[8])
{
    if (!plan || !out || workgroup < 0 || workgroup >= (int32_t)plan->p.pitems_by_wg.size())
        return fail(POD_ERR_INVALID_ARG, "workgroup index out of range");
    const pod::PrefillItem &it = plan->p.pitems_by_wg[(size_t)workgroup];
    const int32_t v[8] = {it.req, it.kv_head, it.row0, it.n_rows, it.kv_begin, it.kv_end, it.prow0, it.split};
    std::memcpy(out, v, sizeof v);
    return POD_OK;
}

pod_status pod_attn_plan_decode_unit(const pod_attn_plan *plan, int32_t index, int32_t out[8])
{
    if (!plan || !out || index < 0 || index >= (int32_t)plan->p.dunits.size())
        return fail(POD_ERR_INVALID_ARG, "decode unit index out of range");
    const pod::DecodeUnit &u = plan->p.dunits[(size_t)index];
    const int32_t v[8] = {u.req, u.kv_head, u.t0, u.t1, u.prow0, u.split, u.q_start, u.cache_row};
    std::memcpy(out, v, sizeof v);
    return POD_OK;
}

pod_status pod_attn_plan_decode_queue(const pod_attn_plan *plan, int32_t q, int32_t *begin, int32_t *end)
{
    if (!plan || !begin || !end || q < 0 || q >= pod::kXcdQueues)
        return fail(POD_ERR_INVALID_ARG, "decode queue index out of range");
    *begin = plan->p.dq_begin[q];
    *end = plan->p.dq_begin[q + 1];
    return POD_OK;
}

pod_status pod_attn_plan_upload(const pod_attn_plan *plan, void *workspace, size_t workspace_bytes,
                                void *stream)
{
    if (!plan) return fail(POD_ERR_INVALID_ARG, "plan is null");
    const pod::Plan &p = plan->p;
    if (!workspace || workspace_bytes < p.ws_bytes) return fail(POD_ERR_WORKSPACE, "workspace missing or too small");
    if (((uintptr_t)workspace & 255u) != 0) return fail(POD_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    return upload_tables(p, workspace, (hipStream_t)stream);
}

static pod_status forward_impl(const void *prefill_q, const void *decode_q, const void *k_cache,
                               const void *v_cache, const int32_t *seq_meta, const int32_t *block_table,
                               void *out, const pod_attn_plan *plan, void *workspace,
                               size_t workspace_bytes, int32_t mode, void *stream, bool use_static)
{
    if (!plan) return fail(POD_ERR_INVALID_ARG, "plan is null");
    pod::Plan &p = const_cast<pod_attn_plan *>(plan)->p;
    const bool paged = p.prm.block_size > 0;
    const int n_req = p.prm.n_prefill + p.prm.n_decode;
    const bool no_combine = (mode & POD_MODE_FLAG_NO_COMBINE) != 0;
    const bool cta_parallel = (mode & POD_MODE_FLAG_CTA_PARALLEL) != 0;
    const bool heavy = (mode & POD_MODE_FLAG_PREFILL_HEAVY) != 0;
    mode &= ~(POD_MODE_FLAG_NO_COMBINE | POD_MODE_FLAG_CTA_PARALLEL | POD_MODE_FLAG_PREFILL_HEAVY);
    if (heavy && cta_parallel) return fail(POD_ERR_INVALID_ARG, "POD_MODE_FLAG_PREFILL_HEAVY and POD_MODE_FLAG_CTA_PARALLEL exclude each other");
    if (heavy && mode != POD_MODE_FUSED && mode != POD_MODE_DECODE_ONLY && mode != POD_MODE_PREFILL_ONLY)
        return fail(POD_ERR_INVALID_ARG, "POD_MODE_FLAG_PREFILL_HEAVY goes with POD_MODE_FUSED (or with one operation alone)");
    if (cta_parallel && mode != POD_MODE_FUSED)
        return fail(POD_ERR_INVALID_ARG, "POD_MODE_FLAG_CTA_PARALLEL goes with POD_MODE_FUSED only");
    if (mode < POD_MODE_FUSED || mode > POD_MODE_DECODE_ONLY) return fail(POD_ERR_INVALID_ARG, "unknown mode");
    if (n_req == 0) return POD_OK;
    if (!k_cache || !v_cache || !seq_meta || !out) return fail(POD_ERR_INVALID_ARG, "k_cache, v_cache, seq_meta or out is null");
    if (p.prm.n_prefill > 0 && !prefill_q) return fail(POD_ERR_INVALID_ARG, "prefill_q is null");
    if (p.prm.n_decode > 0 && !decode_q) return fail(POD_ERR_INVALID_ARG, "decode_q is null");
    if (paged && !block_table) return fail(POD_ERR_INVALID_ARG, "block_table is null for a paged cache");
    if (heavy) {
        const bool block_wise = !paged || ((p.prm.block_size & (p.prm.block_size - 1)) == 0 && p.prm.block_size >= 16);
        if (p.prm.head_dim != 128 || !block_wise)
            return fail(POD_ERR_UNSUPPORTED, "the prefill-heavy configuration is built for head_dim 128 and contiguous or "
                                             "power-of-two (>= 16) block caches");
    }
    if (use_static) {
        if (mode == POD_MODE_STREAMS || (heavy && mode == POD_MODE_FUSED))
            return fail(POD_ERR_UNSUPPORTED, "the two-stream mode creates streams and events; it is not available "
                                             "from the entry point that allocates nothing");
        if (p.ws_bytes > pod::kStaticScratchBytes)
            return fail(POD_ERR_WORKSPACE, "this batch needs " + std::to_string(p.ws_bytes) + " bytes of workspace, the "
                        "library's static scratch holds " + std::to_string(pod::kStaticScratchBytes) +
                        ": use pod_attn_forward with a workspace of the caller's");
    } else {
        if (!workspace || workspace_bytes < p.ws_bytes) return fail(POD_ERR_WORKSPACE, "workspace missing or too small");
        if (((uintptr_t)workspace & 255u) != 0) return fail(POD_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    }
    // every row is read and written in 16-byte pieces
    if ((((uintptr_t)prefill_q | (uintptr_t)decode_q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out) & 15u) != 0)
        return fail(POD_ERR_INVALID_ARG, "prefill_q, decode_q, k_cache, v_cache and out must be 16-byte aligned");
    if ((((uintptr_t)seq_meta | (uintptr_t)block_table) & 3u) != 0)
        return fail(POD_ERR_INVALID_ARG, "seq_meta and block_table must be 4-byte aligned");
    if (use_static) {
        // This GPU's copy of the static array.  It is shared by every call on the GPU and keeps the
        // last call's contents: when it holds another plan's tables (or none), the counters are
        // cleared and this plan's tables copied in before the launch.
        int dev = 0;
        hipError_t de = hipGetDevice(&dev);
        if (de != hipSuccess) return fail_hip(de, "asking for the current device");
        if (dev < 0 || dev >= kMaxDevices) return fail(POD_ERR_UNSUPPORTED, "device index beyond what the static scratch tracks");
        de = pod::static_scratch(&workspace);
        if (de != hipSuccess) return fail_hip(de, "looking up the static scratch of this device");
        std::lock_guard<std::mutex> lock(g_static_mu);
        if (g_static_owner[dev] != plan->serial) {
            g_static_owner[dev] = 0;
            const pod_status up = upload_tables(p, workspace, (hipStream_t)stream);
            if (up != POD_OK) return up;
            g_static_owner[dev] = plan->serial;
        }
    }

    pod::KernelArgs a = make_args(p, prefill_q, decode_q, k_cache, v_cache, seq_meta, block_table, out, workspace);
    hipStream_t s = (hipStream_t)stream;
    const int dt = p.prm.dtype, hd = p.prm.head_dim;
    hipError_t e = hipSuccess;
    auto go = [&](int which, const pod::KernelArgs &args, hipStream_t on) {
        if (which == pod::kLaunchCombine && no_combine) return;
        if (e == hipSuccess) e = pod::launch(which, args, dt, hd, paged, on);
    };

    // The combine pass only touches rows whose partials were produced in this call; the row list
    // holds the rows of prefill groups first, then those of decode groups.
    pod::KernelArgs only_p = a, only_d = a;
    only_p.n_crows = p.n_crows_prefill;
    only_d.crows = a.crows + 2 * (size_t)p.n_crows_prefill;
    only_d.n_crows = a.n_crows - p.n_crows_prefill;

    // Prefill kernel and decode kernel on the library's two side streams, forked from and joined
    // back into the caller's stream; the merge follows on the caller's stream.
    auto two_streams = [&](int prefill_kind, int decode_kind) -> pod_status {
        hipStream_t s0 = nullptr, s1 = nullptr;
        {
            const pod_status ss = side_streams(&s0, &s1);
            if (ss != POD_OK) return ss;
        }
        for (void *&ev : p.events)
            if (!ev) {
                hipEvent_t ne;
                hipError_t ce = hipEventCreateWithFlags(&ne, hipEventDisableTiming);
                if (ce != hipSuccess) return fail_hip(ce, "creating event");
                ev = ne;
            }
        hipEvent_t fork = (hipEvent_t)p.events[0], j0 = (hipEvent_t)p.events[1], j1 = (hipEvent_t)p.events[2];
        auto chk = [&](hipError_t x) { if (e == hipSuccess) e = x; };
        chk(hipEventRecord(fork, s));
        chk(hipStreamWaitEvent(s0, fork, 0));
        chk(hipStreamWaitEvent(s1, fork, 0));
        go(prefill_kind, a, s0);
        go(decode_kind, a, s1);
        chk(hipEventRecord(j0, s0));
        chk(hipEventRecord(j1, s1));
        chk(hipStreamWaitEvent(s, j0, 0));
        chk(hipStreamWaitEvent(s, j1, 0));
        go(pod::kLaunchCombine, a, s);
        return POD_OK;
    };

    switch (mode) {
    case POD_MODE_FUSED:
        if (heavy) {
            // two prefill workgroups and one light decode workgroup per compute unit, from two kernels
            if (p.prm.n_prefill == 0 || p.prm.n_decode == 0) {
                go(p.prm.n_decode == 0 ? pod::kLaunchPrefillHeavy : pod::kLaunchDecodeLite, a, s);
                go(pod::kLaunchCombine, a, s);
            } else {
                const pod_status st = two_streams(pod::kLaunchPrefillHeavy, pod::kLaunchDecodeLite);
                if (st != POD_OK) return st;
            }
            break;
        }
        if (cta_parallel) {
            // one workgroup per work item: every decode workgroup is given its four units by index
            pod::KernelArgs c = a;
            c.n_static_seats = c.n_dctas;
            c.single_unit = 1;
            go(pod::kLaunchFusedCta, c, s);
        } else {
            go(pod::kLaunchFused, a, s);
        }
        go(pod::kLaunchCombine, a, s);
        break;
    case POD_MODE_SERIAL:
        go(pod::kLaunchPrefill, a, s);
        go(pod::kLaunchDecode, a, s);
        go(pod::kLaunchCombine, a, s);
        break;
    case POD_MODE_PREFILL_ONLY:
        go(heavy ? pod::kLaunchPrefillHeavy : pod::kLaunchPrefill, a, s);
        go(pod::kLaunchCombine, only_p, s);
        break;
    case POD_MODE_DECODE_ONLY:
        go(heavy ? pod::kLaunchDecodeLite : pod::kLaunchDecode, a, s);
        go(pod::kLaunchCombine, only_d, s);
        break;
    case POD_MODE_STREAMS: {
        const pod_status st = two_streams(pod::kLaunchPrefill, pod::kLaunchDecode);
        if (st != POD_OK) return st;
        break;
    }
    default:
        break;
    }
    if (e != hipSuccess) return fail_hip(e, "launching attention kernels");
    return POD_OK;
}

pod_status pod_attn_forward(const void *prefill_q, const void *decode_q, const void *k_cache,
                            const void *v_cache, const int32_t *seq_meta, const int32_t *block_table,
                            void *out, const pod_attn_plan *plan, void *workspace,
                            size_t workspace_bytes, int32_t mode, void *stream)
{
    return forward_impl(prefill_q, decode_q, k_cache, v_cache, seq_meta, block_table, out, plan, workspace,
                        workspace_bytes, mode, stream, false);
}

pod_status pod_attn_forward_static(const void *prefill_q, const void *decode_q, const void *k_cache,
                                   const void *v_cache, const int32_t *seq_meta, const int32_t *block_table,
                                   void *out, const pod_attn_plan *plan, int32_t mode, void *stream)
{
    return forward_impl(prefill_q, decode_q, k_cache, v_cache, seq_meta, block_table, out, plan, nullptr, 0,
                        mode, stream, true);
}

static_assert(pod::kStaticScratchBytes == POD_ATTN_STATIC_SCRATCH_BYTES, "the header states the size of the static scratch");

int32_t pod_attn_role_for_ticket(int32_t ticket, int32_t prefill_ratio, int32_t decode_ratio, int32_t unit)
{
    if (ticket < 0 || unit < 0 || prefill_ratio < 0 || decode_ratio < 0 || prefill_ratio + decode_ratio <= 0) return -1;
    return pod::role_for_ticket((uint32_t)ticket, prefill_ratio, decode_ratio, unit);
}

// Host model of the fused launch.  Every actor is a small state machine whose steps are the
// atomic operations the device code performs, in the device's order; `order` decides whose step
// comes next, which stands for every timing the hardware could produce.
int32_t pod_attn_simulate_launch(const pod_attn_plan *plan, const int32_t *unit_of_wg, int32_t n_wgs,
                                 const int32_t *order, int32_t n_order, int32_t *first_role,
                                 int32_t *seat_of_wg, int32_t *item_owner, int32_t *unit_owner)
{
    if (!plan || n_wgs < 0 || n_order < 0 || (n_wgs > 0 && !unit_of_wg) || (n_order > 0 && !order)) return -1;
    const pod::Plan &p = plan->p;
    const int n_items = (int)p.pitems.size(), n_units = (int)p.dunits.size();
    for (int i = 0; i < n_items && item_owner; ++i) item_owner[i] = -1;
    for (int i = 0; i < n_units && unit_owner; ++i) unit_owner[i] = -1;
    constexpr int W = pod::kWavesPerWg, Q = pod::kXcdQueues;

    // the counters of the workspace header
    std::vector<uint32_t> cu_ticket(pod::kCuSlots, 0u);
    uint32_t next_seat = 0, next_pitem[Q] = {0}, next_dunit[Q] = {0};

    enum Phase { kBind, kPrefillClaims, kSeat, kDecodeWaves, kEnd };
    struct Wave { int cq = 0, tried = 0; bool started = false, done = false; };
    struct Wg {
        Phase phase = kBind;
        int first = pod::kNone, roles_done = 0, xcd = 0, seat = -1;
        int pq = 0, ptried = 0;                // prefill queue cursor (kept across the role switch, as on the device)
        Wave wave[W];
    };
    std::vector<Wg> wgs((size_t)n_wgs);
    int32_t owner_errors = 0;

    auto next_phase = [&](Wg &g) {
        // after a role has run dry: the other role, then the end
        ++g.roles_done;
        if (g.roles_done >= 2) { g.phase = kEnd; return; }
        const int next_role = g.first == pod::kPrefill ? pod::kDecode : pod::kPrefill;
        g.phase = next_role == pod::kPrefill ? kPrefillClaims : kSeat;
    };
    auto start_role = [&](Wg &g, int role) { g.phase = role == pod::kPrefill ? kPrefillClaims : kSeat; };
    auto wg_finished = [&](const Wg &g) { return g.phase == kEnd; };

    // One step of workgroup w's leader (actor 4w) or of its wavefront v (actor 4w + v) while the
    // workgroup is a decode worker.  Returns false when that actor has nothing to do right now.
    auto step = [&](int actor) -> bool {
        const int w = actor / W, v = actor % W;
        if (w < 0 || w >= n_wgs) return false;
        Wg &g = wgs[(size_t)w];
        switch (g.phase) {
        case kBind: {
            if (v != 0) return false;
            const unsigned cu = (unsigned)unit_of_wg[w] & (pod::kCuSlots - 1);
            const uint32_t ticket = cu_ticket[cu]++;
            g.first = pod::role_for_ticket(ticket, p.p_ratio, p.d_ratio, (int)cu);
            g.xcd = (int)(cu >> 6);
            g.pq = g.xcd & (Q - 1);
            if (first_role) first_role[w] = g.first;
            start_role(g, g.first);
            return true;
        }
        case kPrefillClaims: {
            if (v != 0) return false;
            // one claim: the queue's counter is only touched while the queue is not known to be empty
            if (g.ptried >= Q) { next_phase(g); return true; }
            const int len = p.pq_begin[g.pq + 1] - p.pq_begin[g.pq];
            const int k = len > 0 ? (int)next_pitem[g.pq]++ : len;
            if (k < len) {
                const int item = p.pq_begin[g.pq] + k;
                if (item_owner) { if (item_owner[item] != -1) ++owner_errors; item_owner[item] = w; }
            } else {
                g.pq = (g.pq + 1) & (Q - 1);
                ++g.ptried;
            }
            return true;
        }
        case kSeat: {
            if (v != 0) return false;
            g.seat = (int)next_seat++;
            if (seat_of_wg) seat_of_wg[w] = g.seat;
            if (g.seat < p.n_dwgs) {
                g.phase = kDecodeWaves;
                for (Wave &x : g.wave) { x = Wave(); x.cq = g.xcd & (Q - 1); }
            } else {
                next_phase(g);                  // every seat is taken: the seated workers stream the decode work
            }
            return true;
        }
        case kDecodeWaves: {
            Wave &x = g.wave[v];
            if (x.done) return false;
            auto own = [&](int unit) { if (unit_owner) { if (unit_owner[unit] != -1) ++owner_errors; unit_owner[unit] = actor; } };
            if (!x.started && g.seat < p.n_static_seats) {
                x.started = true;
                own(g.seat * W + v);            // the fixed first unit: no claim
            } else {
                x.started = true;
                // one claim on the queue the wavefront is at; a used-up queue sends it to the next
                // non-empty one, and after all eight it is done
                const int q0 = p.dq_begin[x.cq], q1 = p.dq_begin[x.cq + 1];
                const int k = (int)next_dunit[x.cq]++;
                if (k < q1 - q0) own(q0 + k);
                else {
                    do {
                        x.cq = (x.cq + 1) & (Q - 1);
                        ++x.tried;
                    } while (x.tried < Q && p.dq_begin[x.cq + 1] == p.dq_begin[x.cq]);
                    if (x.tried >= Q) x.done = true;
                }
            }
            bool all = true;
            for (const Wave &y : g.wave) all = all && y.done;
            if (all) next_phase(g);
            return true;
        }
        default:
            return false;
        }
    };

    int32_t steps = 0;
    for (int32_t i = 0; i < n_order; ++i)
        if (step(order[i])) ++steps;
    // whoever is not finished yet runs on, round-robin, until the launch has drained
    for (bool progress = true; progress;) {
        progress = false;
        for (int w = 0; w < n_wgs; ++w) {
            if (wg_finished(wgs[(size_t)w])) continue;
            for (int v = 0; v < W; ++v)
                if (step(w * W + v)) { ++steps; progress = true; }
        }
    }
    return owner_errors ? -2 : steps;
}

}  // extern "C"
