// Host planner: validates a hybrid batch and cuts it into work items (paper Section 4.1: the
// numbers of prefill and decode workgroups are fixed on the host before the launch).
#include "pod_planner.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <numeric>

namespace pod {

namespace {

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
int ceil_div(int a, int b) { return (a + b - 1) / b; }
int round_up(int a, int b) { return ceil_div(a, b) * b; }

std::string fmt(const char *f, long long a = 0, long long b = 0, long long c = 0)
{
    char buf[256];
    std::snprintf(buf, sizeof buf, f, a, b, c);
    return buf;
}

}  // namespace

void role_ratio(int policy, int n_prefill_wgs, int n_decode_wgs, int &p, int &d)
{
    if (n_prefill_wgs <= 0 && n_decode_wgs <= 0) { p = 1; d = 1; return; }
    if (n_prefill_wgs <= 0) { p = 0; d = 1; return; }
    if (n_decode_wgs <= 0) { p = 1; d = 0; return; }
    if (policy == POD_POLICY_ALTERNATE) { p = 1; d = 1; return; }
    // Proportional (Section 4.1; Section 5.4.2 gives 50 prefill + 100 decode -> 1 : 2).
    const int kMaxSide = 8;
    if (n_decode_wgs >= n_prefill_wgs) {
        p = 1;
        d = std::min(kMaxSide, (int)std::lround((double)n_decode_wgs / n_prefill_wgs));
    } else {
        d = 1;
        p = std::min(kMaxSide, (int)std::lround((double)n_prefill_wgs / n_decode_wgs));
    }
    p = std::max(p, 1);
    d = std::max(d, 1);
}

pod_status build_plan(const pod_attn_params &prm, const int32_t *seq_meta, int n_cus, Plan &plan,
                      std::string &err)
{
    // ---- parameters --------------------------------------------------------------------
    if (prm.n_prefill < 0 || prm.n_decode < 0) { err = "negative request count"; return POD_ERR_INVALID_ARG; }
    if (prm.n_q_heads <= 0 || prm.n_kv_heads <= 0 || prm.n_q_heads % prm.n_kv_heads != 0) {
        err = "n_q_heads must be a positive multiple of n_kv_heads";
        return POD_ERR_INVALID_ARG;
    }
    const int group = prm.n_q_heads / prm.n_kv_heads;
    if (group > kMaxGroup) { err = "more than 16 query heads per K/V head"; return POD_ERR_UNSUPPORTED; }
    if (prm.head_dim != 64 && prm.head_dim != 128 && prm.head_dim != 256) { err = "head_dim must be 64, 128 or 256"; return POD_ERR_UNSUPPORTED; }
    if (prm.head_dim == 256 && group > kMaxGroup256) { err = "head_dim 256: more than 8 query heads per K/V head"; return POD_ERR_UNSUPPORTED; }
    if (prm.dtype != POD_F16 && prm.dtype != POD_BF16) { err = "dtype must be POD_F16 or POD_BF16"; return POD_ERR_UNSUPPORTED; }
    if (!(prm.softmax_scale > 0.f) || !std::isfinite(prm.softmax_scale)) {
        err = "softmax_scale must be positive and finite";
        return POD_ERR_INVALID_ARG;
    }
    if (prm.block_size < 0) { err = "negative block_size"; return POD_ERR_INVALID_ARG; }
    if (prm.n_cache_rows <= 0) { err = "n_cache_rows must be positive"; return POD_ERR_INVALID_ARG; }
    const bool paged = prm.block_size > 0;
    if (paged && (prm.max_blocks_per_seq <= 0 || prm.n_blocks <= 0)) {
        err = "paged cache needs max_blocks_per_seq and n_blocks";
        return POD_ERR_INVALID_ARG;
    }
    if (!paged && prm.kv_seq_stride <= 0) { err = "contiguous cache needs kv_seq_stride"; return POD_ERR_INVALID_ARG; }
    if (!paged && prm.kv_seq_stride % 8 != 0) { err = "kv_seq_stride must be a multiple of 8 elements (rows are read in 16-byte pieces)"; return POD_ERR_INVALID_ARG; }
    if (prm.kv_order != POD_KV_TOKEN_MAJOR && prm.kv_order != POD_KV_HEAD_MAJOR) { err = "unknown kv_order"; return POD_ERR_INVALID_ARG; }
    if (!paged && prm.kv_order == POD_KV_HEAD_MAJOR && prm.kv_seq_stride % ((int64_t)prm.n_kv_heads * prm.head_dim) != 0) {
        err = "head-major contiguous cache: kv_seq_stride must be a multiple of n_kv_heads * head_dim";
        return POD_ERR_INVALID_ARG;
    }
    if (prm.policy < POD_POLICY_AUTO || prm.policy > POD_POLICY_PROPORTIONAL) { err = "unknown policy"; return POD_ERR_INVALID_ARG; }
    if (prm.max_prefill_waves < 0 || prm.decode_chunk < 0 || prm.prefill_split_len < 0) {
        err = "negative tuning parameter";
        return POD_ERR_INVALID_ARG;
    }
    const int n_req = prm.n_prefill + prm.n_decode;
    if (n_req > 0 && seq_meta == nullptr) { err = "seq_meta is null"; return POD_ERR_INVALID_ARG; }
    if (n_cus <= 0) { err = "n_compute_units must be positive"; return POD_ERR_INVALID_ARG; }

    // ---- requests ----------------------------------------------------------------------
    const int64_t token_elems = (int64_t)prm.n_kv_heads * prm.head_dim;
    std::vector<std::pair<int, int>> spans;         // prefill (q_start, q_len)
    std::vector<char> decode_row_used((size_t)prm.n_decode, 0);
    int64_t n_prefill_rows = 0;
    for (int r = 0; r < n_req; ++r) {
        const int32_t *m = seq_meta + 4 * r;
        const int q_start = m[0], q_len = m[1], kv_len = m[2], row = m[3];
        if (q_len < 1) { err = fmt("request %lld: q_len must be >= 1", r); return POD_ERR_INVALID_ARG; }
        if (kv_len < q_len) { err = fmt("request %lld: kv_len %lld < q_len %lld", r, kv_len, q_len); return POD_ERR_INVALID_ARG; }
        if (q_start < 0) { err = fmt("request %lld: negative q_start", r); return POD_ERR_INVALID_ARG; }
        if (row < 0 || row >= prm.n_cache_rows) { err = fmt("request %lld: cache_row %lld out of range", r, row); return POD_ERR_INVALID_ARG; }
        if (paged) {
            if (ceil_div(kv_len, prm.block_size) > prm.max_blocks_per_seq) {
                err = fmt("request %lld: kv_len %lld needs more than max_blocks_per_seq blocks", r, kv_len);
                return POD_ERR_INVALID_ARG;
            }
        } else if ((int64_t)kv_len * token_elems > prm.kv_seq_stride) {
            err = fmt("request %lld: kv_len %lld does not fit in kv_seq_stride", r, kv_len);
            return POD_ERR_INVALID_ARG;
        }
        if (r < prm.n_prefill) {
            spans.emplace_back(q_start, q_len);
            n_prefill_rows = std::max<int64_t>(n_prefill_rows, (int64_t)q_start + q_len);
        } else {
            if (q_len != 1) { err = fmt("decode request %lld: q_len must be 1", r); return POD_ERR_INVALID_ARG; }
            if (q_start >= prm.n_decode) { err = fmt("decode request %lld: q_start out of range", r); return POD_ERR_INVALID_ARG; }
            if (decode_row_used[(size_t)q_start]) { err = fmt("decode request %lld: q_start used twice", r); return POD_ERR_INVALID_ARG; }
            decode_row_used[(size_t)q_start] = 1;
        }
    }
    // The prefill query ranges must tile [0, sum q_len): `out` holds exactly sum q_len prefill rows
    // followed by the decode rows, so a gap would push the decode rows past the end of a buffer
    // sized as documented, and an overlap would have two requests write one row.
    std::sort(spans.begin(), spans.end());
    int64_t next_row = 0;
    for (size_t i = 0; i < spans.size(); ++i) {
        if (spans[i].first != next_row) {
            err = spans[i].first < next_row ? "prefill query ranges overlap"
                                            : "prefill query ranges leave a gap (q_start must continue where the previous chunk ends)";
            return POD_ERR_INVALID_ARG;
        }
        next_row += spans[i].second;
    }
    // packed rows (token x head-in-group) are indexed with 32 bits
    if (n_prefill_rows * group > (int64_t)1 << 30) { err = "too many prefill rows"; return POD_ERR_INVALID_ARG; }

    plan = Plan();
    plan.prm = prm;
    plan.n_cus = n_cus;
    plan.group = group;
    plan.meta.assign(seq_meta, seq_meta + 4 * (size_t)n_req);
    plan.n_prefill_rows = n_prefill_rows;

    int64_t next_prow = 0;

    // ---- decode chunk (needed first: how much decode there is decides the prefill split cap) ------
    int64_t token_heads = 0;
    for (int r = prm.n_prefill; r < n_req; ++r) token_heads += (int64_t)seq_meta[4 * r + 2] * prm.n_kv_heads;
    int decode_chunk = prm.decode_chunk;
    if (decode_chunk <= 0) {
        // About four units per streaming wavefront (there are four of those per compute unit):
        // ragged contexts and wavefronts of unequal speed still balance (units are claimed
        // longest first), and units stay long enough (>= 512 keys) that their partial rows
        // stay small next to the stream.  (Measured: between 1024 and 4096 keys the choice
        // moves the time by 1 %; finer cuts gain nothing once the ring runs on across unit
        // boundaries, and cost partial rows and claims.)
        const int64_t slots = (int64_t)n_cus * 8;
        // The floor is 768 keys as long as that still leaves a unit for every streaming wavefront
        // (measured on batches of 16 requests at 4K-16K keys, 1.5-2.2 units per wavefront: 2-6 %
        // faster than 512, which in turn beats 256 and 384; 1024 is slower again), else 512.
        const int64_t floor_keys = token_heads / 768 >= (int64_t)n_cus * kWavesPerWg ? 768 : 512;
        decode_chunk = (int)std::min<int64_t>(2048, std::max<int64_t>(floor_keys, (token_heads + 2 * slots - 1) / (2 * slots)));
        decode_chunk = round_up(decode_chunk, 256);
    }
    decode_chunk = round_up(std::max(decode_chunk, kDecodeStep), kDecodeStep);
    // Does the decode work seat a worker on every compute unit (at least four units for each)?
    int64_t decode_units_at_least = 0;
    for (int r = prm.n_prefill; r < n_req; ++r)
        decode_units_at_least += (int64_t)prm.n_kv_heads * ceil_div(seq_meta[4 * r + 2], decode_chunk);
    const bool decode_on_every_unit = decode_units_at_least >= (int64_t)kWavesPerWg * n_cus;

    // ---- prefill items -----------------------------------------------------------------
    // Row blocks of 128 packed rows per K/V head; split-KV only when there are too few blocks to
    // fill the chip, and never beyond `max_prefill_waves` chip-wide rounds (Section 4.2.4).
    {
        const int kPrefillRows = prefill_item_rows(prm.head_dim), kPrefillKvTile = prefill_kv_tile(prm.head_dim);
        int64_t base_items = 0;
        for (int r = 0; r < prm.n_prefill; ++r)
            base_items += (int64_t)prm.n_kv_heads * ceil_div(seq_meta[4 * r + 1] * group, kPrefillRows);
        // Default: two rounds of the chip, as in the paper; one, when a decode worker holds one of
        // the two slots of every unit for most of the launch, so that the items fill the other
        // slots once (measured on the ratio sweep: equal or up to 3 % faster, never slower; fewer
        // items also mean fewer partial rows to merge).
        const int waves = prm.max_prefill_waves > 0 ? prm.max_prefill_waves : (decode_on_every_unit ? 1 : 2);
        const int64_t cap_items = (int64_t)waves * n_cus;
        const int s_cap = base_items > 0 ? (int)std::max<int64_t>(1, cap_items / base_items) : 1;
        const int min_split = round_up(prm.prefill_split_len > 0 ? prm.prefill_split_len : 1024, kPrefillKvTile);
        for (int r = 0; r < prm.n_prefill; ++r) {
            const int q_len = seq_meta[4 * r + 1], kv_len = seq_meta[4 * r + 2];
            const int prefix = kv_len - q_len;
            const int rows_total = q_len * group;
            for (int kvh = 0; kvh < prm.n_kv_heads; ++kvh)
                for (int row0 = 0; row0 < rows_total; row0 += kPrefillRows) {
                    const int n_rows = std::min(kPrefillRows, rows_total - row0);
                    const int last_tok = (row0 + n_rows - 1) / group;
                    const int kmax = prefix + last_tok + 1;          // keys this block can see
                    const int n_tiles = ceil_div(kmax, kPrefillKvTile);
                    int s = std::min(s_cap, std::max(1, kmax / min_split));
                    const int tps = ceil_div(n_tiles, s);
                    s = ceil_div(n_tiles, tps);
                    int64_t prow_base = -1;
                    if (s > 1) {
                        prow_base = next_prow;
                        next_prow += (int64_t)s * kPrefillRows;
                        plan.centries.push_back(CombineEntry{kPrefill, r, kvh, row0, n_rows, s,
                                                             (int32_t)prow_base, kPrefillRows,
                                                             seq_meta[4 * r], q_len, 0, 0});
                    }
                    for (int i = 0; i < s; ++i) {
                        PrefillItem it;
                        it.req = r; it.kv_head = kvh; it.row0 = row0; it.n_rows = n_rows;
                        it.kv_begin = i * tps * kPrefillKvTile;
                        it.kv_end = std::min(kmax, (i + 1) * tps * kPrefillKvTile);
                        it.prow0 = s > 1 ? (int32_t)(prow_base + (int64_t)i * kPrefillRows) : -1;
                        it.split = i;
                        plan.pitems.push_back(it);
                    }
                    plan.max_psplits = std::max(plan.max_psplits, s);
                }
        }
        // One queue per XCD (each XCD has its own L2): items of one K/V head go to one queue, so
        // the workgroups that re-read that head's K/V tiles share an L2 and the re-reads do not
        // reach HBM.  Inside a queue: longest first, since ids are claimed in order.  A worker
        // whose own queue is empty takes items from the other queues.
        // With fewer (request, K/V head) streams than queues, a stream's row blocks are dealt over
        // several queues, so that every XCD has a queue of its own to start from.
        const int n_streams = prm.n_prefill * prm.n_kv_heads;
        const int per = n_streams > 0 && n_streams < kXcdQueues ? kXcdQueues / n_streams : 1;
        auto queue_of = [&](const PrefillItem &x) {
            const int stream = x.req * prm.n_kv_heads + x.kv_head;
            return (stream * per + (x.row0 / kPrefillRows) % per) % kXcdQueues;
        };
        std::stable_sort(plan.pitems.begin(), plan.pitems.end(), [&](const PrefillItem &x, const PrefillItem &y) {
            const int qx = queue_of(x), qy = queue_of(y);
            if (qx != qy) return qx < qy;
            return (x.kv_end - x.kv_begin) > (y.kv_end - y.kv_begin);
        });
        int at = 0;
        for (int q = 0; q <= kXcdQueues; ++q) {
            while (at < (int)plan.pitems.size() && queue_of(plan.pitems[(size_t)at]) < q) ++at;
            plan.pq_begin[q] = q == kXcdQueues ? (int)plan.pitems.size() : at;
        }
        // Order for the kernels that take items by workgroup index (one workgroup per item, no
        // claims): workgroup b runs on XCD b % 8 (measured: the dispatcher deals them round-robin
        // without exception), so it gets the next item of queue b % 8 and a K/V head's tiles stay in
        // the L2 of the XCDs its queue belongs to.  Queues of unequal length: what is left over goes
        // to the workgroups whose own queue has run out.
        {
            const int n = (int)plan.pitems.size();
            plan.pitems_by_wg.assign((size_t)n, PrefillItem{});
            int next[kXcdQueues];
            for (int q = 0; q < kXcdQueues; ++q) next[q] = plan.pq_begin[q];
            std::vector<int> unfilled;
            for (int b = 0; b < n; ++b) {
                const int q = b % kXcdQueues;
                if (next[q] < plan.pq_begin[q + 1]) plan.pitems_by_wg[(size_t)b] = plan.pitems[(size_t)next[q]++];
                else unfilled.push_back(b);
            }
            size_t u = 0;
            for (int q = 0; q < kXcdQueues; ++q)
                while (next[q] < plan.pq_begin[q + 1]) plan.pitems_by_wg[(size_t)unfilled[u++]] = plan.pitems[(size_t)next[q]++];
        }
    }

    // ---- decode units ------------------------------------------------------------------
    {
        const int chunk = decode_chunk;
        plan.decode_chunk = chunk;
        std::vector<int> cuts;
        {
            size_t n_est = 0;
            for (int r = prm.n_prefill; r < n_req; ++r)
                n_est += (size_t)prm.n_kv_heads * (size_t)(seq_meta[4 * r + 2] / chunk + 3);
            plan.dunits.reserve(n_est);
            plan.centries.reserve(plan.centries.size() + (size_t)prm.n_decode * prm.n_kv_heads);
        }
        for (int r = prm.n_prefill; r < n_req; ++r) {
            const int kv_len = seq_meta[4 * r + 2];
            const int s = ceil_div(kv_len, chunk);
            const int tps = round_up(ceil_div(kv_len, s), kDecodeStep);
            // Token ranges of the request: equal pieces of tps keys, except that the last piece
            // is cut again into a half and two quarters when those are still at least 128 keys
            // (a request that fits one piece stays whole and needs no merge).
            // Units are claimed longest first, so the short pieces are what is left at the end of
            // a launch, when the wavefronts that are still busy decide when it ends.
            cuts.clear();
            for (int t = 0; t < kv_len; t += tps) cuts.push_back(t);
            {
                const int t_last = cuts.back(), len = kv_len - t_last;
                const int quarter = round_up(len / 4, kDecodeStep);
                const int half = (len - 2 * quarter) / kDecodeStep * kDecodeStep;    // cuts stay multiples of a step
                if (cuts.size() >= 2 && quarter >= 128 && half > 0 && half + quarter < len) {
                    cuts.push_back(t_last + half);
                    cuts.push_back(t_last + half + quarter);
                }
            }
            cuts.push_back(kv_len);
            const int s_eff = (int)cuts.size() - 1;
            for (int kvh = 0; kvh < prm.n_kv_heads; ++kvh) {
                int64_t prow_base = -1;
                if (s_eff > 1) {
                    prow_base = next_prow;
                    next_prow += (int64_t)s_eff * group;
                    plan.centries.push_back(CombineEntry{kDecode, r, kvh, 0, group, s_eff, (int32_t)prow_base, group,
                                                         seq_meta[4 * r], 1, 0, 0});
                }
                for (int i = 0; i < s_eff; ++i) {
                    DecodeUnit u;
                    u.req = r; u.kv_head = kvh;
                    u.t0 = cuts[(size_t)i];
                    u.t1 = cuts[(size_t)i + 1];
                    u.prow0 = s_eff > 1 ? (int32_t)(prow_base + (int64_t)i * group) : -1;
                    u.split = i; u.q_start = seq_meta[4 * r]; u.cache_row = seq_meta[4 * r + 3];
                    plan.dunits.push_back(u);
                }
                plan.max_dsplits = std::max(plan.max_dsplits, s_eff);
            }
        }
        std::stable_sort(plan.dunits.begin(), plan.dunits.end(), [](const DecodeUnit &x, const DecodeUnit &y) {
            return (x.t1 - x.t0) > (y.t1 - y.t0);
        });
        // Decode workers are persistent: each of their wavefronts claims units until none is left.
        // One worker per compute unit: four streaming wavefronts per unit already keep HBM busy,
        // and a second worker on the unit makes the stream slower, not faster (measured: 681 ->
        // 656 us on a 4.3 GB batch; the eight wavefronts of a unit and the XCDs among each other
        // then get very unequal shares, and the slowest wavefronts decide when the launch ends).
        plan.n_dwgs = std::min(n_cus, ceil_div((int)plan.dunits.size(), kWavesPerWg));
        // The first workers to take a decode seat (one per compute unit) start with four fixed
        // units each, the longest ones, and claim nothing for them.  The other units are dealt
        // round-robin, still longest first, to one queue per XCD: a wavefront claims from the
        // queue of the XCD it runs on and moves to the next queue when that one is empty, so the
        // eight counters are each hit by an eighth of the chip.
        const int n_units = (int)plan.dunits.size();
        plan.n_static_seats = std::min(n_cus, n_units / kWavesPerWg);
        const int n_fixed = plan.n_static_seats * kWavesPerWg;
        std::vector<DecodeUnit> dealt;
        dealt.reserve((size_t)(n_units - n_fixed));
        for (int q = 0; q < kXcdQueues; ++q) {
            plan.dq_begin[q] = n_fixed + (int)dealt.size();
            for (int j = n_fixed + q; j < n_units; j += kXcdQueues) dealt.push_back(plan.dunits[(size_t)j]);
        }
        plan.dq_begin[kXcdQueues] = n_units;
        std::copy(dealt.begin(), dealt.end(), plan.dunits.begin() + n_fixed);
    }
    if (next_prow > (int64_t)1 << 30) { err = "too many partial rows"; return POD_ERR_INVALID_ARG; }
    plan.n_partial_rows = next_prow;

    // One (entry, row) pair per output row that is merged from partials, prefill entries first.
    {
        size_t n_pairs = 0;
        for (const CombineEntry &c : plan.centries) n_pairs += (size_t)c.n_rows;
        plan.crows.reserve(2 * n_pairs);
    }
    for (size_t e = 0; e < plan.centries.size(); ++e) {
        const CombineEntry &c = plan.centries[e];
        for (int r = 0; r < c.n_rows; ++r) {
            if (c.kind == kPrefill && (c.row0 + r) / group >= c.q_len) continue;
            plan.crows.push_back((int32_t)e);
            plan.crows.push_back(r);
        }
        if (c.kind == kPrefill) plan.n_crows_prefill = (int)(plan.crows.size() / 2);
    }

    // The ratio compares workgroup counts as the paper does (Section 4.1): decode work counts as the
    // workgroups it would fill at one wavefront per unit, up to one resident round.
    const int n_decode_ctas = std::min(2 * n_cus, ceil_div((int)plan.dunits.size(), kWavesPerWg));
    role_ratio(prm.policy, (int)plan.pitems.size(), n_decode_ctas, plan.p_ratio, plan.d_ratio);
    // Automatic policy: a unit seats one decode worker at most, so starting more than one of its
    // two workgroups in the decode role only leaves some units with two candidates for a seat and
    // others with none (measured on a 256-token chunk beside 256 decodes: 1812 against 1750 us).
    if (prm.policy == POD_POLICY_AUTO && plan.d_ratio > plan.p_ratio && plan.p_ratio > 0) plan.d_ratio = plan.p_ratio;
    // The fused launch is one resident round of workgroups (two per compute unit) that loop over
    // work, or fewer when the batch is smaller than that.
    plan.fused_grid = std::min(2 * n_cus, (int)plan.pitems.size() + plan.n_dwgs);
    // With a decode worker for every unit and some prefill work, the round is launched in full
    // even when the items are fewer than the remaining slots: every unit then gets one workgroup
    // that starts in each operation, and the decode seats are taken one per unit at once (a unit
    // that got a single workgroup would start it on prefill and be left without a decode worker).
    if (plan.n_dwgs == n_cus && !plan.pitems.empty()) plan.fused_grid = 2 * n_cus;

    // ---- which occupancy configuration suits the batch (Section 4.2.2) ----------------------
    // The prefill-heavy configuration pays when the prefill work outlasts the decode stream even
    // though that stream is the slower one there: matrix time of the prefill (at the datasheet
    // peak) above 1.2 x the time the batch's K/V bytes take at the HBM peak.
    {
        double pairs = 0.0, kv_tokens = 0.0;
        for (int r = 0; r < n_req; ++r) {
            const double q_len = seq_meta[4 * r + 1], kv_len = seq_meta[4 * r + 2];
            kv_tokens += kv_len;
            if (r < prm.n_prefill) pairs += q_len * (kv_len - q_len) + q_len * (q_len + 1.0) / 2.0;
        }
        const double flop_time = 4.0 * prm.head_dim * pairs * prm.n_q_heads / 2.5e15;
        const double byte_time = kv_tokens * prm.n_kv_heads * prm.head_dim * 4.0 / 8.0e12;
        const bool block_wise = prm.block_size == 0 || (prm.block_size >= 16 && (prm.block_size & (prm.block_size - 1)) == 0);
        plan.heavy_advised = prm.head_dim == 128 && block_wise && prm.n_prefill > 0 && prm.n_decode > 0 &&
                             flop_time > 1.2 * byte_time;
    }

    // ---- workspace layout --------------------------------------------------------------
    size_t off = align256(sizeof(WsHeader));
    plan.off_pitems = off;   off = align256(off + plan.pitems.size() * sizeof(PrefillItem));
    plan.off_pitems_by_wg = off; off = align256(off + plan.pitems_by_wg.size() * sizeof(PrefillItem));
    plan.off_dunits = off;   off = align256(off + plan.dunits.size() * sizeof(DecodeUnit));
    plan.off_centries = off; off = align256(off + plan.centries.size() * sizeof(CombineEntry));
    plan.off_crows = off;    off = align256(off + plan.crows.size() * sizeof(int32_t));
    plan.off_dq = off;       off = align256(off + sizeof plan.dq_begin);
    plan.off_part_o = off;   off = align256(off + (size_t)plan.n_partial_rows * prm.head_dim * sizeof(float));
    plan.off_part_ml = off;  off = align256(off + (size_t)plan.n_partial_rows * 2 * sizeof(float));
    plan.ws_bytes = off;
    return POD_OK;
}

}  // namespace pod
