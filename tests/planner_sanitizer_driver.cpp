// Host-only driver for the planner, built by tests/test_planner_sanitizers.py with the address and
// undefined-behaviour sanitizers of the host compiler: seeded random batches (valid and invalid),
// every tuning value, and structural checks on each plan that was accepted.  Prints one summary
// line and returns 0, or the first violated check and 1.  No GPU, no HIP runtime.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <string>
#include <utility>
#include <vector>

#include "../paper_2410_18038_amd/csrc/pod_planner.h"

namespace {

uint64_t g_state = 0x9e3779b97f4a7c15ull;
uint32_t rnd()
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(g_state >> 33);
}
int pick(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }
template <class T, size_t N> T one_of(const T (&v)[N]) { return v[rnd() % N]; }

#define CHECK(cond, ...)                                                              \
    do {                                                                               \
        if (!(cond)) {                                                                 \
            std::printf("case %d: check failed: %s  (", g_case, #cond);               \
            std::printf(__VA_ARGS__);                                                  \
            std::printf(")\n");                                                        \
            return false;                                                              \
        }                                                                              \
    } while (0)

int g_case = 0;

bool check_plan(const pod_attn_params &prm, const std::vector<int32_t> &meta, const pod::Plan &p)
{
    const int n_req = prm.n_prefill + prm.n_decode;
    const int group = prm.n_q_heads / prm.n_kv_heads;
    CHECK(p.group == group, "group %d", p.group);
    // prefill items: in bounds, and every (request, K/V head, row block) covers its keys exactly once
    std::map<std::pair<int, std::pair<int, int>>, std::vector<std::pair<int, int>>> cover;
    for (const pod::PrefillItem &it : p.pitems) {
        CHECK(it.req >= 0 && it.req < prm.n_prefill, "item request %d", it.req);
        const int q_len = meta[4 * it.req + 1], kv_len = meta[4 * it.req + 2];
        CHECK(it.kv_head >= 0 && it.kv_head < prm.n_kv_heads, "item head %d", it.kv_head);
        CHECK(it.row0 >= 0 && it.n_rows > 0 && it.row0 + it.n_rows <= q_len * group, "rows %d+%d", it.row0, it.n_rows);
        CHECK(it.kv_begin >= 0 && it.kv_begin < it.kv_end && it.kv_end <= kv_len, "keys %d..%d of %d", it.kv_begin,
              it.kv_end, kv_len);
        CHECK(it.prow0 == -1 || (it.prow0 >= 0 && it.prow0 + pod::prefill_item_rows(prm.head_dim) <= p.n_partial_rows), "partial row %d",
              it.prow0);
        cover[{it.req, {it.kv_head, it.row0}}].push_back({it.kv_begin, it.kv_end});
    }
    for (auto &kv : cover) {
        auto &v = kv.second;
        std::sort(v.begin(), v.end());
        const int r = kv.first.first, row0 = kv.first.second.second;
        const int q_len = meta[4 * r + 1], kv_len = meta[4 * r + 2];
        const int n_rows = std::min(pod::prefill_item_rows(prm.head_dim), q_len * group - row0);
        const int kmax = kv_len - q_len + (row0 + n_rows - 1) / group + 1;
        CHECK(v.front().first == 0 && v.back().second == kmax, "cover %d..%d of %d", v.front().first, v.back().second, kmax);
        for (size_t i = 1; i < v.size(); ++i) CHECK(v[i].first == v[i - 1].second, "gap at %d", v[i].first);
    }
    for (int q = 0; q < pod::kXcdQueues; ++q)
        CHECK(p.pq_begin[q] >= 0 && p.pq_begin[q] <= p.pq_begin[q + 1] && p.pq_begin[q + 1] <= (int)p.pitems.size(),
              "prefill queue %d", q);
    // decode units: in bounds, every (request, K/V head) covered exactly once
    std::map<std::pair<int, int>, int64_t> keys;
    for (const pod::DecodeUnit &u : p.dunits) {
        CHECK(u.req >= prm.n_prefill && u.req < n_req, "unit request %d", u.req);
        const int kv_len = meta[4 * u.req + 2];
        CHECK(u.kv_head >= 0 && u.kv_head < prm.n_kv_heads, "unit head %d", u.kv_head);
        CHECK(u.t0 >= 0 && u.t0 < u.t1 && u.t1 <= kv_len, "unit keys %d..%d of %d", u.t0, u.t1, kv_len);
        CHECK(u.t0 % pod::kDecodeStep == 0, "unit start %d", u.t0);
        CHECK(u.prow0 == -1 || (u.prow0 >= 0 && u.prow0 + group <= p.n_partial_rows), "unit partial row %d", u.prow0);
        CHECK(u.q_start == meta[4 * u.req] && u.cache_row == meta[4 * u.req + 3], "unit copy of request %d", u.req);
        keys[{u.req, u.kv_head}] += u.t1 - u.t0;
    }
    for (int r = prm.n_prefill; r < n_req; ++r)
        for (int h = 0; h < prm.n_kv_heads; ++h) {
            const int64_t covered = keys[std::make_pair(r, h)];
            CHECK(covered == meta[4 * r + 2], "decode cover of request %d head %d", r, h);
        }
    CHECK(p.n_dwgs >= 0 && p.n_dwgs <= p.n_cus && p.n_static_seats <= p.n_dwgs, "workers %d seats %d", p.n_dwgs,
          p.n_static_seats);
    CHECK(p.dq_begin[0] == p.n_static_seats * pod::kWavesPerWg, "first queue %d", p.dq_begin[0]);
    for (int q = 0; q < pod::kXcdQueues; ++q)
        CHECK(p.dq_begin[q] <= p.dq_begin[q + 1] && p.dq_begin[q + 1] <= (int)p.dunits.size(), "decode queue %d", q);
    CHECK(p.dq_begin[pod::kXcdQueues] == (int)p.dunits.size(), "last queue %d", p.dq_begin[pod::kXcdQueues]);
    // combine entries and the row list
    for (const pod::CombineEntry &c : p.centries) {
        CHECK(c.n_splits >= 2, "splits %d", c.n_splits);
        CHECK(c.prow0 >= 0 && (int64_t)c.prow0 + (int64_t)(c.n_splits - 1) * c.split_stride + c.n_rows <= p.n_partial_rows,
              "entry partial rows %d", c.prow0);
    }
    CHECK(p.crows.size() % 2 == 0, "row list");
    for (size_t i = 0; i < p.crows.size(); i += 2) {
        CHECK(p.crows[i] >= 0 && p.crows[i] < (int)p.centries.size(), "row list entry %d", p.crows[i]);
        CHECK(p.crows[i + 1] >= 0 && p.crows[i + 1] < p.centries[(size_t)p.crows[i]].n_rows, "row list row %d", p.crows[i + 1]);
    }
    CHECK(p.n_crows_prefill >= 0 && (size_t)p.n_crows_prefill * 2 <= p.crows.size(), "prefill rows %d", p.n_crows_prefill);
    CHECK(p.fused_grid >= 0 && p.fused_grid <= 2 * p.n_cus, "grid %d", p.fused_grid);
    CHECK(p.fused_grid >= p.n_dwgs, "grid %d below the seats %d", p.fused_grid, p.n_dwgs);
    CHECK(p.off_part_ml + (size_t)p.n_partial_rows * 2 * sizeof(float) <= p.ws_bytes, "workspace");
    CHECK(p.p_ratio >= 0 && p.d_ratio >= 0 && p.p_ratio + p.d_ratio > 0, "ratio %d:%d", p.p_ratio, p.d_ratio);
    return true;
}

}  // namespace

int main(int argc, char **argv)
{
    const int n_cases = argc > 1 ? std::atoi(argv[1]) : 400;
    int n_ok = 0, n_rejected = 0;
    for (g_case = 0; g_case < n_cases; ++g_case) {
        pod_attn_params prm{};
        const int hkv = one_of({1, 2, 3, 4, 5, 8, 32});
        const int group = one_of({1, 2, 4, 8, 16});
        prm.n_kv_heads = hkv;
        prm.n_q_heads = hkv * group;
        prm.head_dim = group <= 8 ? one_of({64, 128, 256}) : one_of({64, 128});   // 256 channels: at most 8 heads per K/V head
        prm.dtype = pick(0, 1);
        prm.softmax_scale = 0.1f;
        prm.n_prefill = pick(0, 3);
        prm.n_decode = one_of({0, 1, 2, 7, 33, 200});
        prm.block_size = one_of({0, 0, 16, 32, 48, 256});
        prm.policy = pick(0, 2);
        prm.max_prefill_waves = one_of({0, 0, 1, 2, 64});
        prm.decode_chunk = one_of({0, 0, 16, 100, 512, 4096});
        prm.prefill_split_len = one_of({0, 0, 64, 1000});
        prm.n_compute_units = one_of({256, 256, 8, 1, 304});
        prm.kv_order = pick(0, 1);
        const int n_req = prm.n_prefill + prm.n_decode;
        std::vector<int32_t> meta((size_t)4 * (size_t)std::max(n_req, 1));
        int q_rows = 0, max_len = 1;
        for (int r = 0; r < n_req; ++r) {
            const bool is_p = r < prm.n_prefill;
            const int q_len = is_p ? one_of({1, 5, 64, 130, 700}) : 1;
            const int kv_len = q_len + one_of({0, 0, 3, 500, 5000, 40000}) - (is_p ? 0 : (int)(rnd() % 2) * 0);
            meta[(size_t)4 * r + 0] = is_p ? q_rows : r - prm.n_prefill;
            meta[(size_t)4 * r + 1] = q_len;
            meta[(size_t)4 * r + 2] = kv_len;
            meta[(size_t)4 * r + 3] = r;
            if (is_p) q_rows += q_len;
            max_len = std::max(max_len, kv_len);
        }
        prm.n_cache_rows = std::max(n_req, 1);
        if (prm.block_size > 0) {
            prm.max_blocks_per_seq = (max_len + prm.block_size - 1) / prm.block_size + 1;
            prm.n_blocks = prm.max_blocks_per_seq * std::max(n_req, 1);
        }
        prm.kv_seq_stride = (int64_t)((max_len + 7) / 8 * 8) * prm.n_kv_heads * prm.head_dim;
        // every fifth case is broken on purpose: the planner must refuse it without touching bad memory
        const bool broken = g_case % 5 == 4;
        if (broken) {
            switch (rnd() % 8) {
            case 0: prm.head_dim = 96; break;
            case 1: prm.n_q_heads += 1; break;
            case 2: if (n_req) meta[2] = meta[1] - 1; else prm.dtype = 7; break;
            case 3: prm.softmax_scale = -1.f; break;
            case 4: prm.kv_order = 5; break;
            case 5: if (prm.n_decode) meta[(size_t)4 * prm.n_prefill + 1] = 2; else prm.policy = 9; break;
            case 6: prm.block_size = -16; break;
            default: if (n_req) meta[3] = -1; else prm.n_decode = -1; break;
            }
        }
        pod::Plan plan;
        std::string err;
        const pod_status st = pod::build_plan(prm, meta.data(), prm.n_compute_units, plan, err);
        if (st != POD_OK) {
            if (!broken) {
                std::printf("case %d: a valid batch was refused: %s\n", g_case, err.c_str());
                return 1;
            }
            if (err.empty()) {
                std::printf("case %d: refused without a message\n", g_case);
                return 1;
            }
            ++n_rejected;
            continue;
        }
        if (!check_plan(prm, meta, plan)) return 1;
        ++n_ok;
    }
    std::printf("planner under sanitizers: %d plans checked, %d invalid batches refused\n", n_ok, n_rejected);
    return 0;
}
