// Structures shared by the host planner and the gfx950 kernels.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define POD_HD __host__ __device__
#else
#define POD_HD
#endif

namespace pod {

constexpr int kWaveSize = 64;
constexpr int kWgThreads = 256;            // 4 wavefronts per workgroup, one per SIMD
constexpr int kWavesPerWg = 4;
constexpr int kDecodeStep = 16;            // decode units are cut at multiples of this many keys
// Shape of a prefill work item by head dimension.  Up to 128 channels a wavefront owns 32 packed
// (token, head-in-group) query rows and all output channels, a workgroup 128 rows, and K/V tiles
// hold 64 keys.  At 256 channels the accumulators and queries of 32 rows no longer fit a
// wavefront that shares its SIMD with another one, so two wavefronts share a row group: both
// compute its scores, each owns half of the output channels; a workgroup then covers 64 rows, and
// tiles hold 32 keys so that the four tile buffers still take 64 KB of LDS.
POD_HD constexpr int prefill_item_rows(int head_dim) { return head_dim == 256 ? 64 : 128; }
POD_HD constexpr int prefill_kv_tile(int head_dim) { return head_dim == 256 ? 32 : 64; }
// Keys per decode step of one wavefront: a step's K and V rows are one slot of the register ring
// (head_dim / 4 registers at 16 keys), which at 256 channels is halved to keep two slots.
POD_HD constexpr int decode_step_keys(int head_dim) { return head_dim == 256 ? 8 : 16; }
constexpr int kMaxGroup256 = 8;            // query heads per K/V head at head_dim 256 (the decode worker's query buffers)
constexpr int kMaxGroup = 16;              // query heads per K/V head a decode unit can hold
constexpr int kXcdQueues = 8;               // work is queued per XCD (one L2 each); a queue's counter is claimed mostly from its own XCD
constexpr int kSlotsPerUnit = 2;            // resident workgroups per compute unit (register and LDS budget)
constexpr int kNullClaimLines = 512;       // power of two, at least the number of resident workgroups
constexpr int kCuSlots = 1024;             // hardware unit ids are sparse: (xcc << 6 | se << 4 | cu) < 1024

enum Role : int { kPrefill = 0, kDecode = 1, kNone = -1 };

// Cache layouts the kernels are specialised for: contiguous; paged with a power-of-two block size
// of at least 16 and a power-of-two number of bytes per token (a 16-key step then lies in one
// block, found with one scalar lookup, and addresses need shifts only); paged, any.
enum Layout : int { kLayoutContiguous = 0, kLayoutPaged16 = 1, kLayoutPagedAny = 2 };

// One prefill work item: a block of packed query rows of one K/V head over a key range.
// Packed row R of a request stands for token R / group, query head kv_head * group + R % group,
// so that the heads sharing a K/V head also share each staged K/V tile (Section 4.2.1 notes the
// query tile grows by the group size under grouped-query attention).
struct PrefillItem {
    int32_t req, kv_head, row0, n_rows;
    int32_t kv_begin, kv_end;              // keys [kv_begin, kv_end); causal limit applied inside
    int32_t prow0;                         // first partial row, or -1 when the item writes `out`
    int32_t split;
};

// One decode work unit: all query heads of one K/V head of one request over a token range.
// One wavefront runs it (the "virtual CTA" of Section 4.2.3).
struct DecodeUnit {
    int32_t req, kv_head, t0, t1;
    int32_t prow0;                         // first partial row (group rows), or -1
    int32_t split;
    int32_t q_start, cache_row;            // copied from the request: a unit starts with one lookup
};

// One group of output rows merged from split partials.
struct CombineEntry {
    int32_t kind;                          // kPrefill or kDecode
    int32_t req, kv_head, row0, n_rows;
    int32_t n_splits, prow0, split_stride; // partial row of split s, row r: prow0 + s*split_stride + r
    int32_t q_start, q_len;                // copied from the request, so the merge needs no second lookup
    int32_t pad0, pad1;
};

// Counters at the head of the device workspace.  All zero between launches: the last
// workgroup of a fused launch clears them.
struct WsHeader {
    // Per compute unit: workgroups that have arrived on it so far in this launch (the ticket of
    // Section 4.1's listing).
    uint32_t cu_state[kCuSlots];
    uint32_t next_item[2];                 // [kDecode]: next decode seat
    uint32_t done;                         // workgroups that have finished
    uint32_t pad0;
    uint32_t next_pitem_xcd[kXcdQueues];   // next prefill item of each per-XCD queue (offset inside the queue)
    uint32_t pad[52];
    // Next decode unit of each per-XCD queue (offset inside the queue), claimed by wavefronts.
    // One 128-byte line per counter, so the eight hot words are served by different channels.
    uint32_t next_dunit_xcd[kXcdQueues][32];
    // Words that decode wavefronts add zero to in the turns in which they claim nothing (one
    // line per workgroup; see the decode worker).  Always zero.
    uint32_t null_claim[kNullClaimLines][32];
};

// Which operation the workgroup holding `ticket` on hardware unit `unit` starts with: the ticket
// rule of Section 4.1 (ticket mod (p + d) < p means prefill).  A unit holds only kSlotsPerUnit
// workgroups at a time, so its own tickets would never get past the first entries of a longer
// pattern; unit u therefore counts from kSlotsPerUnit * u, which spreads the pattern over the
// chip (4:1 puts a decode workgroup on every fifth slot; 1:1 still gives every unit one of each).
// The workgroups of the fused kernel arrive together and stay until the work is done, so the
// ticket alone decides: the split does not depend on which of two simultaneous arrivals is seen
// first, and there is no departure to account for.
POD_HD inline int role_for_ticket(uint32_t ticket, int p, int d, int unit = 0)
{
    const int t = (int)(ticket & 0xfffffu) + kSlotsPerUnit * unit;
    return (t % (p + d)) < p ? kPrefill : kDecode;
}

// Optional execution trace: where each workgroup of an attention kernel ran, which operation it
// took first, when it switched to the other one and how many work items it processed in each.
struct TraceRecord {
    int32_t cu;                            // hardware unit id (xcc << 6 | se << 4 | cu)
    int32_t first_role;                    // kPrefill or kDecode
    int32_t n_first, n_second;             // items done in the first role, then in the other one
    uint64_t t_begin, t_switch, t_end;     // constant-rate device clock (100 MHz)
    uint64_t pad;
};

// Optional event log: one record per prefill item (written by the workgroup) and per decode unit
// (written by the wavefront).  The log starts with a 16-byte header whose first word counts the
// records appended so far; records beyond the capacity are counted but not stored.
struct EventRecord {
    int32_t kind;                          // kPrefill or kDecode
    int32_t item;                          // prefill item or decode unit index
    int32_t cu;                            // hardware unit id
    int32_t wg;                            // workgroup index * 4 + wavefront
    uint64_t t_begin, t_end;               // constant-rate device clock (100 MHz)
};

// Everything a kernel needs; passed by value.
struct KernelArgs {
    const void *prefill_q, *decode_q, *k_cache, *v_cache;
    const int32_t *seq_meta, *block_table;
    void *out;
    const PrefillItem *pitems;
    const PrefillItem *pitems_by_wg;       // the same items in workgroup order, for the kernels that run item blockIdx.x
    const DecodeUnit *dunits;
    const CombineEntry *centries;
    const int32_t *crows;                  // [n_crows][2] = (combine entry, row inside it): one merged output row each
    float *part_o;                         // [n_partial_rows][d]  un-normalised fp32 output
    float *part_ml;                        // [n_partial_rows][2]  running max (log2 domain), weight sum
    WsHeader *hdr;
    TraceRecord *trace;                    // optional: one record per workgroup of the attention kernels
    uint32_t *evlog;                       // optional: event log (16-byte header, then EventRecords)
    uint32_t evlog_cap;                    // records the event log can hold
    int64_t kv_seq_stride;
    // Cache strides in elements, the same three for the token-major and the head-major order:
    // between consecutive tokens of one head, between the heads of a sequence (or of a block), and
    // between blocks of a paged cache.
    int64_t head_stride, block_elems;
    int32_t tok_stride;
    int32_t n_prefill, n_q_heads, n_kv_heads, group;
    int32_t block_size, max_blocks_per_seq;
    int32_t bs_shift;                      // log2(block_size) when it is a power of two, else -1
    int32_t n_crows;
    int32_t n_pitems, n_dunits, n_dwgs, n_combine;   // n_dwgs: decode worker workgroups
    int32_t n_prefill_rows;
    int32_t fused_grid;
    int32_t pq_begin[kXcdQueues + 1];      // prefill queue q holds items pq_begin[q] .. pq_begin[q+1]-1
    const int32_t *dq_begin;               // [kXcdQueues + 1]: decode queue q holds units dq_begin[q] .. dq_begin[q+1]-1
    int32_t n_static_seats;                // decode seats that start with four fixed units (units 0 .. 4*seats-1)
    int32_t n_dctas;                       // decode workgroups of the CTA-parallel launch: ceil(n_dunits / 4)
    int32_t single_unit;                   // CTA-parallel launch: a decode wavefront runs its fixed unit and stops
    int32_t p_ratio, d_ratio;
    float scale_log2;                      // softmax_scale * log2(e)
};

}  // namespace pod
