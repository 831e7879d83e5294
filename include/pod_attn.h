/*
 * pod_attn.h - C ABI of the MI355X (gfx950) hybrid-batch attention library.
 *
 * One call computes attention for a batch that mixes causal chunked-prefill
 * requests (a chunk of new query tokens over its cached prefix plus itself) and
 * single-token decode requests, all against a KV cache, with both kinds of work
 * running at the same time on the same compute units (paper Section 4: one fused
 * kernel; Section 4.1: each workgroup picks its operation after it has landed on
 * a compute unit).
 *
 * What is computed, per request r with (q_len, kv_len), local query row i, query
 * head h (paper Section 2.1, the attention equation and the paragraph on heads):
 *
 *     pos  = kv_len - q_len + i            absolute position of the query token
 *     kvh  = h / (n_q_heads / n_kv_heads)  K/V head that serves query head h
 *     s_j  = softmax_scale * <Q[r,i,h,:], K[r,j,kvh,:]>        j = 0 .. pos
 *     out[r,i,h,:] = sum_j softmax_j(s) * V[r,j,kvh,:]
 *
 * The new tokens' K/V are already in the cache (kv_len counts them).  A decode
 * request is the case q_len == 1.  Inputs and output are 16-bit floats; scores,
 * the softmax and all sums are fp32 on the GPU.
 *
 * Conventions for every entry point:
 *   - "host" pointers are ordinary CPU memory; "device" pointers are memory of the
 *     HIP device that is current when the call is made.  The library never takes
 *     ownership of a caller buffer and never frees one.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Device work is asynchronous with respect to the host and ordered on `stream`.
 *   - Every function that returns pod_status returns POD_OK or a negative code and
 *     launches nothing when it fails; pod_attn_last_error() gives a message
 *     (thread-local storage, valid until the same thread's next failing call).
 *   - No CPU fallback exists: without a HIP device the compute calls fail.
 */
#ifndef POD_ATTN_H
#define POD_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    POD_OK = 0,
    POD_ERR_INVALID_ARG = -1,   /* null pointer, inconsistent sizes, bad seq_meta      */
    POD_ERR_UNSUPPORTED = -2,   /* head_dim / dtype / group size outside what is built */
    POD_ERR_WORKSPACE = -3,     /* workspace missing or too small                      */
    POD_ERR_HIP = -4            /* a HIP runtime call failed                           */
} pod_status;

typedef enum { POD_F16 = 0, POD_BF16 = 1 } pod_dtype;

/* How pod_attn_forward schedules the two operations. */
typedef enum {
    POD_MODE_FUSED = 0,         /* one launch, roles bound per workgroup at run time (Section 4.1) */
    POD_MODE_SERIAL = 1,        /* prefill kernel, then decode kernel, one stream (Section 3.1)    */
    POD_MODE_STREAMS = 2,       /* the same two kernels on two streams, joined (Section 3.1)       */
    POD_MODE_PREFILL_ONLY = 3,  /* only the prefill rows of `out` are written                      */
    POD_MODE_DECODE_ONLY = 4    /* only the decode rows of `out` are written                       */
} pod_mode;

/* May be OR-ed into `mode`: leave the split-KV partials in the workspace and skip the combine
 * pass, so that a profiler or a pair of events sees the attention kernel alone.  Rows whose
 * work was split are then not written to `out`. */
#define POD_MODE_FLAG_NO_COMBINE 0x100

/* May be OR-ed into POD_MODE_FUSED: launch the fused kernel CTA-parallel, as Section 4.1 prints it
 * (one workgroup per prefill item or per four decode units; each takes its unit's ticket, picks
 * its operation, claims one work id, runs it and leaves), instead of as one resident round of
 * persistent workgroups (Section 4.4's variant, the default).  Same result bit for bit; exists so
 * that the two launch styles can be timed against each other (once the chip's clocks are up the
 * persistent one is level on the MFMA-bound benchmark batch and 6-17 % faster on all others). */
#define POD_MODE_FLAG_CTA_PARALLEL 0x200

/* May be OR-ed into POD_MODE_FUSED: the prefill-heavy occupancy configuration (Section 4.2.2 ships
 * two configurations, with more or fewer resident workgroups per multiprocessor, and picks one per
 * batch).  Instead of the one fused kernel with two workgroups per compute unit, two kernels are
 * started together on the library's two side streams: the prefill kernel held to 208 registers
 * and a light decode kernel of 96 registers and 16 KB of LDS, so that every compute unit holds two
 * prefill workgroups AND one decode workgroup for the whole launch (what places them together is
 * that nothing else fits; the trace records show where each workgroup ran).  Same result within
 * rounding (the decode kernel adds its weights in another order).  Built for head_dim 128 and for
 * contiguous caches or paged ones with power-of-two blocks of at least 16 tokens; otherwise
 * POD_ERR_UNSUPPORTED.  Not chosen automatically: on this chip it ends a prefill-heavy batch
 * 3-8 % sooner when launches are spaced out and 1-3 % sooner in a sustained loop, where the chip
 * clocks down under the power the two kernels draw together, and is slower on decode-bound batches.
 * Also accepted with POD_MODE_PREFILL_ONLY and POD_MODE_DECODE_ONLY, which then run that
 * configuration's prefill or decode kernel alone.  Like POD_MODE_STREAMS it creates streams and
 * events on first use, is not meant for graph capture, and is rejected by pod_attn_forward_static. */
#define POD_MODE_FLAG_PREFILL_HEAVY 0x400

/* Which operation a workgroup takes first on its compute unit (Section 4.1, the two policies). */
typedef enum {
    POD_POLICY_AUTO = 0,        /* proportional, but never more decode than prefill workgroups at the
                                   start: a compute unit seats one decode worker                      */
    POD_POLICY_ALTERNATE = 1,   /* 50:50 - successive workgroups of a unit alternate             */
    POD_POLICY_PROPORTIONAL = 2 /* in the ratio of prefill to decode work of this batch          */
} pod_policy;

/* Order of the two middle dimensions of the cache.  The paper does not fix a cache layout; both
 * orders in use by serving systems are accepted. */
typedef enum {
    POD_KV_TOKEN_MAJOR = 0,     /* [..][token][Hkv][d]: a token's heads lie together               */
    POD_KV_HEAD_MAJOR = 1       /* [..][Hkv][token][d]: a head's tokens lie together               */
} pod_kv_order;

typedef struct {
    int32_t n_prefill;          /* prefill requests (may be 0)                                   */
    int32_t n_decode;           /* decode requests (may be 0)                                    */
    int32_t n_q_heads;          /* Hq                                                            */
    int32_t n_kv_heads;         /* Hkv; Hq % Hkv == 0 and Hq / Hkv <= 16 (<= 8 at head_dim 256)  */
    int32_t head_dim;           /* d: 64, 128 or 256                                             */
    int32_t dtype;              /* pod_dtype of q, k, v and out                                  */
    float   softmax_scale;      /* multiplies Q K^T; must be > 0 (1/sqrt(d) in normal use)       */
    int32_t block_size;         /* tokens per cache block; 0 = contiguous cache                  */
    int32_t max_blocks_per_seq; /* paged: row length of block_table                              */
    int32_t n_cache_rows;       /* contiguous: sequences in the cache; paged: block_table rows   */
    int32_t n_blocks;           /* paged: physical blocks in the cache                           */
    int64_t kv_seq_stride;      /* contiguous: elements between sequences (>= max kv_len*Hkv*d)  */
    int32_t policy;             /* pod_policy                                                    */
    int32_t max_prefill_waves;  /* cap on prefill split-KV (Section 4.2.4): prefill work items
                                   fill at most this many chip-wide rounds; 0 = automatic: 2, or
                                   1 when the decode work puts a worker on every compute unit    */
    int32_t decode_chunk;       /* tokens per decode work unit (split-KV length); 0 = automatic  */
    int32_t prefill_split_len;  /* minimum keys per prefill split; 0 = automatic                 */
    int32_t n_compute_units;    /* 0 = ask the current device (256 on MI355X if none is present) */
    int32_t kv_order;           /* pod_kv_order; with POD_KV_HEAD_MAJOR a contiguous cache needs
                                   kv_seq_stride to be a multiple of Hkv*d (= max_len*Hkv*d)     */
} pod_attn_params;

/* Counts that describe a plan; filled by pod_attn_plan_info. */
typedef struct {
    int32_t n_prefill_items;    /* prefill work items (row block x K/V head x split)             */
    int32_t n_decode_units;     /* decode work units (request x K/V head x split), one per wave  */
    int32_t n_combine;          /* output groups that are merged from split partials             */
    int32_t max_prefill_splits;
    int32_t max_decode_splits;
    int32_t decode_chunk;       /* tokens per decode unit actually chosen                        */
    int32_t prefill_ratio;      /* roles per compute unit, prefill : decode                      */
    int32_t decode_ratio;
    int32_t fused_grid;         /* workgroups of the fused launch (persistent, <= 2 per unit)    */
    int32_t n_compute_units;
    int64_t n_prefill_rows;     /* sum of q_len over prefill requests                            */
    int64_t n_partial_rows;     /* rows of fp32 partial output held in the workspace             */
    int64_t workspace_bytes;
    int32_t prefill_heavy_advised; /* 1 when the batch is one the prefill-heavy configuration is built
                                   for and its prefill work outweighs its decode stream (FLOP time
                                   at the matrix peak above 1.2 x byte time at the HBM peak): the
                                   caller may OR POD_MODE_FLAG_PREFILL_HEAVY into POD_MODE_FUSED  */
    int32_t reserved0;
} pod_attn_plan_info;

typedef struct pod_attn_plan pod_attn_plan;   /* opaque, host memory, owned by the caller */

/*
 * seq_meta: int32 [n_prefill + n_decode][4] = {q_start, q_len, kv_len, cache_row},
 * prefill requests first.
 *   q_start    first row of the request in prefill_q (prefill) / its row in decode_q (decode)
 *   q_len      new query tokens (prefill: >= 1; decode: exactly 1)
 *   kv_len     tokens visible to the request's last query, the new ones included (>= q_len)
 *   cache_row  sequence slot (contiguous cache) or block_table row (paged cache)
 *
 * pod_attn_plan_create: host-only.  Validates params and seq_meta (host pointer) and
 * splits the batch into work items, as the paper does before its launch (Section 4.1:
 * the numbers of prefill and decode CTAs are fixed on the host): prefill row blocks with
 * split-KV capped per Section 4.2.4, decode units of one wavefront each (Section 4.2.3),
 * and the role ratio (Section 4.1).  On success *plan is a new object that the caller
 * releases with pod_attn_plan_destroy.  Needs no GPU when n_compute_units is given.
 */
pod_status pod_attn_plan_create(const pod_attn_params *params, const int32_t *seq_meta_host,
                                pod_attn_plan **plan);
void       pod_attn_plan_destroy(pod_attn_plan *plan);
pod_status pod_attn_plan_info_get(const pod_attn_plan *plan, pod_attn_plan_info *info);

/*
 * Optional execution trace, the evidence for co-location (Section 4.1 wants both operations
 * resident on every multiprocessor).  `trace` is device memory of at least 48 bytes per workgroup
 * of the largest launch (the larger of pod_attn_plan_info.fused_grid and n_prefill_items +
 * (n_decode_units + 3) / 4, the grid of the CTA-parallel launch), or NULL to switch tracing off.  After a forward
 * call, record w of the fused launch holds int32 {hardware unit id, first operation (0 prefill /
 * 1 decode), work items done in the first operation, work items done after switching} followed by
 * three uint64 device timestamps (100 MHz): begin, switch of operation, end, and 8 bytes of
 * padding.  Prefill items are counted per workgroup, decode units per leading wavefront.  The
 * stand-alone kernels write one record per prefill item, then one per decode workgroup.
 */
pod_status pod_attn_plan_set_trace(pod_attn_plan *plan, void *trace, size_t trace_bytes);

/*
 * Optional event log: when each prefill item and each decode unit ran, the evidence for how the
 * two operations overlap in time inside one launch (Section 4.1, Section 5.1).  `log` is 16-byte
 * aligned device memory, or NULL to switch logging off: a 16-byte header whose first uint32 counts
 * the records appended (the caller zeroes it before a forward call), then 32-byte records
 * {int32 kind (0 prefill / 1 decode), int32 item or unit index, int32 hardware unit id,
 * int32 workgroup * 4 + wavefront, uint64 begin, uint64 end} (100 MHz device clock).  Records
 * beyond the capacity (log_bytes - 16) / 32 are counted, not stored.  Logging costs one atomic
 * per item; timings taken with it on are slightly slower.
 */
pod_status pod_attn_plan_set_event_log(pod_attn_plan *plan, void *log, size_t log_bytes);

/* Bytes of device workspace the plan needs (work tables, counters, split partials). */
size_t     pod_attn_workspace_size(const pod_attn_plan *plan);

/*
 * Copy the plan's work tables into `workspace` (device, >= pod_attn_workspace_size bytes,
 * 256-byte aligned) and zero its counters.  Once per batch; the workspace then serves any
 * number of pod_attn_forward calls with this plan (one per layer in a model).  Calls that
 * share a workspace must not overlap in time.  Returns after the copy has completed.
 */
pod_status pod_attn_plan_upload(const pod_attn_plan *plan, void *workspace, size_t workspace_bytes,
                                void *stream);

/*
 * The hybrid-batch attention call (Section 4: prefill and decode attention of one batch in
 * one kernel; rows ordered as in Figure 3, prefill tokens first, then decode tokens).
 *
 * All pointers are device memory:
 *   prefill_q   [sum q_len][Hq][d]           16-bit; may be NULL when n_prefill == 0
 *   decode_q    [n_decode][Hq][d]            16-bit; may be NULL when n_decode == 0
 *   k_cache,    contiguous: [n_cache_rows][max_len][Hkv][d] with kv_seq_stride elements
 *   v_cache                 between sequences;
 *               paged:      [n_blocks][block_size][Hkv][d]
 *               with kv_order = POD_KV_HEAD_MAJOR the two middle dimensions change places:
 *               [n_cache_rows][Hkv][max_len][d] (max_len = kv_seq_stride / (Hkv*d)) and
 *               [n_blocks][Hkv][block_size][d]
 *   seq_meta    device copy of the array given to pod_attn_plan_create
 *   block_table paged: int32 [n_cache_rows][max_blocks_per_seq], entry [row][t / block_size]
 *               is the physical block of token t (token t sits at offset t % block_size);
 *               NULL for a contiguous cache.  Entries past a sequence's last block, cache
 *               slots at positions >= kv_len and unreferenced blocks are never read.
 *   out         [sum q_len + n_decode][Hq][d] 16-bit, prefill rows first, then one row per
 *               decode request in decode_q order; rounded to nearest-even from fp32.
 *   workspace   as prepared by pod_attn_plan_upload with this plan.
 *
 * The 16-bit arrays must be 16-byte aligned (rows are read and written in 16-byte pieces; a
 * contiguous cache also needs kv_seq_stride to be a multiple of 8 elements), else POD_ERR_INVALID_ARG.
 * The device arrays are trusted: a seq_meta that differs from the planned one, or a block
 * table entry outside [0, n_blocks), is undefined behaviour.  `mode` is a pod_mode, optionally OR-ed with
 * the POD_MODE_FLAG_ values above.
 * The call only launches kernels on `stream` (no allocation, no memset, no wait on the host), so
 * in the FUSED, SERIAL and single-operation modes it may be recorded into a HIP graph; the
 * STREAMS mode (and the prefill-heavy configuration) creates two side streams per GPU, kept until the
 * process ends, and three events per plan, destroyed with it, on first use (that first call must not
 * run beside another call on the same plan from a second host thread) and is not meant for capture.
 * Two forward calls that use the same workspace must not overlap in time.
 */
pod_status pod_attn_forward(const void *prefill_q, const void *decode_q,
                            const void *k_cache, const void *v_cache,
                            const int32_t *seq_meta, const int32_t *block_table,
                            void *out,
                            const pod_attn_plan *plan, void *workspace, size_t workspace_bytes,
                            int32_t mode, void *stream);

/*
 * The same call for callers that cannot allocate device memory or be handed a workspace: code
 * under HIP graph capture set-ups that forbid allocation, tight serving loops, harnesses that
 * forbid hipMalloc.  Everything pod_attn_forward keeps in the caller's workspace (counters, work
 * tables, split-KV partials) lives in a fixed array inside the library instead: device memory of
 * POD_ATTN_STATIC_SCRATCH_BYTES bytes that every GPU the library runs on holds from the moment the
 * library's code is loaded there until the process ends.  The call allocates nothing and frees
 * nothing (no hipMalloc, hipFree, stream or event creation): it launches kernels on `stream`, and,
 * whenever the array does not already hold this plan's work tables (the first call with a plan
 * on a GPU, or after a call with another plan there), it first clears the array's counters with a
 * kernel and copies the tables in with hipMemcpyAsync, waiting for those copies.  No
 * pod_attn_plan_upload is needed.  Arguments, results and modes are those of pod_attn_forward,
 * except:
 *   - a plan whose pod_attn_workspace_size exceeds POD_ATTN_STATIC_SCRATCH_BYTES is rejected with
 *     POD_ERR_WORKSPACE (the message gives both numbers) and nothing is launched;
 *   - POD_MODE_STREAMS, and POD_MODE_FUSED with POD_MODE_FLAG_PREFILL_HEAVY, are rejected with
 *     POD_ERR_UNSUPPORTED (they create streams and events).
 * All calls on one GPU share that GPU's array: two calls of this entry point on the same GPU must
 * not overlap in time (not from two streams, not from two host threads); calls on different
 * GPUs are independent.  pod_attn_forward and its workspaces are not affected in any way.
 */
#define POD_ATTN_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
pod_status pod_attn_forward_static(const void *prefill_q, const void *decode_q,
                                   const void *k_cache, const void *v_cache,
                                   const int32_t *seq_meta, const int32_t *block_table,
                                   void *out, const pod_attn_plan *plan, int32_t mode, void *stream);

/*
 * The role rule of the on-device binder (Section 4.1, the scheduling listing), host-callable for
 * tests: the first operation of the workgroup that holds `ticket` (arrivals on its hardware unit
 * before it, counted from 0) on unit `unit`: 0 prefill when (ticket + 2 * unit) mod (p + d) < p,
 * else 1 decode.  Unit u counts from 2u because a unit holds two workgroups of the fused kernel at
 * a time, so that a pattern longer than two is spread over the units; with all arrivals on unit 0
 * this is the listing's own rule (Section 5.4.2: 50 prefill and 100 decode CTAs run P, D, D, ...).
 * The fused kernel calls the same code.  Returns -1 for bad arguments.
 */
int32_t pod_attn_role_for_ticket(int32_t ticket, int32_t prefill_ratio, int32_t decode_ratio, int32_t unit);

/*
 * Host model of one fused launch, for tests: what the workgroups do between landing on a compute
 * unit and leaving it (Section 4.1: the scheme must hold however the hardware places and times
 * the workgroups; Section 4.4: persistent workgroups that loop over work).  No GPU is used.
 *   unit_of_wg[w]  hardware unit id (xcc << 6 | se << 4 | cu, < 1024) workgroup w lands on
 *   order[k]       actor whose next step runs at time k.  Actor 4w is workgroup w's leader, whose
 *                  steps are: take the unit's ticket and pick the first operation; as a prefill
 *                  worker, one claim on the prefill queue it is at (its XCD's queue first, then the
 *                  others; a used-up queue moves it on, after all eight the operation is done); as
 *                  a decode worker, take a seat (workers beyond the plan's seats skip the
 *                  operation).  Actors 4w .. 4w+3 are its wavefronts while it is a decode worker:
 *                  the fixed first unit 4 * seat + v of the first seats without a claim, then one
 *                  claim per step on the decode queue the wavefront is at (same walk over the eight
 *                  queues).  A workgroup switches operation once and then ends.  Entries naming an
 *                  actor that has nothing to do at that moment are skipped; when `order` is used
 *                  up, all unfinished actors run on in turn until the launch has drained.
 * Outputs (host, each may be NULL): first_role[w] 0 prefill / 1 decode; seat_of_wg[w] (untouched if
 * w never asked); item_owner[i] = workgroup that ran prefill item i; unit_owner[u] = actor that ran
 * decode unit u (-1 = nobody).  Returns the number of steps executed, -1 for bad arguments, -2 if
 * any work id was handed out twice.
 */
int32_t pod_attn_simulate_launch(const pod_attn_plan *plan, const int32_t *unit_of_wg, int32_t n_wgs,
                                 const int32_t *order, int32_t n_order, int32_t *first_role,
                                 int32_t *seat_of_wg, int32_t *item_owner, int32_t *unit_owner);

/*
 * Read one row of the plan's work tables (host), for tests:
 *   prefill item: {request, kv_head, first packed row, n packed rows, kv_begin, kv_end,
 *                  first partial row or -1, split index}
 *   decode unit : {request, kv_head, token_begin, token_end, first partial row or -1,
 *                  split index, first query row of the request, cache row of the request}
 * Returns POD_ERR_INVALID_ARG when index is out of range.
 */
pod_status pod_attn_plan_prefill_item(const pod_attn_plan *plan, int32_t index, int32_t out[8]);
/* The prefill item that workgroup `workgroup` of a stand-alone prefill kernel runs (SERIAL, STREAMS,
 * PREFILL_ONLY and the prefill-heavy configuration launch one workgroup per item, and the
 * hardware deals workgroups to the XCDs round-robin): the same items as above in another order,
 * workgroup b taking the next item of queue b % 8, so that a K/V head's tiles are read through the
 * L2 of the XCDs its queue belongs to. */
pod_status pod_attn_plan_prefill_item_of_workgroup(const pod_attn_plan *plan, int32_t workgroup, int32_t out[8]);
pod_status pod_attn_plan_decode_unit(const pod_attn_plan *plan, int32_t index, int32_t out[8]);

/*
 * How the decode units are handed out (host, for tests).  Units [0, begin of queue 0) are the fixed
 * first units of the decode workers: worker w's wavefront v starts with unit 4*w + v and claims
 * nothing for it.  Every other unit sits in one of 8 queues, one per XCD; queue q holds units
 * [*begin, *end), and a wavefront claims from the queue of the XCD it runs on before it tries the
 * others (the virtual decode CTAs of Section 4.2.3 are these units; which multiprocessor runs
 * which of them is decided at run time as in Section 4.1).  Units are sorted longest first inside
 * the fixed range and inside each queue.  Returns POD_ERR_INVALID_ARG when q is not in 0..7.
 */
pod_status pod_attn_plan_decode_queue(const pod_attn_plan *plan, int32_t q, int32_t *begin, int32_t *end);

/*
 * Measurement aids (Section 5.1 reports compute and bandwidth utilisation; these give the two
 * ceilings this GPU actually sustains).  Both enqueue one kernel on `stream`; the caller times it.
 *   pod_attn_probe_hbm_read: reads `bytes` of device memory at `buf` once, fully coalesced.
 *   pod_attn_probe_mfma:     every wavefront of a chip-filling grid issues 4*iters dense fp16 MFMA
 *                            (32x32x16) instructions; *flops_out (host, may be NULL) receives the
 *                            total flop count.
 * `sink` is 16 bytes of device memory that is never written in practice.
 */
pod_status pod_attn_probe_hbm_read(const void *buf, size_t bytes, void *sink, void *stream);
pod_status pod_attn_probe_mfma(int32_t iters, void *sink, double *flops_out, void *stream);

/*
 * What one SIMD overlaps (Section 4.2.1 sizes the tiles by how much vector work runs beside the
 * tensor-core work; this measures the same trade on this chip).  Enqueues one kernel in which
 * every wavefront of `wgs_per_unit` (1 or 2) workgroups of 256 threads per compute unit, i.e. one
 * or two wavefronts per SIMD, runs `iters` rounds of a fixed instruction mix:
 *   0  four dense bf16 32x32x16 matrix instructions
 *   1  the same, each followed by one 2^x
 *   2  each followed by the vector work of one softmax score: 2^x, two multiply-adds, one
 *      two-to-one rounding to bf16, one three-way maximum
 *   3  mix 2 plus one two-element dot product (the weight sum taken over the rounded pairs)
 *   4  each followed by one two-element dot product only
 *   5  a software-pipelined turn, three per round: one 16-byte LDS read, one matrix instruction,
 *      and the softmax work of one score in three stages one turn apart
 *   6  the same turn with two matrix instructions per LDS read and the work of two scores (a
 *      wavefront that holds two row blocks)
 *   7  no matrix instruction: eight independent multiply-adds per round
 *   8  no matrix instruction: eight independent 2^x per round
 * *matrix_ops_per_wave (host, may be NULL) receives the matrix instructions one wavefront issued
 * (variants 7 and 8: the vector instructions);
 * the caller times the kernel.  `sink`: 4 writable bytes of device memory, never written in
 * practice.  Returns POD_ERR_INVALID_ARG for an unknown variant or bad arguments.
 */
pod_status pod_attn_probe_issue(int32_t variant, int32_t iters, int32_t wgs_per_unit, void *sink,
                                double *matrix_ops_per_wave, void *stream);

/*
 * The co-location experiment of Section 3.3 (Figure 7), independent of attention: a compute-bound
 * operation (n_compute_items workgroups' worth of multiply-add loops, compute_iters rounds each)
 * and a memory-bound one (c = a + b over n_memory_items chunks of bytes_per_item bytes per array),
 * launched as
 *   variant 0: the compute operation alone          variant 1: the memory operation alone
 *   variant 2: one kernel, operation chosen by workgroup index (compute first)
 *   variant 3: one kernel, operation bound at run time per compute unit as in Section 4.1
 *              (ticket from that unit's counter, alternate operations, claim the next item).
 * a, b, c: device arrays of n_memory_items * bytes_per_item bytes (bytes_per_item a multiple of
 * 16); counters: 4104 bytes of device memory, needed by variant 3 only, which clears them on the
 * stream itself (with a memset: do not capture this call in a graph); sink: 4 writable bytes.
 * Serial execution is variants 0 and 1 on one stream, "streams" the same two on two streams.
 * Asynchronous on `stream`.  Returns POD_ERR_INVALID_ARG for bad arguments.
 */
pod_status pod_attn_probe_colocation(int32_t variant, const void *a, const void *b, void *c,
                                     size_t bytes_per_item, int32_t n_memory_items,
                                     int32_t n_compute_items, int32_t compute_iters, void *counters,
                                     void *sink, void *stream);

const char *pod_attn_last_error(void);
const char *pod_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* POD_ATTN_H */
