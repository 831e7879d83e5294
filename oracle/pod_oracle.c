/*
 * fp64 CPU oracle for hybrid-batch attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the GPU library is
 * compared against; nothing in the product path may call it.  It shares no
 * code, header, table or helper with the HIP implementation.
 *
 * What it computes (paper Section 2.1, the attention equation):
 *     Attention(Q, K, V) = softmax(Q K^T * scale) V
 * where Q holds the tokens being processed now and K/V hold every token of the
 * sequence seen so far (Section 2.1).  A prefill chunk of q_len new tokens
 * attends over the cache of all earlier chunks plus itself (Sections 2.1 and
 * 5.2, chunked prefill); a decode request is the case q_len == 1 (Section
 * 2.1: one output token per request per iteration).  Query heads are split
 * into groups, each group served by one K/V head (Section 2.1, the sentence
 * on query heads and K/V heads; Section 4.2.1 gives the group sizes 2-8).
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - "scale" is passed in as a multiplier of Q K^T (1/sqrt(head_dim) in use).
 *   - Causal alignment is bottom-right: local query row i of a request with
 *     (q_len, kv_len) sits at absolute position pos = kv_len - q_len + i and
 *     sees keys 0..pos inclusive; the chunk's own K/V are already cached.
 *   - Query head h reads K/V head h / (Hq / Hkv) (contiguous groups).
 *   - Cache layouts: contiguous [seq][token][Hkv][d] with a per-sequence
 *     stride, or paged [block][block_size][Hkv][d] resolved through
 *     block_table[cache_row][token / block_size]; in the head-major variant of
 *     either, the token and head dimensions change places.
 *
 * Method: the plain definition, written out.  Two-pass softmax (all scores,
 * then their maximum, then the weights), no tiling, no online rescaling, no
 * split/merge.  Inputs are the 16-bit values the GPU sees, widened exactly to
 * double; every operation is in double; the output stays in double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* IEEE binary16 bit pattern -> double, exactly. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)mant, -24);               /* subnormal or zero */
    else if (expo == 31)
        v = mant ? NAN : INFINITY;
    else
        v = ldexp((double)(mant | 0x400), expo - 25);
    return sign ? -v : v;
}

/* bfloat16 bit pattern -> double, exactly (bfloat16 is the top half of binary32). */
static double bfloat_bits_to_double(uint16_t b)
{
    uint32_t w = (uint32_t)b << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* Exposed so that a test can pin the widening against numpy's own. */
double pod_oracle_widen(int dtype, uint16_t bits)
{
    return dtype == ORACLE_BF16 ? bfloat_bits_to_double(bits) : half_bits_to_double(bits);
}

int pod_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

typedef struct {
    const uint16_t *k_cache, *v_cache;
    const int32_t *block_table;
    int n_kv_heads, head_dim, block_size, max_blocks_per_seq;
    int64_t kv_seq_stride;
    int head_major;
} cache_view;

/* Element offset of token `t` of cache row `row`, K/V head `kvh`, channel 0.
 * The cache is a 4-d array [outer][n_mid0][n_mid1][d]: `outer` is the sequence or
 * the physical block, `slot` the token's place inside it and `n_slots` its
 * capacity in tokens; (mid0, mid1) = (slot, head) or, head-major, (head, slot). */
static int64_t cache_offset(const cache_view *c, int row, int t, int kvh)
{
    int64_t outer_elems, slot, n_slots, outer;
    if (c->block_size > 0) {
        outer = c->block_table[(int64_t)row * c->max_blocks_per_seq + t / c->block_size];
        slot = t % c->block_size;
        n_slots = c->block_size;
        outer_elems = n_slots * c->n_kv_heads * c->head_dim;
    } else {
        outer = row;
        slot = t;
        outer_elems = c->kv_seq_stride;
        n_slots = c->kv_seq_stride / ((int64_t)c->n_kv_heads * c->head_dim);
    }
    if (c->head_major)
        return outer * outer_elems + ((int64_t)kvh * n_slots + slot) * c->head_dim;
    return outer * outer_elems + (slot * c->n_kv_heads + kvh) * c->head_dim;
}

/*
 * seq_meta: int32 [n_prefill + n_decode][4] = {q_start, q_len, kv_len, cache_row},
 * prefill requests first.  Output rows: prefill rows (in q_start order) first,
 * then one row per decode request at n_prefill_rows + q_start.
 *
 * rows == NULL : compute every output row; out is [n_rows_total][Hq][d].
 * rows != NULL : compute only the listed global output rows (n_rows of them);
 *                out is [n_rows][Hq][d] in list order.
 * Returns 0, or a negative number for an argument that makes no sense.
 */
int pod_oracle_attention(const uint16_t *prefill_q, const uint16_t *decode_q,
                         const uint16_t *k_cache, const uint16_t *v_cache,
                         const int32_t *seq_meta, const int32_t *block_table,
                         int n_prefill, int n_decode,
                         int n_q_heads, int n_kv_heads, int head_dim, int dtype,
                         double softmax_scale,
                         int block_size, int max_blocks_per_seq, int64_t kv_seq_stride,
                         int head_major,
                         const int32_t *rows, int64_t n_rows,
                         double *out)
{
    if (n_prefill < 0 || n_decode < 0 || n_q_heads <= 0 || n_kv_heads <= 0 ||
        head_dim <= 0 || n_q_heads % n_kv_heads != 0)
        return -1;
    if (dtype != ORACLE_F16 && dtype != ORACLE_BF16)
        return -2;

    const int n_req = n_prefill + n_decode;
    const int group = n_q_heads / n_kv_heads;
    int64_t n_prefill_rows = 0;
    int max_kv = 1;
    for (int r = 0; r < n_req; ++r) {
        const int32_t *m = seq_meta + 4 * r;
        if (m[1] < 0 || m[2] < m[1] || (m[1] > 0 && m[2] <= 0))
            return -3;
        if (r >= n_prefill && m[1] != 1)
            return -4;
        if (r < n_prefill && m[0] + m[1] > n_prefill_rows)
            n_prefill_rows = m[0] + m[1];
        if (m[2] > max_kv)
            max_kv = m[2];
    }
    const int64_t n_total = n_prefill_rows + n_decode;

    /* For each global output row: which request it belongs to and its local index. */
    int32_t *row_req = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_total ? n_total : 1));
    int32_t *row_loc = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_total ? n_total : 1));
    if (!row_req || !row_loc) { free(row_req); free(row_loc); return -5; }
    for (int64_t i = 0; i < n_total; ++i) row_req[i] = -1;
    for (int r = 0; r < n_req; ++r) {
        const int32_t *m = seq_meta + 4 * r;
        for (int i = 0; i < m[1]; ++i) {
            int64_t g = (r < n_prefill) ? (int64_t)m[0] + i : n_prefill_rows + m[0];
            if (g < 0 || g >= n_total) { free(row_req); free(row_loc); return -6; }
            row_req[g] = r;
            row_loc[g] = i;
        }
    }

    double *widen = (double *)malloc(sizeof(double) * 65536);
    if (!widen) { free(row_req); free(row_loc); return -5; }
    for (int b = 0; b < 65536; ++b)
        widen[b] = pod_oracle_widen(dtype, (uint16_t)b);

    cache_view cv = { k_cache, v_cache, block_table, n_kv_heads, head_dim,
                      block_size, max_blocks_per_seq, kv_seq_stride, head_major != 0 };
    const int64_t n_work = (rows ? n_rows : n_total) * n_q_heads;
    int failed = 0;

#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)max_kv);
        double *qrow = (double *)malloc(sizeof(double) * (size_t)head_dim);
        if (!score || !qrow) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 4)
            for (int64_t w = 0; w < n_work; ++w) {
                const int64_t slot = w / n_q_heads;
                const int h = (int)(w % n_q_heads);
                const int64_t g = rows ? rows[slot] : slot;
                double *o = out + (slot * n_q_heads + h) * head_dim;
                if (g < 0 || g >= n_total || row_req[g] < 0) {
                    for (int c = 0; c < head_dim; ++c) o[c] = NAN;
                    continue;
                }
                const int r = row_req[g];
                const int i = row_loc[g];
                const int32_t *m = seq_meta + 4 * r;
                const int q_len = m[1], kv_len = m[2], cache_row = m[3];
                const int pos = kv_len - q_len + i;        /* last visible key */
                const int kvh = h / group;

                const uint16_t *qsrc = (r < n_prefill)
                    ? prefill_q + (((int64_t)m[0] + i) * n_q_heads + h) * head_dim
                    : decode_q + ((int64_t)m[0] * n_q_heads + h) * head_dim;
                for (int c = 0; c < head_dim; ++c) qrow[c] = widen[qsrc[c]];

                /* pass 1: scores s_j = scale * <q, k_j>, j = 0..pos */
                double smax = -INFINITY;
                for (int j = 0; j <= pos; ++j) {
                    const uint16_t *kr = k_cache + cache_offset(&cv, cache_row, j, kvh);
                    double dot = 0.0;
                    for (int c = 0; c < head_dim; ++c) dot += qrow[c] * widen[kr[c]];
                    score[j] = softmax_scale * dot;
                    if (score[j] > smax) smax = score[j];
                }
                /* pass 2: weights and their sum */
                double wsum = 0.0;
                for (int j = 0; j <= pos; ++j) {
                    score[j] = exp(score[j] - smax);
                    wsum += score[j];
                }
                /* pass 3: weighted sum of the V rows, then normalise */
                for (int c = 0; c < head_dim; ++c) o[c] = 0.0;
                for (int j = 0; j <= pos; ++j) {
                    const uint16_t *vr = v_cache + cache_offset(&cv, cache_row, j, kvh);
                    const double wj = score[j];
                    for (int c = 0; c < head_dim; ++c) o[c] += wj * widen[vr[c]];
                }
                for (int c = 0; c < head_dim; ++c) o[c] /= wsum;
            }
        }
        free(score);
        free(qrow);
    }

    free(widen);
    free(row_req);
    free(row_loc);
    return failed ? -5 : 0;
}
