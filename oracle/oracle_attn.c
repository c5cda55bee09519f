/*
 * CPU oracle for paged decode attention and log-sum-exp merging.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64.  Nothing in the GPU library
 * includes, links or calls this file, and this file uses nothing of the GPU
 * library.  It exists so the GPU results can be checked against the plain
 * definition of the operation.
 *
 * What is computed (paper, Background, "Attention computation", Eq. 1): for a
 * decoding request only the last token's query q takes part, against all
 * cached keys and values:
 *
 *     Attention(q, K, V) = softmax(q K^T / sqrt(d_k)) V .
 *
 * The context of a decoding request counts the current token as well
 * (latency-model section, definition of the decode load c_DA as the sum of
 * l_j + 1), so a context of one token is legal.
 *
 * The KV cache is paged (the paper builds on a paged-attention engine and
 * gives no page format).  This build's format: pool[page][kv_head][slot][d],
 * 16-token pages, logical token t of sequence i lives in page
 * block_table[i][t / bs], slot t % bs.  Query head j reads kv head j / G with
 * G = num_q_heads / num_kv_heads.
 *
 * A *partial* is the same attention restricted to a token range R of the
 * context, returned with LSE(R) = ln sum_{t in R} exp(s_t), s_t being the
 * scaled logit.  The paper says only that CPU threads compute partial loads
 * and aggregate intermediate results (System Implementation, CPU Attention);
 * the aggregation rule used here is the exact identity of Eq. 1 over a
 * disjoint union of ranges:
 *
 *     O = sum_p w_p O_p / sum_p w_p,  w_p = exp(LSE_p - max_p LSE_p),
 *     LSE = max_p LSE_p + ln sum_p w_p.
 *
 * Conventions where the paper is silent: an empty range gives O = 0 and
 * LSE = -inf; such a partial has weight zero in a merge; if every partial of
 * a row is empty the merged row is O = 0, LSE = -inf.
 *
 * Every function below is pinned by tests that do not go through this file:
 * dense numpy/scipy brute force, a library softmax-attention routine, closed
 * forms (identical keys, zero query, single token, dominant key, logit shift)
 * and the split = unsplit identity.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* exact widening of one stored element to double */
static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/* element offset of (sequence seq, logical token t, kv head h, dim 0) in a pool */
static int64_t token_offset(const int32_t *block_table, int max_blocks, int seq, int t,
                            int h, int hkv, int bs, int d)
{
    int64_t page = block_table[(int64_t)seq * max_blocks + t / bs];
    int slot = t % bs;
    return ((page * hkv + h) * bs + slot) * (int64_t)d;
}

/*
 * Partial attention for a list of work items.  Item n is (sequence, query
 * head, begin, end): attention of q[seq][head] over logical tokens
 * [begin, end).  Two passes: all logits, their maximum, then the exponentials.
 *
 *   q          [batch, hq, d]                     dtype
 *   k_pool     [num_blocks, hkv, bs, d]           dtype
 *   v_pool     same
 *   block_table[batch, max_blocks] int32
 *   items      [n_items, 4] int32 (seq, head, begin, end)
 *   out_o      [n_items, d] double  (normalised within the range)
 *   out_lse    [n_items]    double  (natural log; -inf for an empty range)
 * Returns 0, or -1 if scratch memory could not be obtained.
 */
int oracle_paged_attn(int hq, int hkv, int d, int bs, int max_blocks, int dtype, double scale,
                      const void *q, const void *k_pool, const void *v_pool,
                      const int32_t *block_table, int64_t n_items, const int32_t *items,
                      double *out_o, double *out_lse, int n_threads)
{
    int group = hq / hkv;
    int failed = 0;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
    for (int64_t n = 0; n < n_items; ++n) {
        int seq = items[4 * n + 0], head = items[4 * n + 1];
        int begin = items[4 * n + 2], end = items[4 * n + 3];
        int h = head / group;
        double *o = out_o + n * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        if (end <= begin) {
            out_lse[n] = -INFINITY;
            continue;
        }
        int len = end - begin;
        double *s = (double *)malloc(sizeof(double) * (size_t)len);
        if (!s) {
#pragma omp atomic write
            failed = 1;
            out_lse[n] = NAN;
            continue;
        }
        int64_t qoff = ((int64_t)seq * hq + head) * d;
        /* pass 1: scaled logits s_t = scale * <q, k_t>, and their maximum */
        double m = -INFINITY;
        for (int t = begin; t < end; ++t) {
            int64_t koff = token_offset(block_table, max_blocks, seq, t, h, hkv, bs, d);
            double dot = 0.0;
            for (int c = 0; c < d; ++c)
                dot += load_elem(q, qoff + c, dtype) * load_elem(k_pool, koff + c, dtype);
            s[t - begin] = scale * dot;
            if (s[t - begin] > m) m = s[t - begin];
        }
        /* pass 2: weights exp(s_t - m), their sum Z, weighted sum of values */
        double z = 0.0;
        for (int t = begin; t < end; ++t) {
            double w = exp(s[t - begin] - m);
            int64_t voff = token_offset(block_table, max_blocks, seq, t, h, hkv, bs, d);
            z += w;
            for (int c = 0; c < d; ++c) o[c] += w * load_elem(v_pool, voff + c, dtype);
        }
        for (int c = 0; c < d; ++c) o[c] /= z;
        out_lse[n] = m + log(z);
        free(s);
    }
    return failed ? -1 : 0;
}

/*
 * Merge of partials.  Output row r combines partial rows
 * offsets[r] .. offsets[r+1]-1 (CSR) of part_o [n_part, d] / part_lse [n_part].
 */
void oracle_merge(int64_t n_rows, int d, const int64_t *offsets, const double *part_o,
                  const double *part_lse, double *out_o, double *out_lse)
{
    for (int64_t r = 0; r < n_rows; ++r) {
        double *o = out_o + r * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        double m = -INFINITY;
        for (int64_t p = offsets[r]; p < offsets[r + 1]; ++p)
            if (part_lse[p] > m) m = part_lse[p];
        if (m == -INFINITY) {            /* no partial carries any weight */
            out_lse[r] = -INFINITY;
            continue;
        }
        double wsum = 0.0;
        for (int64_t p = offsets[r]; p < offsets[r + 1]; ++p) {
            if (part_lse[p] == -INFINITY) continue;
            double w = exp(part_lse[p] - m);
            wsum += w;
            for (int c = 0; c < d; ++c) o[c] += w * part_o[p * d + c];
        }
        for (int c = 0; c < d; ++c) o[c] /= wsum;
        out_lse[r] = m + log(wsum);
    }
}

/*
 * Copy the K and V rows of logical tokens [begin, end) of one sequence, all kv
 * heads, out of the pools: k_out/v_out [end-begin, hkv, d] raw elements.
 */
void oracle_gather_kv(int hkv, int d, int bs, int max_blocks, int elem_bytes,
                      const void *k_pool, const void *v_pool, const int32_t *block_table,
                      int seq, int begin, int end, void *k_out, void *v_out)
{
    size_t row = (size_t)d * (size_t)elem_bytes;
    for (int t = begin; t < end; ++t)
        for (int h = 0; h < hkv; ++h) {
            int64_t src = token_offset(block_table, max_blocks, seq, t, h, hkv, bs, d);
            size_t dst = ((size_t)(t - begin) * hkv + h) * row;
            memcpy((char *)k_out + dst, (const char *)k_pool + (size_t)src * elem_bytes, row);
            memcpy((char *)v_out + dst, (const char *)v_pool + (size_t)src * elem_bytes, row);
        }
}

/*
 * KV-cache data movement (plain copies).  The decode context counts the token being decoded (latency-
 * model section: l_j + 1), so its k, v enter the paged cache before attention; a request's KV moves
 * between GPU and CPU memory as whole pages (KV cache management).
 *
 * oracle_kv_append: row (seq i, kv head h) of k_new/v_new [batch, hkv, d] goes to page
 * block_table[i][pos/bs], slot pos%bs, pos = positions[i]; nothing is written for a position outside
 * [0, max_blocks*bs) or a table entry outside [0, num_blocks).
 */
void oracle_kv_append(int batch, int hkv, int d, int bs, int max_blocks, int64_t num_blocks, int elem_bytes,
                      void *k_pool, void *v_pool, const int32_t *block_table,
                      const void *k_new, const void *v_new, const int32_t *positions)
{
    size_t row = (size_t)d * (size_t)elem_bytes;
    for (int i = 0; i < batch; ++i) {
        int pos = positions[i];
        if (pos < 0 || pos / bs >= max_blocks) continue;
        int64_t page = block_table[(int64_t)i * max_blocks + pos / bs];
        if (page < 0 || page >= num_blocks) continue;
        for (int h = 0; h < hkv; ++h) {
            size_t dst = ((size_t)((page * hkv + h) * bs + pos % bs)) * row;
            size_t src = ((size_t)i * hkv + h) * row;
            memcpy((char *)k_pool + dst, (const char *)k_new + src, row);
            memcpy((char *)v_pool + dst, (const char *)v_new + src, row);
        }
    }
}

/*
 * oracle_kv_pages: to_pool = 0 copies pages page_ids[0..n) of both pools into staging buffers
 * [n, hkv, bs, d] (ids outside [0, num_blocks) give zero pages); to_pool = 1 copies the staging pages
 * back into the pools (such ids are skipped).
 */
void oracle_kv_pages(int hkv, int d, int bs, int64_t num_blocks, int elem_bytes, void *k_pool, void *v_pool,
                     const int32_t *page_ids, int64_t n, void *k_stage, void *v_stage, int to_pool)
{
    size_t page_bytes = (size_t)hkv * bs * d * elem_bytes;
    for (int64_t s = 0; s < n; ++s) {
        int64_t page = page_ids[s];
        int ok = page >= 0 && page < num_blocks;
        char *ks = (char *)k_stage + (size_t)s * page_bytes, *vs = (char *)v_stage + (size_t)s * page_bytes;
        if (to_pool) {
            if (!ok) continue;
            memcpy((char *)k_pool + (size_t)page * page_bytes, ks, page_bytes);
            memcpy((char *)v_pool + (size_t)page * page_bytes, vs, page_bytes);
        } else if (ok) {
            memcpy(ks, (char *)k_pool + (size_t)page * page_bytes, page_bytes);
            memcpy(vs, (char *)v_pool + (size_t)page * page_bytes, page_bytes);
        } else {
            memset(ks, 0, page_bytes);
            memset(vs, 0, page_bytes);
        }
    }
}

/*
 * Row queues and residual store (System Implementation: CPU Attention queue, Residual management).
 * A queue is a ring of `capacity` rows with head / tail counters in state[0] / state[1]; counter value c
 * lives in slot c % capacity.  Push appends all n rows at the tail or, if they do not all fit, none;
 * pop takes up to max_rows rows from the head, oldest first.  Both return the number of rows moved.
 */
int oracle_queue_push(void *data, int32_t *tags, uint32_t *state, int capacity, int row_bytes,
                      const void *rows, const int32_t *row_tags, int n_rows)
{
    uint32_t head = state[0], tail = state[1];
    if ((tail - head) + (uint32_t)n_rows > (uint32_t)capacity) return 0;
    for (int r = 0; r < n_rows; ++r) {
        uint32_t slot = (tail + (uint32_t)r) % (uint32_t)capacity;
        memcpy((char *)data + (size_t)slot * row_bytes, (const char *)rows + (size_t)r * row_bytes, (size_t)row_bytes);
        if (tags) tags[slot] = row_tags ? row_tags[r] : 0;
    }
    state[1] = tail + (uint32_t)n_rows;
    return n_rows;
}

int oracle_queue_pop(const void *data, const int32_t *tags, uint32_t *state, int capacity, int row_bytes,
                     void *rows_out, int32_t *tags_out, int max_rows)
{
    uint32_t head = state[0], tail = state[1];
    uint32_t n = tail - head;
    if (n > (uint32_t)max_rows) n = (uint32_t)max_rows;
    for (uint32_t r = 0; r < n; ++r) {
        uint32_t slot = (head + r) % (uint32_t)capacity;
        memcpy((char *)rows_out + (size_t)r * row_bytes, (const char *)data + (size_t)slot * row_bytes, (size_t)row_bytes);
        if (tags_out) tags_out[r] = tags ? tags[slot] : 0;
    }
    state[0] = head + n;
    return (int)n;
}

/* Residual store: rows to / from slots slot_ids[r]; ids outside [0, n_slots) are skipped / read as zero. */
void oracle_store_rows(void *store, int64_t n_slots, int row_bytes, const int32_t *slot_ids, int n_rows,
                       void *rows, int save)
{
    for (int r = 0; r < n_rows; ++r) {
        int64_t slot = slot_ids[r];
        int ok = slot >= 0 && slot < n_slots;
        char *row = (char *)rows + (size_t)r * row_bytes;
        if (save) {
            if (ok) memcpy((char *)store + (size_t)slot * row_bytes, row, (size_t)row_bytes);
        } else if (ok) {
            memcpy(row, (char *)store + (size_t)slot * row_bytes, (size_t)row_bytes);
        } else {
            memset(row, 0, (size_t)row_bytes);
        }
    }
}
