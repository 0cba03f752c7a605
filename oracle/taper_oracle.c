/*
 * CPU oracle for decode-step attention over a paged KV cache whose parallel
 * branches share their request's prefix pages.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the GPU library must compute.  It shares no code with the HIP path and
 * must never be called from it; only the tests, the smoke check and the
 * benchmark's "cpu_baseline" leg may use it.
 *
 * What is computed (paper §3.1, visibility rule; §1/§2.3, one new token per
 * admitted sequence per decode step): for every admitted sequence s -- a
 * serial request or one branch of a parallel phase -- and every query head h,
 * ordinary softmax attention of the single query row q[s,h,:] over the
 * sequence's visible context
 *
 *     shared prefix (P ++ H)  ++  own private tokens (h_i ++ y_{i,<t}),
 *
 * and over nothing that belongs to a sibling branch.  The shared prefix is
 * stored once ("a single set of prefix blocks", §3.1): all members of a request
 * list the same physical pages for it; private tokens live in pages of their
 * own that start at block-table entry ceil(prefix_len/page).
 *
 * The paper does not print the attention formula; it is the textbook one,
 *     o = sum_t softmax_t(scale * q.k_t) v_t ,   scale = 1/sqrt(head_dim),
 * with grouped-query heads: query head h reads KV head h / (Hq/Hkv).
 *
 * The method on the GPU (split prefix/suffix partials, chunking, log-sum-exp
 * merge) is an exact re-association of this sum, so the oracle is the plain
 * definition: one pass over the whole visible context, no splitting.
 *
 * Pool layout (the library's boundary; stated in include/taper_attn.h and
 * re-derived here independently): the pool is [n_pages][2][Hkv][page*D] bf16.
 * Inside a (page, K, kv head) tile element (tok, d) sits at
 *     (d / 8) * (page*8) + tok * 8 + d % 8          ("K in groups of 8 dims")
 * and inside a (page, V, kv head) tile at
 *     (tok / 4) * (4*D) + d * 4 + tok % 4           ("V^T in groups of 4 tokens").
 *
 * Pins: tests/test_oracle_pins.py (library softmax on a dense gather, closed
 * forms, brute force with explicit term lists, invariances).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

/* element offset of K[page, hk, tok, d] (is_v = 0) or V[page, hk, tok, d] (is_v = 1) in the pool */
static int64_t kv_elem(int is_v, int64_t page, int hk, int tok, int d, int Hkv, int D, int P)
{
    int64_t tile = ((page * 2 + is_v) * Hkv + hk) * (int64_t)(P * D);
    if (!is_v)
        return tile + (int64_t)(d / 8) * (P * 8) + tok * 8 + d % 8;
    return tile + (int64_t)(tok / 4) * (4 * D) + d * 4 + tok % 4;
}

/* physical page and in-page token of logical position t of sequence s */
static void locate(const int32_t *bt_row, int prefix_len, int P, int t, int64_t *page, int *tok)
{
    if (t < prefix_len) {
        *page = bt_row[t / P];
        *tok = t % P;
    } else {
        int j = t - prefix_len;
        int npp = (int)ceil_div(prefix_len, P);
        *page = bt_row[npp + j / P];
        *tok = j % P;
    }
}

/*
 * Integer side.  For every sequence: context length, number of shared prefix
 * pages, number of private pages (the marginal memory of a branch, App. C:
 * blocks(branch-local tokens), zero for a branch with no tokens), the CSR of
 * requests over sequences, and the physical slot id (page*P + tok) of every
 * logical position (slots is [S, slots_stride], filled with -1 past the end).
 * Returns the number of groups, or -1 on malformed input.
 */
int taper_oracle_resolve(int S, int P, const int32_t *block_table, int bt_stride,
                         const int32_t *branch_group, const int32_t *prefix_len,
                         const int32_t *suffix_len, int32_t *ctx_len, int32_t *n_prefix_pages,
                         int32_t *n_suffix_pages, int32_t *group_start /* [S+1] */,
                         int64_t *slots, int64_t slots_stride)
{
    int G = 0;
    for (int s = 0; s < S; ++s) {
        if (s == 0 || branch_group[s] != branch_group[s - 1]) {
            if (s > 0 && branch_group[s] != branch_group[s - 1] + 1) return -1;
            if (s == 0 && branch_group[0] != 0) return -1;
            group_start[G++] = s;
        }
        ctx_len[s] = prefix_len[s] + suffix_len[s];
        n_prefix_pages[s] = (int32_t)ceil_div(prefix_len[s], P);
        n_suffix_pages[s] = (int32_t)ceil_div(suffix_len[s], P);
        if (slots) {
            for (int64_t t = 0; t < slots_stride; ++t) slots[s * slots_stride + t] = -1;
            for (int t = 0; t < ctx_len[s] && t < slots_stride; ++t) {
                int64_t page; int tok;
                locate(block_table + (int64_t)s * bt_stride, prefix_len[s], P, t, &page, &tok);
                slots[s * slots_stride + t] = page * P + tok;
            }
        }
    }
    group_start[G] = S;
    return G;
}

/*
 * Floating-point side: out[s,h,:] (fp64) and, if lse != NULL, the natural-log
 * normaliser lse[s,h] = m + log(sum_t exp(x_t - m)).  weights_sum, if given,
 * receives sum_t w_t / Z per (s,h) (should be 1).  Returns threads used.
 */
int taper_oracle_attention(int S, int Hq, int Hkv, int D, int P, double scale,
                           const uint16_t *q, const uint16_t *kv_pool,
                           const int32_t *block_table, int bt_stride,
                           const int32_t *prefix_len, const int32_t *suffix_len,
                           double *out, double *lse, double *weights_sum, int n_threads)
{
    int g = Hq / Hkv;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
    used = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int sh = 0; sh < S * Hq; ++sh) {
        int s = sh / Hq, h = sh % Hq, hk = h / g;
        const int32_t *row = block_table + (int64_t)s * bt_stride;
        int n = prefix_len[s] + suffix_len[s];
        double *x = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        double *o = out + ((int64_t)s * Hq + h) * D;
        const uint16_t *qrow = q + ((int64_t)s * Hq + h) * D;
        double m = -INFINITY;
        for (int t = 0; t < n; ++t) {
            int64_t page; int tok;
            locate(row, prefix_len[s], P, t, &page, &tok);
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += bf16_to_double(qrow[d]) * bf16_to_double(kv_pool[kv_elem(0, page, hk, tok, d, Hkv, D, P)]);
            x[t] = scale * acc;
            if (x[t] > m) m = x[t];
        }
        double Z = 0.0;
        for (int t = 0; t < n; ++t) { x[t] = exp(x[t] - m); Z += x[t]; }
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int t = 0; t < n; ++t) {
            int64_t page; int tok;
            locate(row, prefix_len[s], P, t, &page, &tok);
            for (int d = 0; d < D; ++d)
                o[d] += x[t] * bf16_to_double(kv_pool[kv_elem(1, page, hk, tok, d, Hkv, D, P)]);
        }
        double wsum = 0.0;
        for (int t = 0; t < n; ++t) wsum += x[t] / Z;
        for (int d = 0; d < D; ++d) o[d] /= Z;
        if (lse) lse[(int64_t)s * Hq + h] = m + log(Z);
        if (weights_sum) weights_sum[(int64_t)s * Hq + h] = wsum;
        free(x);
    }
    return used;
}

/* ------------------------------------------------------------------------
 * Reduce phase and KV append (the two steps around the parallel phase).
 *
 * Reduce-phase visibility (paper §3.1): a reduce token attends to the shared
 * prefix followed by ALL completed branches in canonical order and then the
 * reduce tokens generated so far,
 *     P ++ H ++ (h_1 ++ y_1) ++ ... ++ (h_n ++ y_n) ++ z_<t .
 * In a paged cache every one of these pieces keeps the pages it was written
 * to: the sequence's block-table row lists the prefix pages and then, piece by
 * piece, the pages of each private segment; a segment starts on a fresh page,
 * so partially filled pages occur in the middle of the context.  The context
 * is therefore a list of physical slots, and attention over it is the same
 * textbook sum as above.
 * ------------------------------------------------------------------------ */

/* Slot (page * P + token) of every logical position of sequences whose private
 * context is a list of segments: seg_len[seg_start[s] .. seg_start[s+1]).
 * ctx_len and n_private_pages are per sequence; slots is [S, stride], -1 past
 * the end.  n_private_pages is also the memory the private part occupies
 * (App. C memory accounting: blocks of branch-local tokens, none for an empty
 * segment). */
void taper_oracle_resolve_segments(int S, int P, const int32_t *block_table, int bt_stride,
                                   const int32_t *prefix_len, const int32_t *seg_start,
                                   const int32_t *seg_len, int32_t *ctx_len,
                                   int32_t *n_private_pages, int64_t *slots, int64_t slots_stride)
{
    for (int s = 0; s < S; ++s) {
        const int32_t *row = block_table + (int64_t)s * bt_stride;
        int64_t t = 0;
        int entry = 0, priv_pages = 0;
        if (slots)
            for (int64_t i = 0; i < slots_stride; ++i) slots[s * slots_stride + i] = -1;
        for (int j = 0; j < prefix_len[s]; ++j, ++t)
            if (slots && t < slots_stride) slots[s * slots_stride + t] = (int64_t)row[j / P] * P + j % P;
        entry = (int)ceil_div(prefix_len[s], P);
        for (int k = seg_start[s]; k < seg_start[s + 1]; ++k) {
            for (int j = 0; j < seg_len[k]; ++j, ++t)
                if (slots && t < slots_stride) slots[s * slots_stride + t] = (int64_t)row[entry + j / P] * P + j % P;
            entry += (int)ceil_div(seg_len[k], P);
            priv_pages += (int)ceil_div(seg_len[k], P);
        }
        ctx_len[s] = (int32_t)t;
        n_private_pages[s] = priv_pages;
    }
}

/* Attention of one query row per (sequence, head) over an explicit slot list. */
int taper_oracle_attention_slots(int S, int Hq, int Hkv, int D, int P, double scale,
                                 const uint16_t *q, const uint16_t *kv_pool, const int64_t *slots,
                                 int64_t slots_stride, const int32_t *ctx_len, double *out, double *lse,
                                 int n_threads)
{
    int g = Hq / Hkv;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
    used = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int sh = 0; sh < S * Hq; ++sh) {
        int s = sh / Hq, h = sh % Hq;
        int hk = (h - h % g) / g; /* grouped-query map: g consecutive query heads per KV head */
        const int64_t *sl = slots + (int64_t)s * slots_stride;
        int n = ctx_len[s];
        double *w = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        double *o = out + ((int64_t)s * Hq + h) * D;
        const uint16_t *qrow = q + ((int64_t)s * Hq + h) * D;
        double m = -INFINITY;
        for (int t = 0; t < n; ++t) {
            double acc = 0.0;
            for (int d = 0; d < D; ++d)
                acc += bf16_to_double(qrow[d]) * bf16_to_double(kv_pool[kv_elem(0, sl[t] / P, hk, (int)(sl[t] % P), d, Hkv, D, P)]);
            w[t] = acc * scale;
            if (w[t] > m) m = w[t];
        }
        double Z = 0.0;
        for (int t = 0; t < n; ++t) {
            w[t] = exp(w[t] - m);
            Z += w[t];
        }
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int t = 0; t < n; ++t)
            for (int d = 0; d < D; ++d)
                o[d] += w[t] * bf16_to_double(kv_pool[kv_elem(1, sl[t] / P, hk, (int)(sl[t] % P), d, Hkv, D, P)]);
        for (int d = 0; d < D; ++d) o[d] /= Z;
        if (lse) lse[(int64_t)s * Hq + h] = m + log(Z);
        free(w);
    }
    return used;
}

/* KV append: the step's new key and value rows (bf16 bits, [S][Hkv][D] each)
 * are written to slot[s] of the pool -- the position right after the
 * sequence's last cached token.  A pure copy into the tile layout above. */
void taper_oracle_kv_append(int S, int Hkv, int D, int P, const uint16_t *k_new, const uint16_t *v_new,
                            const int64_t *slot, uint16_t *kv_pool)
{
    for (int s = 0; s < S; ++s)
        for (int hk = 0; hk < Hkv; ++hk)
            for (int d = 0; d < D; ++d) {
                int64_t page = slot[s] / P;
                int tok = (int)(slot[s] % P);
                kv_pool[kv_elem(0, page, hk, tok, d, Hkv, D, P)] = k_new[((int64_t)s * Hkv + hk) * D + d];
                kv_pool[kv_elem(1, page, hk, tok, d, Hkv, D, P)] = v_new[((int64_t)s * Hkv + hk) * D + d];
            }
}
