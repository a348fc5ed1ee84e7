/*
 * jo_attention.c -- CPU oracle for paged decode attention.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, fp64 statement of what one rollout decode step's
 * attention computes.  It exists so that tests, the smoke check and the benchmark's
 * CPU-baseline leg have something to compare the GPU library against.  It shares no
 * code, header, table or helper with the GPU path, the product never calls it, and it
 * is not tuned.
 *
 * What it computes.  The paper runs rollout on a third-party inference engine and
 * prints no attention formula; it fixes only the setting (System Design, "Sub-Stage
 * Graph Abstraction": each forward step processes the active decoding requests;
 * Sub-stage Multiplexing, "GPU Memory Utilization": the KV cache bounds the concurrent
 * decoding requests; Motivation, "Varied Decoding Lengths": lengths are ragged and
 * long-tailed).  The result is therefore the textbook definition of softmax attention
 * for one new token per request, written out term by term:
 *
 *   for request b with L = seq_lens[b] tokens, query head h, kv head kv = h / (Hq/Hkv):
 *     token j lives at page = block_table[b][j / page_size], slot = j % page_size
 *     s_j = scale * sum_d q[b][h][d] * K[page][kv][slot][d]           j = 0 .. L-1
 *     m   = max_j s_j
 *     w_j = exp(s_j - m) / sum_i exp(s_i - m)
 *     out[b][h][d] = sum_j w_j * V[page][kv][slot][d]                 (j ascending)
 *
 * Readings taken where nothing fixes the detail: scale defaults to 1/sqrt(D); query head
 * h uses kv head floor(h / G) with G = Hq/Hkv; seq_lens counts the token being decoded
 * (its K/V are already in the cache, so no causal mask is needed); L = 0 gives a zero
 * row; slots beyond L, unowned pages and block-table entries beyond ceil(L/page) are
 * never read.  bf16 inputs are widened exactly; all arithmetic is fp64; the fp32 result
 * is one final round-to-nearest of the fp64 sum.
 *
 * Every function here is pinned by tests against closed forms (single key, equal keys,
 * two-key logistic weight, shift invariance, dominant key), invariants (page
 * permutation, convex hull, weights sum to one, split-and-merge), a library routine
 * (torch scaled_dot_product_attention in float64) and a separately written numpy
 * brute force.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    const uint16_t *q, *k, *v;
    const int32_t *bt, *lens;
    int B, Hq, Hkv, D, page, maxp;
    double scale;
} jo_problem;

static double bf16_to_f64(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static const uint16_t *token_row(const jo_problem *p, const uint16_t *pool, int b, int kv, int j)
{
    int64_t page = p->bt[(int64_t)b * p->maxp + j / p->page];
    int slot = j % p->page;
    return pool + ((page * p->Hkv + kv) * p->page + slot) * (int64_t)p->D;
}

static double score(const jo_problem *p, int b, int h, int j)
{
    int kv = h / (p->Hq / p->Hkv);
    const uint16_t *qr = p->q + ((int64_t)b * p->Hq + h) * p->D;
    const uint16_t *kr = token_row(p, p->k, b, kv, j);
    double s = 0.0;
    for (int d = 0; d < p->D; ++d)
        s += bf16_to_f64(qr[d]) * bf16_to_f64(kr[d]);
    return p->scale * s;
}

static double resolve_scale(double scale, int D)
{
    return scale == 0.0 ? 1.0 / sqrt((double)D) : scale;
}

/* One output row by the definition above.  w must hold L doubles; on return it holds
 * the normalised softmax weights. */
static void attend_row(const jo_problem *p, int b, int h, double *w, double *out)
{
    int L = p->lens[b];
    int kv = h / (p->Hq / p->Hkv);
    for (int d = 0; d < p->D; ++d)
        out[d] = 0.0;
    if (L <= 0)
        return;
    double m = -INFINITY;
    for (int j = 0; j < L; ++j) {
        w[j] = score(p, b, h, j);
        if (w[j] > m)
            m = w[j];
    }
    double z = 0.0;
    for (int j = 0; j < L; ++j) {
        w[j] = exp(w[j] - m);
        z += w[j];
    }
    for (int j = 0; j < L; ++j)
        w[j] /= z;
    for (int j = 0; j < L; ++j) {
        const uint16_t *vr = token_row(p, p->v, b, kv, j);
        for (int d = 0; d < p->D; ++d)
            out[d] += w[j] * bf16_to_f64(vr[d]);
    }
}

static int check(const jo_problem *p)
{
    if (!p->q || !p->k || !p->v || !p->bt || !p->lens)
        return 1;
    if (p->B < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->D <= 0 || p->page <= 0 || p->maxp <= 0)
        return 1;
    if (p->Hq % p->Hkv)
        return 1;
    return 0;
}

/*
 * Attention rows of one decode step.
 *   rows_bh  NULL: every (b, h), b-major, n_rows ignored, outputs are [B*Hq, D];
 *            else n_rows pairs (b, h) and outputs are [n_rows, D] in that order.
 *   out64 / out32  either may be NULL.  out32 is the fp64 result rounded once to fp32.
 *   threads  <= 0 means the OpenMP default.
 * Returns 0, or 1 on a malformed argument (nothing written).
 */
int jo_decode_attention(const uint16_t *q, const uint16_t *k_pages, const uint16_t *v_pages,
                        const int32_t *block_table, const int32_t *seq_lens, int B, int Hq, int Hkv,
                        int D, int page_size, int max_pages_per_seq, double scale,
                        const int32_t *rows_bh, int n_rows, double *out64, float *out32, int threads)
{
    jo_problem p = { q, k_pages, v_pages, block_table, seq_lens, B, Hq, Hkv, D, page_size,
                     max_pages_per_seq, resolve_scale(scale, D) };
    if (check(&p))
        return 1;
    int64_t n = rows_bh ? n_rows : (int64_t)B * Hq;
    int bad = 0;
    for (int64_t r = 0; r < n && rows_bh; ++r)
        if (rows_bh[2 * r] < 0 || rows_bh[2 * r] >= B || rows_bh[2 * r + 1] < 0 || rows_bh[2 * r + 1] >= Hq)
            bad = 1;
    if (bad)
        return 1;
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#endif
    (void)threads;
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < n; ++r) {
            int b = rows_bh ? rows_bh[2 * r] : (int)(r / Hq);
            int h = rows_bh ? rows_bh[2 * r + 1] : (int)(r % Hq);
            int L = seq_lens[b] > 0 ? seq_lens[b] : 0;
            double *w = (double *)malloc(sizeof(double) * (size_t)(L + 1));
            attend_row(&p, b, h, w, acc);
            for (int d = 0; d < D; ++d) {
                if (out64)
                    out64[r * D + d] = acc[d];
                if (out32)
                    out32[r * D + d] = (float)acc[d];
            }
            free(w);
        }
        free(acc);
    }
    return 0;
}

/* Softmax weights w[0..L) of row (b, h); they sum to one.  Returns L, or -1 on error. */
int jo_softmax_weights(const uint16_t *q, const uint16_t *k_pages, const uint16_t *v_pages,
                       const int32_t *block_table, const int32_t *seq_lens, int B, int Hq, int Hkv,
                       int D, int page_size, int max_pages_per_seq, double scale, int b, int h,
                       double *w)
{
    jo_problem p = { q, k_pages, v_pages, block_table, seq_lens, B, Hq, Hkv, D, page_size,
                     max_pages_per_seq, resolve_scale(scale, D) };
    if (check(&p) || b < 0 || b >= B || h < 0 || h >= Hq || !w)
        return -1;
    double *acc = (double *)malloc(sizeof(double) * (size_t)D);
    attend_row(&p, b, h, w, acc);
    free(acc);
    return seq_lens[b] > 0 ? seq_lens[b] : 0;
}

/*
 * Unnormalised attention state of row (b, h) over an arbitrary subset of its tokens:
 *   m = max_j s_j,  l = sum_j exp(s_j - m),  acc[d] = sum_j exp(s_j - m) v_j[d],  j in tokens[0..n).
 * With n = 0: m = -inf, l = 0, acc = 0.  This is the quantity a split of the sequence
 * produces per piece; jo_merge_states puts pieces back together.
 */
int jo_partial_state(const uint16_t *q, const uint16_t *k_pages, const uint16_t *v_pages,
                     const int32_t *block_table, const int32_t *seq_lens, int B, int Hq, int Hkv,
                     int D, int page_size, int max_pages_per_seq, double scale, int b, int h,
                     const int32_t *tokens, int n, double *m_out, double *l_out, double *acc)
{
    jo_problem p = { q, k_pages, v_pages, block_table, seq_lens, B, Hq, Hkv, D, page_size,
                     max_pages_per_seq, resolve_scale(scale, D) };
    if (check(&p) || b < 0 || b >= B || h < 0 || h >= Hq || n < 0 || (n && !tokens))
        return 1;
    for (int i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= seq_lens[b])
            return 1;
    int kv = h / (Hq / Hkv);
    double m = -INFINITY, l = 0.0;
    for (int d = 0; d < D; ++d)
        acc[d] = 0.0;
    for (int i = 0; i < n; ++i) {
        double s = score(&p, b, h, tokens[i]);
        if (s > m)
            m = s;
    }
    for (int i = 0; i < n; ++i) {
        double e = exp(score(&p, b, h, tokens[i]) - m);
        const uint16_t *vr = token_row(&p, v_pages, b, kv, tokens[i]);
        l += e;
        for (int d = 0; d < D; ++d)
            acc[d] += e * bf16_to_f64(vr[d]);
    }
    *m_out = m;
    *l_out = l;
    return 0;
}

/*
 * Log-sum-exp merge of n partial states into the normalised output row:
 *   M = max_i m_i,  out[d] = sum_i exp(m_i - M) acc_i[d] / sum_i exp(m_i - M) l_i.
 * Pieces with l_i = 0 (empty subsets, m_i = -inf) contribute nothing; if every piece is
 * empty the row is zero.
 */
int jo_merge_states(int n, const double *m, const double *l, const double *acc, int D, double *out)
{
    if (n < 0 || D <= 0 || !out)
        return 1;
    double M = -INFINITY, z = 0.0;
    for (int d = 0; d < D; ++d)
        out[d] = 0.0;
    for (int i = 0; i < n; ++i)
        if (l[i] > 0.0 && m[i] > M)
            M = m[i];
    if (M == -INFINITY)
        return 0;
    for (int i = 0; i < n; ++i) {
        if (!(l[i] > 0.0))
            continue;
        double e = exp(m[i] - M);
        z += e * l[i];
        for (int d = 0; d < D; ++d)
            out[d] += e * acc[(int64_t)i * D + d];
    }
    for (int d = 0; d < D; ++d)
        out[d] /= z;
    return 0;
}

/*
 * Causal attention of a chunk of new tokens over the paged cache (prefill / KV recomputation).
 * Request b has L = seq_lens[b] tokens in the cache, the last n = q_lens[b] of which are the new ones;
 * their queries are rows q_offsets[b] .. q_offsets[b] + n - 1 of q ([TQ, Hq, D]).  New token t
 * (0 <= t < n) sits at position c + t with c = L - n and attends to positions 0 .. c + t:
 *
 *     out[q_offsets[b] + t][h] = sum_{j <= c + t} softmax_j(scale * <q_t,h , K_j>) V_j
 *
 * This is what a migrated request pays to rebuild its cache (Sub-stage Merging: the migration
 * overhead is dominated by KV cache recomputation), and what every new turn of a multi-turn
 * rollout starts with (Motivation, "Multi-turn Rollout Idling").  With n = 1 it is exactly
 * jo_decode_attention.  Outputs are [TQ, Hq, D]; out64 / out32 may be NULL.  Returns 0, or 1 on a
 * malformed argument (n < 0, n > L, offsets not increasing by at least n).
 */
int jo_prefill_attention(const uint16_t *q, const uint16_t *k_pages, const uint16_t *v_pages,
                         const int32_t *block_table, const int32_t *seq_lens, const int32_t *q_lens,
                         const int32_t *q_offsets, int B, int Hq, int Hkv, int D, int page_size,
                         int max_pages_per_seq, double scale, double *out64, float *out32, int threads)
{
    jo_problem p = { q, k_pages, v_pages, block_table, seq_lens, B, Hq, Hkv, D, page_size,
                     max_pages_per_seq, resolve_scale(scale, D) };
    if (check(&p) || !q_lens || !q_offsets)
        return 1;
    for (int b = 0; b < B; ++b) {
        int L = seq_lens[b] > 0 ? seq_lens[b] : 0;
        if (q_lens[b] < 0 || q_lens[b] > L || q_offsets[b] < 0)
            return 1;
        if (b + 1 < B && q_offsets[b + 1] < q_offsets[b] + q_lens[b])
            return 1;
    }
#ifdef _OPENMP
    if (threads > 0)
        omp_set_num_threads(threads);
#endif
    (void)threads;
    int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < Hq; ++h) {
            int L = seq_lens[b] > 0 ? seq_lens[b] : 0;
            int n = q_lens[b], c = L - n, kv = h / G;
            double *w = (double *)malloc(sizeof(double) * (size_t)(L + 1));
            double *acc = (double *)malloc(sizeof(double) * (size_t)D);
            for (int t = 0; t < n; ++t) {
                int64_t row = (int64_t)q_offsets[b] + t;
                const uint16_t *qr = q + (row * Hq + h) * D;
                int last = c + t; /* attends to positions 0 .. last */
                double m = -INFINITY, z = 0.0;
                for (int j = 0; j <= last; ++j) {
                    const uint16_t *kr = token_row(&p, k_pages, b, kv, j);
                    double s = 0.0;
                    for (int d = 0; d < D; ++d)
                        s += bf16_to_f64(qr[d]) * bf16_to_f64(kr[d]);
                    w[j] = p.scale * s;
                    if (w[j] > m)
                        m = w[j];
                }
                for (int j = 0; j <= last; ++j) {
                    w[j] = exp(w[j] - m);
                    z += w[j];
                }
                for (int d = 0; d < D; ++d)
                    acc[d] = 0.0;
                for (int j = 0; j <= last; ++j) {
                    const uint16_t *vr = token_row(&p, v_pages, b, kv, j);
                    double wj = w[j] / z;
                    for (int d = 0; d < D; ++d)
                        acc[d] += wj * bf16_to_f64(vr[d]);
                }
                for (int d = 0; d < D; ++d) {
                    if (out64)
                        out64[(row * Hq + h) * D + d] = acc[d];
                    if (out32)
                        out32[(row * Hq + h) * D + d] = (float)acc[d];
                }
            }
            free(w);
            free(acc);
        }
    }
    return 0;
}

int jo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
