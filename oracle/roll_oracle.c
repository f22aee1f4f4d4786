/*
 * roll_oracle.c - plain fp64 CPU oracle of the rollout decode step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the decode step of a
 * ROLL Flash (arXiv 2510.11345) serving worker computes, written as the
 * textbook definitions with no blocking, no online softmax, no splitting
 * and no fast-math.  It shares no code with the GPU library; only tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Passages followed.  The paper treats the inference-engine step as a
 * black box: Section 4.2 says each iteration of the worker loop executes
 * one decode step over the batch of requests; Section 1 says decoding is
 * memory-bandwidth bound; Appendix A.1 fixes temperature 1, top_p 1,
 * top_k disabled, one beam, and says the engine must return the original
 * token probabilities, which become pi_vllm in the truncated importance
 * weight min(pi_megatron / pi_vllm, C).  The arithmetic below is therefore
 * the standard definition of each named operation:
 *   - scaled dot-product attention of one query token per head against a
 *     paged KV cache with grouped-query head sharing,
 *   - softmax with temperature, nucleus (top-p) truncation, Gumbel-max
 *     sampling, log-prob of the drawn token under the sampled distribution,
 *   - Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) as the counter-based
 *     generator.
 * Readings taken where the paper is silent are stated at each function.
 *
 * Parity pins (tests/test_oracle_*.py): Philox against the published
 * known-answer vectors and an independent big-integer implementation;
 * attention against L=1, identical keys, q=0, dominant key, convex hull,
 * page permutation, GQA sharing, split/merge, dense library softmax(QK^T)V
 * and two-key closed form; sampling against library log_softmax, uniform
 * logits, shift and scale invariance, brute-force subset enumeration of the
 * top-p set, chi-square of sampled frequencies on tiny vocabularies; the
 * off-policy objectives against hand-computed values, the reductions between
 * them that the paper's description implies, and a numerical derivative.
 * End-to-end numbers: parity unpinned against the paper (it prints no
 * worked numeric example for this path).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_BF16 0
#define ORACLE_F32 1

/* ------------------------------------------------------------------ */
/* Number formats                                                      */
/* ------------------------------------------------------------------ */

/* bf16 is the upper half of a binary32: widening is exact. */
static double bf16_to_double(uint16_t h)
{
    uint32_t bits = (uint32_t)h << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

double oracle_bf16_to_double(uint16_t h) { return bf16_to_double(h); }

/* ------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon et al., SC'11, Section 3.3 and Table 2 consts) */
/* ------------------------------------------------------------------ */

void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t mul_a = 0xD2511F53u, mul_b = 0xCD9E8D57u;
    const uint32_t weyl_a = 0x9E3779B9u, weyl_b = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += weyl_a;
            k1 += weyl_b;
        }
        uint64_t pa = mul_a * (uint64_t)c0;
        uint64_t pb = mul_b * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)pb;
        uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)pa;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/*
 * Uniform of vocabulary entry i of row row_id at decode step `step`:
 * counter (i >> 2, row_id, step_lo, step_hi), key (seed_lo, seed_hi),
 * word i & 3; the top 23 bits k of the word give u = (k + 0.5) * 2^-23,
 * which lies in [2^-24, 1 - 2^-24] and is exact in binary32 and binary64.
 * (Reading: the paper fixes only `seed`; the mapping is ours.)
 */
double oracle_uniform(uint64_t seed, uint64_t step, uint32_t row_id, uint32_t i)
{
    uint32_t ctr[4] = { i >> 2, row_id, (uint32_t)step, (uint32_t)(step >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t w[4];
    oracle_philox4x32_10(ctr, key, w);
    return ((double)(w[i & 3] >> 9) + 0.5) * 0x1p-23;
}

/* ------------------------------------------------------------------ */
/* Paged KV cache: index formulas of the two page layouts              */
/*   K: [page][h][d / 8][kpos(t)][d % 8]   V: [page][h][t / 8][d][t % 8] */
/* ------------------------------------------------------------------ */

/*
 * Slot of token t inside a K block row.  Tokens are taken in blocks of
 * width = min(P, 32); inside a block, every run of 8 tokens is split: its
 * first four go to the first half of the block, its last four to the second
 * half, runs kept in order.
 */
int oracle_k_slot(int t, int P)
{
    int width = P < 32 ? P : 32;
    int block = t / width, u = t % width;
    int run = u / 8, in_run = u % 8;
    int half = in_run / 4, quad_pos = in_run % 4;
    return block * width + half * (width / 2) + run * 4 + quad_pos;
}

int64_t oracle_k_index(int64_t page, int h, int t, int d, int Hkv, int D, int P)
{
    return ((((page * Hkv + h) * (D / 8) + d / 8) * P + oracle_k_slot(t, P)) * 8) + d % 8;
}

int64_t oracle_v_index(int64_t page, int h, int t, int d, int Hkv, int D, int P)
{
    return ((((page * Hkv + h) * (P / 8) + t / 8) * D + d) * 8) + t % 8;
}

/* Store one token's K and V vectors (bf16 [Hkv, D] each) at slot t of a page. */
void oracle_kv_store(uint16_t* k_pages, uint16_t* v_pages, int64_t page, int t,
                     const uint16_t* k_tok, const uint16_t* v_tok, int Hkv, int D, int P)
{
    for (int h = 0; h < Hkv; ++h)
        for (int d = 0; d < D; ++d) {
            k_pages[oracle_k_index(page, h, t, d, Hkv, D, P)] = k_tok[h * D + d];
            v_pages[oracle_v_index(page, h, t, d, Hkv, D, P)] = v_tok[h * D + d];
        }
}

/* ------------------------------------------------------------------ */
/* Decode attention                                                    */
/* ------------------------------------------------------------------ */

/*
 * Scores and un-normalised sums of one (row, head) over KV positions
 * [j0, j1): m = max_j s_j, l = sum_j exp(s_j - m), acc[d] = sum_j
 * exp(s_j - m) V_j[d].  j1 <= j0 gives m = -inf, l = 0, acc = 0.
 * Readings: scale is a parameter (default 1/sqrt(D) chosen by the caller);
 * Q and K arrive position-encoded; no mask beyond the length.
 */
void oracle_attn_range(const uint16_t* q, const uint16_t* k_pages, const uint16_t* v_pages,
                       const int32_t* page_table, int b, int h, int j0, int j1,
                       int Hq, int Hkv, int D, int P, int max_pages, double scale,
                       double* m_out, double* l_out, double* acc /* [D] */)
{
    const int group = Hq / Hkv;
    const int kvh = h / group;
    const uint16_t* qv = q + ((int64_t)b * Hq + h) * D;
    const int32_t* pt = page_table + (int64_t)b * max_pages;
    int n = j1 - j0;
    for (int d = 0; d < D; ++d) acc[d] = 0.0;
    if (n <= 0) {
        *m_out = -INFINITY;
        *l_out = 0.0;
        return;
    }
    double* s = (double*)malloc(sizeof(double) * (size_t)n);
    double m = -INFINITY;
    for (int j = j0; j < j1; ++j) {
        int64_t page = pt[j / P];
        int t = j % P;
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += bf16_to_double(qv[d]) *
                   bf16_to_double(k_pages[oracle_k_index(page, kvh, t, d, Hkv, D, P)]);
        s[j - j0] = dot * scale;
        if (s[j - j0] > m) m = s[j - j0];
    }
    double l = 0.0;
    for (int j = j0; j < j1; ++j) {
        int64_t page = pt[j / P];
        int t = j % P;
        double w = exp(s[j - j0] - m);
        l += w;
        for (int d = 0; d < D; ++d)
            acc[d] += w * bf16_to_double(v_pages[oracle_v_index(page, kvh, t, d, Hkv, D, P)]);
    }
    free(s);
    *m_out = m;
    *l_out = l;
}

/*
 * out[b,h,:] = sum_j softmax_j(scale * <q[b,h], K_j>) V_j over j in
 * [0, seq_lens[b]); rows with length 0 give zeros.  `rows` (n_rows entries)
 * selects which batch rows to compute, NULL = all B; out is always indexed
 * by the true row id, [B, Hq, D] fp64.  Returns the number of threads used.
 */
int oracle_decode_attn(const uint16_t* q, const uint16_t* k_pages, const uint16_t* v_pages,
                       const int32_t* page_table, const int32_t* seq_lens, double* out,
                       int B, int Hq, int Hkv, int D, int P, int max_pages, double scale,
                       const int32_t* rows, int n_rows, int n_threads)
{
    int n = rows ? n_rows : B;
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
    used = omp_get_max_threads();
#endif
    int64_t units = (int64_t)n * Hq;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        int b = rows ? rows[u / Hq] : (int)(u / Hq);
        int h = (int)(u % Hq);
        double* o = out + ((int64_t)b * Hq + h) * D;
        int L = seq_lens[b];
        if (L <= 0) {
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            continue;
        }
        double m, l;
        oracle_attn_range(q, k_pages, v_pages, page_table, b, h, 0, L, Hq, Hkv, D, P,
                          max_pages, scale, &m, &l, o);
        for (int d = 0; d < D; ++d) o[d] /= l;
    }
    return used;
}

/* ------------------------------------------------------------------ */
/* Chunked prefill                                                     */
/* ------------------------------------------------------------------ */

/*
 * The prefill step of the engine loop (Section 4.2: a request that joins the
 * running batch is first prefilled, then decoded step by step), taken in
 * chunks.  Chunk c holds the n_c = chunk_offset[c+1] - chunk_offset[c]
 * consecutive tokens of slot chunk_slot[c] at positions chunk_start[c] + j;
 * the slot's page-table row already maps those positions.
 *   1. every chunk token's K and V ([Hkv, D] bf16 each) go into the pages at
 *      the token's position;
 *   2. token (c, j) attends causally over its slot's positions
 *      0 .. chunk_start[c] + j:  out = sum_i softmax_i(scale <q, K_i>) V_i.
 * q, out are [T, Hq, D] and k_new, v_new [T, Hkv, D] with T = chunk_offset[C];
 * query head h uses KV head h / (Hq / Hkv).  Everything in fp64.
 * Readings: Q and K arrive position-encoded; plain causal mask, nothing else.
 * Returns the number of threads used.
 */
int oracle_prefill_attn(const uint16_t* q, const uint16_t* k_new, const uint16_t* v_new,
                        const int32_t* chunk_slot, const int32_t* chunk_start,
                        const int32_t* chunk_offset, int C, uint16_t* k_pages, uint16_t* v_pages,
                        const int32_t* page_table, double* out, int Hq, int Hkv, int D, int P,
                        int max_pages, double scale, int n_threads)
{
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
    used = omp_get_max_threads();
#endif
    /* step 1, in token order */
    for (int c = 0; c < C; ++c)
        for (int t = chunk_offset[c]; t < chunk_offset[c + 1]; ++t) {
            int pos = chunk_start[c] + (t - chunk_offset[c]);
            int64_t page = page_table[(int64_t)chunk_slot[c] * max_pages + pos / P];
            oracle_kv_store(k_pages, v_pages, page, pos % P, k_new + (int64_t)t * Hkv * D,
                            v_new + (int64_t)t * Hkv * D, Hkv, D, P);
        }
    /* step 2: tokens and heads are independent */
    const int group = Hq / Hkv;
    for (int c = 0; c < C; ++c) {
        const int32_t* pt = page_table + (int64_t)chunk_slot[c] * max_pages;
        const int t_begin = chunk_offset[c], n_tok = chunk_offset[c + 1] - chunk_offset[c];
        const int64_t units = (int64_t)n_tok * Hq;
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t u = 0; u < units; ++u) {
            const int t = t_begin + (int)(u / Hq), h = (int)(u % Hq), kvh = h / group;
            const int last = chunk_start[c] + (t - t_begin); /* newest position the token sees */
            const uint16_t* qv = q + ((int64_t)t * Hq + h) * D;
            double* o = out + ((int64_t)t * Hq + h) * D;
            double* sc = (double*)malloc(sizeof(double) * (size_t)(last + 1));
            double mx = -INFINITY;
            for (int i = 0; i <= last; ++i) {
                double dot = 0.0;
                for (int d = 0; d < D; ++d)
                    dot += bf16_to_double(qv[d]) *
                           bf16_to_double(k_pages[oracle_k_index(pt[i / P], kvh, i % P, d, Hkv, D, P)]);
                sc[i] = dot * scale;
                if (sc[i] > mx) mx = sc[i];
            }
            double z = 0.0;
            for (int i = 0; i <= last; ++i) z += exp(sc[i] - mx);
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int i = 0; i <= last; ++i) {
                double wgt = exp(sc[i] - mx) / z;
                for (int d = 0; d < D; ++d)
                    o[d] += wgt * bf16_to_double(v_pages[oracle_v_index(pt[i / P], kvh, i % P, d, Hkv, D, P)]);
            }
            free(sc);
        }
    }
    return used;
}

/* ------------------------------------------------------------------ */
/* Sampling                                                            */
/* ------------------------------------------------------------------ */

static double logit_to_double(const void* row, int dtype, int64_t i)
{
    if (dtype == ORACLE_BF16) return bf16_to_double(((const uint16_t*)row)[i]);
    return (double)((const float*)row)[i];
}

static int cmp_desc(const void* a, const void* b)
{
    double x = *(const double*)a, y = *(const double*)b;
    return (x < y) - (x > y);
}

/*
 * Nucleus cut of one row.  x = logits (exact in fp64), z = x / T,
 * p = softmax(z).  Going down the DISTINCT values of x, add the mass of
 * all entries equal to the value; x_cut is the first value at which the
 * running mass is >= top_p, and the kept set is { i : x_i >= x_cut }.
 * top_p >= 1 keeps everything (x_cut = -inf).  Entries of -inf are masked
 * tokens (probability 0); a row without any finite entry has no softmax and
 * therefore no cut: NaN.
 * Readings: truncation applies to the tempered distribution; the token
 * that crosses top_p is kept; entries tied with the cut value are kept,
 * so the set does not depend on any sort order.
 */
double oracle_top_p_cut(const double* x, int V, double T, double top_p)
{
    double m = -INFINITY;
    for (int i = 0; i < V; ++i)
        if (x[i] / T > m) m = x[i] / T;
    if (!(m > -INFINITY)) return NAN; /* no finite entry: no distribution, so no cut */
    if (top_p >= 1.0) return -INFINITY;
    double Z = 0.0;
    for (int i = 0; i < V; ++i) Z += exp(x[i] / T - m);
    double* sorted = (double*)malloc(sizeof(double) * (size_t)V);
    memcpy(sorted, x, sizeof(double) * (size_t)V);
    qsort(sorted, (size_t)V, sizeof(double), cmp_desc);
    double run = 0.0, cut = sorted[V - 1];
    int i = 0;
    while (i < V) {
        double v = sorted[i];
        while (i < V && sorted[i] == v) {
            run += exp(v / T - m) / Z;
            ++i;
        }
        if (run >= top_p) {
            cut = v;
            break;
        }
    }
    free(sorted);
    return cut;
}

/*
 * One row: kept set, Gumbel-max token, its log-prob under the kept,
 * renormalised, tempered distribution.
 *   g_i = -log(-log u_i);  token = argmax_{kept} z_i + g_i, lowest index on
 *   exact ties;  logprob = z_token - log sum_{kept} exp(z_i).
 * Extra outputs for the parity report: gap = best minus second-best
 * perturbed logit (+inf if one entry is kept), kept count, x_cut, and the
 * cuts for top_p - band and top_p + band (the boundary band).
 * Reading (the paper says nothing of masked vocabularies): -inf entries are
 * masked tokens; a row in which every entry is masked defines no distribution,
 * so nothing is drawn from it: token = -1, logprob = raw_logprob = NaN (the
 * importance weight of Appendix A.1 has no denominator), kept = 0,
 * gap = +inf, the three cuts NaN.
 */
static void sample_row(const void* row, int dtype, int V, double T, double top_p,
                       uint64_t seed, uint64_t step, uint32_t row_id, double band,
                       int32_t* token, double* logprob, double* gap, int32_t* kept_count,
                       double* x_cut, double* x_cut_minus, double* x_cut_plus, double* raw_logprob)
{
    double* x = (double*)malloc(sizeof(double) * (size_t)V);
    int finite_entries = 0;
    for (int i = 0; i < V; ++i) {
        x[i] = logit_to_double(row, dtype, i);
        if (x[i] > -INFINITY) ++finite_entries;
    }
    if (finite_entries == 0) { /* every token masked: no distribution, no token */
        *token = -1;
        *logprob = NAN;
        if (raw_logprob) *raw_logprob = NAN;
        if (gap) *gap = INFINITY;
        if (kept_count) *kept_count = 0;
        if (x_cut) *x_cut = NAN;
        if (x_cut_minus) *x_cut_minus = NAN;
        if (x_cut_plus) *x_cut_plus = NAN;
        free(x);
        return;
    }
    double cut = oracle_top_p_cut(x, V, T, top_p);
    if (x_cut) *x_cut = cut;
    if (x_cut_minus) {
        double p = top_p - band;
        *x_cut_minus = band == 0.0 ? cut : oracle_top_p_cut(x, V, T, p > 0.0 ? p : 1e-300);
    }
    if (x_cut_plus) *x_cut_plus = oracle_top_p_cut(x, V, T, top_p + band);

    double m = -INFINITY;
    for (int i = 0; i < V; ++i)
        if (x[i] >= cut && x[i] / T > m) m = x[i] / T;
    double S = 0.0;
    int kept = 0;
    for (int i = 0; i < V; ++i)
        if (x[i] >= cut) {
            S += exp(x[i] / T - m);
            ++kept;
        }
    double lse = m + log(S);

    double best = -INFINITY, second = -INFINITY;
    int arg = -1;
    for (int i = 0; i < V; ++i) {
        if (!(x[i] >= cut)) continue;
        double u = oracle_uniform(seed, step, row_id, (uint32_t)i);
        double y = x[i] / T - log(-log(u));
        if (y > best) {
            second = best;
            best = y;
            arg = i;
        } else if (y > second) {
            second = y;
        }
    }
    *token = arg;
    *logprob = x[arg] / T - lse;
    if (raw_logprob) {
        /* log-prob of the same token under the untouched distribution softmax(x): temperature 1,
         * no truncation (what a training engine recomputes from the raw logits) */
        double xm = -INFINITY, sum = 0.0;
        for (int i = 0; i < V; ++i)
            if (x[i] > xm) xm = x[i];
        for (int i = 0; i < V; ++i) sum += exp(x[i] - xm);
        *raw_logprob = x[arg] - (xm + log(sum));
    }
    if (gap) *gap = best - second;
    if (kept_count) *kept_count = kept;
    free(x);
}

/*
 * All rows.  logits [B, row_stride] of dtype (ORACLE_BF16 / ORACLE_F32);
 * row_ids (NULL = 0..B-1) are the Philox row ids.  Optional outputs may be
 * NULL.  Returns the number of threads used.
 */
int oracle_sample_logprob(const void* logits, int dtype, int B, int V, int64_t row_stride,
                          double temperature, double top_p, uint64_t seed, uint64_t step,
                          const int32_t* row_ids, double band,
                          int32_t* tokens, double* logprob, double* gap, int32_t* kept_count,
                          double* x_cut, double* x_cut_minus, double* x_cut_plus,
                          double* raw_logprob, int n_threads)
{
    int used = 1;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
    used = omp_get_max_threads();
#endif
    size_t elem = dtype == ORACLE_BF16 ? 2 : 4;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < B; ++r) {
        const char* row = (const char*)logits + (size_t)r * (size_t)row_stride * elem;
        uint32_t rid = row_ids ? (uint32_t)row_ids[r] : (uint32_t)r;
        sample_row(row, dtype, V, temperature, top_p, seed, step, rid, band,
                   &tokens[r], &logprob[r], gap ? &gap[r] : NULL,
                   kept_count ? &kept_count[r] : NULL, x_cut ? &x_cut[r] : NULL,
                   x_cut_minus ? &x_cut_minus[r] : NULL, x_cut_plus ? &x_cut_plus[r] : NULL,
                   raw_logprob ? &raw_logprob[r] : NULL);
    }
    return used;
}

/*
 * Perturbed logits z_i - log(-log u_i) of one row for every i (kept or
 * not), and the kept mask; lets tests enumerate tiny vocabularies.
 */
void oracle_row_detail(const void* row, int dtype, int V, double T, double top_p,
                       uint64_t seed, uint64_t step, uint32_t row_id,
                       double* perturbed /* [V] */, uint8_t* kept /* [V] */)
{
    double* x = (double*)malloc(sizeof(double) * (size_t)V);
    for (int i = 0; i < V; ++i) x[i] = logit_to_double(row, dtype, i);
    double cut = oracle_top_p_cut(x, V, T, top_p);
    for (int i = 0; i < V; ++i) {
        double u = oracle_uniform(seed, step, row_id, (uint32_t)i);
        perturbed[i] = x[i] / T - log(-log(u));
        kept[i] = x[i] >= cut;
    }
    free(x);
}

/*
 * Token counts of n_draws independent draws of one row (steps step0 ..
 * step0 + n_draws - 1) for the frequency tests on tiny vocabularies.
 */
void oracle_sample_counts(const void* row, int dtype, int V, double T, double top_p,
                          uint64_t seed, uint64_t step0, int64_t n_draws, uint32_t row_id,
                          int64_t* counts /* [V], zeroed by the caller */)
{
    for (int64_t s = 0; s < n_draws; ++s) {
        int32_t tok;
        double lp;
        sample_row(row, dtype, V, T, top_p, seed, step0 + (uint64_t)s, row_id, 0.0,
                   &tok, &lp, NULL, NULL, NULL, NULL, NULL, NULL);
        if (tok >= 0) counts[tok] += 1; /* a row without a finite entry draws nothing */
    }
}

/* ------------------------------------------------------------------ */
/* Consumer of the recorded log-probs: off-policy objectives           */
/* ------------------------------------------------------------------ */

#define ORACLE_LOSS_PPO 0
#define ORACLE_LOSS_DECOUPLED_PPO 1
#define ORACLE_LOSS_TIS 2
#define ORACLE_LOSS_CISPO 3
#define ORACLE_LOSS_TOPR 4

static double clip_d(double x, double lo, double hi) { return x < lo ? lo : (x > hi ? hi : x); }

/*
 * Per-token value of the five objectives of Section 3.2 ("Loss Objective for
 * Off-policy Algorithms") and its derivative with respect to log pi_theta,
 * with pi_old the rollout engine's recorded probability.  lt, lo, lp are the
 * log-probs of the token under pi_theta, pi_old, pi_prox; R is the learning
 * signal (reward or advantage).  (x)^a_b in the paper is clip(x, b, a).
 *   PPO            min(R r, R clip(r, 1 - eps_lo, 1 + eps_hi)),           r = pi_theta / pi_old
 *   Decoupled PPO  min(R r, R (pi_prox / pi_old) clip(pi_theta / pi_prox, 1 - eps_lo, 1 + eps_hi))
 *   Truncated IS   sg(clip(r, 0, c)) R log pi_theta
 *   CISPO          sg(clip(r, 1 - eps_lo, 1 + eps_hi)) R log pi_theta
 *   TOPR           (1[T+] + 1[T-] sg(clip(r, 0, c))) R log pi_theta
 * Readings: the symmetric eps of PPO is given as the pair (eps_lo, eps_hi) so
 * that CISPO's asymmetric interval uses the same parameters; a trajectory is
 * in T+ when its signal is > 0 (the paper says "high-return / correct"); sg()
 * terms contribute no derivative; at a clip corner the derivative of the
 * clipped branch is taken as 0 and min() prefers the first argument on ties.
 * is_weight = min(r, c): the truncated importance weight of Appendix A.1.
 */
void oracle_policy_loss_token(int kind, double lt, double lo, double lp, double R, double eps_lo,
                              double eps_hi, double c, double* value, double* dvalue_dlt,
                              double* is_weight)
{
    double r = exp(lt - lo);
    double v = 0.0, g = 0.0;
    if (kind == ORACLE_LOSS_PPO) {
        double a = R * r, b = R * clip_d(r, 1.0 - eps_lo, 1.0 + eps_hi);
        int inside = r > 1.0 - eps_lo && r < 1.0 + eps_hi;
        if (a <= b) { v = a; g = R * r; } else { v = b; g = inside ? R * r : 0.0; }
    } else if (kind == ORACLE_LOSS_DECOUPLED_PPO) {
        double rp = exp(lt - lp), w = exp(lp - lo);
        double a = R * r, b = R * w * clip_d(rp, 1.0 - eps_lo, 1.0 + eps_hi);
        int inside = rp > 1.0 - eps_lo && rp < 1.0 + eps_hi;
        if (a <= b) { v = a; g = R * r; } else { v = b; g = inside ? R * w * rp : 0.0; }
    } else if (kind == ORACLE_LOSS_TIS) {
        double w = clip_d(r, 0.0, c);
        v = w * R * lt; g = w * R;
    } else if (kind == ORACLE_LOSS_CISPO) {
        double w = clip_d(r, 1.0 - eps_lo, 1.0 + eps_hi);
        v = w * R * lt; g = w * R;
    } else { /* TOPR */
        double w = R > 0.0 ? 1.0 : clip_d(r, 0.0, c);
        v = w * R * lt; g = w * R;
    }
    *value = v;
    *dvalue_dlt = g;
    *is_weight = r < c ? r : c;
}

/*
 * Whole batch of ragged responses: tokens of sequence s are offsets[s] ..
 * offsets[s+1]-1.  seq_mean[s] = (1/|o_s|) sum_t value (0 for an empty
 * sequence); batch_mean = mean of seq_mean over the non-empty sequences (the
 * E over trajectories with the 1/|o| sum over tokens of the PPO objective).
 */
void oracle_policy_loss(int kind, const float* lt, const float* lo, const float* lp, const float* R,
                        const int64_t* offsets, int n_seq, double eps_lo, double eps_hi, double c,
                        double* value, double* grad, double* is_weight, double* seq_mean,
                        double* batch_mean)
{
    double total = 0.0;
    int live = 0;
    for (int s = 0; s < n_seq; ++s) {
        double acc = 0.0;
        for (int64_t i = offsets[s]; i < offsets[s + 1]; ++i) {
            oracle_policy_loss_token(kind, (double)lt[i], (double)lo[i], lp ? (double)lp[i] : (double)lo[i],
                                     (double)R[i], eps_lo, eps_hi, c, &value[i], &grad[i], &is_weight[i]);
            acc += value[i];
        }
        int64_t n = offsets[s + 1] - offsets[s];
        seq_mean[s] = n > 0 ? acc / (double)n : 0.0;
        if (n > 0) { total += seq_mean[s]; ++live; }
    }
    *batch_mean = live ? total / live : 0.0;
}
