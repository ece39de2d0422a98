/*
 * CPU float64 oracle for the draft-model token-importance pass of speculative
 * prefill (paper: "Cross-Family Speculative Prefill", Algorithm 1 and
 * Appendix A.1).
 *
 * THIS IS TEST INFRASTRUCTURE. It is the plain definition of what the pass
 * computes, written as straight loops in double precision, and exists only so
 * that tests, the smoke check and the benchmark's CPU-baseline leg can compare
 * the GPU library against it. It shares no code, header, table or helper with
 * the GPU library and the GPU library never calls it.
 *
 * What each function follows:
 *   logits, softmax      Appendix A.1.1 (attention scores of the lookahead
 *                        tokens over the prompt, tensor [N, L, S, H])
 *   aggregation          Algorithm 1 "AggregateMaxMean"; Appendix A.1.1
 *                        (max over layers and heads, mean over lookahead), plus
 *                        the variant that averages over layers instead
 *   pooling, chunks      Algorithm 1 "AvgPool1D", "PartitionIntoChunks";
 *                        Appendix A.1.2; Appendix A.3 (kernel 13, chunk 32/128)
 *   top-k, merge         Algorithm 1 "TopKChunks", "MergeAdjacentChunks";
 *                        Section 3.1 (keep rate), Section 3.2 (merging)
 *   projection           Algorithm 1 "MapDraftChunksToTextSpans" and the target
 *                        re-tokenisation, in character-offset-interval form
 *
 * Readings of points the paper leaves open are listed where they are applied.
 * All of them are pinned by tests against closed forms, library routines and
 * brute force; none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* bfloat16 bit pattern -> double (exact: bf16 is the top half of a float32). */
static double bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int sp_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void sp_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Scaled dot-product logits of one layer (Appendix A.1.1):
 *   s[h][n][j] = scale * sum_e Q[h][n][e] * K[kv(h)][j][e],   j in [0, L)
 * Every lookahead row sees every prompt key (the lookahead tokens come after
 * the prompt, so no causal mask applies). Query head h reads kv head h / G with
 * G = H / Hkv (contiguous groups). K element (kv, j, e) sits at
 * k_layer[kv * k_stride_head + j * k_stride_token + e].
 */
int sp_oracle_logits_layer(const uint16_t *q_layer, const uint16_t *k_layer,
                           int64_t k_stride_token, int64_t k_stride_head,
                           int H, int Hkv, int n_q, int d, int64_t L,
                           double scale, double *s)
{
    if (!q_layer || !k_layer || !s || H <= 0 || Hkv <= 0 || H % Hkv != 0 ||
        n_q <= 0 || d <= 0 || L <= 0)
        return 1;
    const int G = H / Hkv;
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < H; ++h) {
        for (int n = 0; n < n_q; ++n) {
            const int kv = h / G;
            const uint16_t *qrow = q_layer + ((int64_t)h * n_q + n) * d;
            double *srow = s + ((int64_t)h * n_q + n) * L;
            for (int64_t j = 0; j < L; ++j) {
                const uint16_t *krow = k_layer + kv * k_stride_head + j * k_stride_token;
                double acc = 0.0;
                for (int e = 0; e < d; ++e)
                    acc += bf16_to_f64(qrow[e]) * bf16_to_f64(krow[e]);
                srow[j] = scale * acc;
            }
        }
    }
    return 0;
}

/*
 * Row softmax in place (Appendix A.1.1, "attention scores"): for each of
 * `rows` rows of length L,  p[j] = exp(s[j] - m) / l  with m = max_j s[j] and
 * l = sum_j exp(s[j] - m). The row is normalised over exactly the L prompt
 * keys. Optionally returns m and l per row.
 */
int sp_oracle_softmax_rows(double *s, int64_t rows, int64_t L, double *row_max, double *row_sum)
{
    if (!s || rows <= 0 || L <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double *x = s + r * L;
        double m = x[0];
        for (int64_t j = 1; j < L; ++j)
            if (x[j] > m) m = x[j];
        double l = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            x[j] = exp(x[j] - m);
            l += x[j];
        }
        for (int64_t j = 0; j < L; ++j) x[j] /= l;
        if (row_max) row_max[r] = m;
        if (row_sum) row_sum[r] = l;
    }
    return 0;
}

/*
 * Row softmax with the lookahead tokens' own keys in the normaliser
 * (Algorithm 1, the ForwardWithAttn loop: the pass of lookahead step i runs
 * after i-1 generated tokens, whose keys a causal decoder also attends to; the
 * paper does not say whether they count, so this is the second reading next to
 * sp_oracle_softmax_rows). Rows are ordered [head][n]; row (h, n) is the
 * concatenation of its L prompt logits s and its visible lookahead logits
 * sl[h][n][m], m < n + look_self (capped at n_q): softmax over that whole row,
 * of which only the prompt part is kept in s.
 */
int sp_oracle_softmax_rows_look(double *s, const double *sl, int64_t rows, int64_t L, int n_q, int look_self)
{
    if (!s || !sl || rows <= 0 || L <= 0 || n_q <= 0 || rows % n_q != 0 || (look_self != 0 && look_self != 1))
        return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double *x = s + r * L;
        const double *y = sl + r * n_q;
        int n_vis = (int)(r % n_q) + look_self;
        if (n_vis > n_q) n_vis = n_q;
        double m = x[0];
        for (int64_t j = 1; j < L; ++j)
            if (x[j] > m) m = x[j];
        for (int t = 0; t < n_vis; ++t)
            if (y[t] > m) m = y[t];
        double l = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            x[j] = exp(x[j] - m);
            l += x[j];
        }
        for (int t = 0; t < n_vis; ++t) l += exp(y[t] - m);
        for (int64_t j = 0; j < L; ++j) x[j] /= l;
    }
    return 0;
}

/*
 * Token importance I[j] (Algorithm 1 "AggregateMaxMean"; Appendix A.1.1).
 *   layer_agg == 1 (the paper's statement): max over layers and heads, then
 *       mean over the lookahead rows:  I[j] = (1/N) sum_n max_{l,h} p[l][h][n][j]
 *   layer_agg == 0 (variant): max over heads, mean over lookahead rows and
 *       layers:  I[j] = (1/(Lyr*N)) sum_l sum_n max_h p[l][h][n][j]
 * q is dense [Lyr][H][n_q][d]; k_layers[l] points at layer l's keys.
 * k_look == NULL: rows are normalised over the prompt keys only
 * (sp_oracle_softmax_rows). Otherwise k_look is dense [Lyr][Hkv][n_q][d], the
 * keys of the lookahead tokens, and rows are normalised as
 * sp_oracle_softmax_rows_look describes.
 */
int sp_oracle_score_look(const uint16_t *q, const uint16_t *const *k_layers,
                         int64_t k_stride_token, int64_t k_stride_head,
                         int Lyr, int H, int Hkv, int n_q, int d, int64_t L,
                         double scale, int layer_agg,
                         const uint16_t *k_look, int look_self, double *I)
{
    if (!q || !k_layers || !I || Lyr <= 0 || (layer_agg != 0 && layer_agg != 1)) return 1;
    const int64_t rows = (int64_t)H * n_q;
    double *p = (double *)malloc(sizeof(double) * rows * L);
    double *acc = (double *)malloc(sizeof(double) * (int64_t)n_q * L); /* per (n, j) */
    double *sl = (double *)malloc(sizeof(double) * rows * n_q);        /* lookahead logits */
    if (!p || !acc || !sl) { free(p); free(acc); free(sl); return 2; }
    for (int64_t i = 0; i < (int64_t)n_q * L; ++i) acc[i] = 0.0;

    for (int l = 0; l < Lyr; ++l) {
        int rc = sp_oracle_logits_layer(q + (int64_t)l * rows * d, k_layers[l],
                                        k_stride_token, k_stride_head,
                                        H, Hkv, n_q, d, L, scale, p);
        if (!rc && !k_look) rc = sp_oracle_softmax_rows(p, rows, L, NULL, NULL);
        if (!rc && k_look) {
            /* the lookahead keys of this layer as a key array of n_q tokens, [Hkv][n_q][d] */
            rc = sp_oracle_logits_layer(q + (int64_t)l * rows * d, k_look + (int64_t)l * Hkv * n_q * d,
                                        d, (int64_t)n_q * d, H, Hkv, n_q, d, n_q, scale, sl);
            if (!rc) rc = sp_oracle_softmax_rows_look(p, sl, rows, L, n_q, look_self);
        }
        if (rc) { free(p); free(acc); free(sl); return rc; }
#pragma omp parallel for schedule(static)
        for (int n = 0; n < n_q; ++n) {
            for (int64_t j = 0; j < L; ++j) {
                double mh = 0.0; /* probabilities are positive */
                for (int h = 0; h < H; ++h) {
                    double v = p[((int64_t)h * n_q + n) * L + j];
                    if (v > mh) mh = v;
                }
                double *a = &acc[(int64_t)n * L + j];
                if (layer_agg == 1) { if (mh > *a) *a = mh; }   /* max over layers */
                else                { *a += mh; }               /* sum over layers */
            }
        }
    }
    const double denom = (layer_agg == 1) ? (double)n_q : (double)n_q * (double)Lyr;
    for (int64_t j = 0; j < L; ++j) {
        double sum = 0.0;
        for (int n = 0; n < n_q; ++n) sum += acc[(int64_t)n * L + j];
        I[j] = sum / denom;
    }
    free(p);
    free(acc);
    free(sl);
    return 0;
}

int sp_oracle_score(const uint16_t *q, const uint16_t *const *k_layers,
                    int64_t k_stride_token, int64_t k_stride_head,
                    int Lyr, int H, int Hkv, int n_q, int d, int64_t L,
                    double scale, int layer_agg, double *I)
{
    return sp_oracle_score_look(q, k_layers, k_stride_token, k_stride_head, Lyr, H, Hkv, n_q, d, L, scale,
                                layer_agg, NULL, 0, I);
}

/*
 * Keys kept as 8-bit floating point (Section 3.1 has the deployment's KV cache in
 * fixed blocks; a quantised cache halves what the importance pass must stream).
 * Format: OCP "E4M3" (the finite-only variant): 1 sign bit, 4 exponent bits with
 * bias 7, 3 mantissa bits; exponent field 0 holds the subnormals m/8 * 2^-6; there
 * are no infinities, and only the all-ones pattern (0x7f / 0xff) is NaN, so the
 * largest finite value is 1.75 * 2^8 = 448. Every E4M3 value is exact in double.
 */
double sp_oracle_e4m3_to_f64(uint8_t b)
{
    const int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/*
 * Logits of one layer over quantised keys: the key vector of (kv, j) is
 *   kscale[kv] * E4M3(k8[kv * k_stride_head + j * k_stride_token + e]),  e in [0, d),
 * taken as exact inputs (the dequantised keys ARE the keys; nothing is rounded
 * here), and otherwise as sp_oracle_logits_layer:
 *   s[h][n][j] = scale * sum_e Q[h][n][e] * kscale[kv(h)] * E4M3(k8[...]).
 */
int sp_oracle_logits_layer_fp8(const uint16_t *q_layer, const uint8_t *k8_layer,
                               int64_t k_stride_token, int64_t k_stride_head,
                               int H, int Hkv, int n_q, int d, int64_t L,
                               const double *kscale, double scale, double *s)
{
    if (!q_layer || !k8_layer || !kscale || !s || H <= 0 || Hkv <= 0 || H % Hkv != 0 ||
        n_q <= 0 || d <= 0 || L <= 0)
        return 1;
    const int G = H / Hkv;
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < H; ++h) {
        for (int n = 0; n < n_q; ++n) {
            const int kv = h / G;
            const uint16_t *qrow = q_layer + ((int64_t)h * n_q + n) * d;
            double *srow = s + ((int64_t)h * n_q + n) * L;
            for (int64_t j = 0; j < L; ++j) {
                const uint8_t *krow = k8_layer + kv * k_stride_head + j * k_stride_token;
                double acc = 0.0;
                for (int e = 0; e < d; ++e)
                    acc += bf16_to_f64(qrow[e]) * (kscale[kv] * sp_oracle_e4m3_to_f64(krow[e]));
                srow[j] = scale * acc;
            }
        }
    }
    return 0;
}

/*
 * Token importance over quantised keys: sp_oracle_score with the logits of
 * sp_oracle_logits_layer_fp8; kscale is [Lyr][Hkv], one scale per layer and kv
 * head. Softmax over the prompt keys, head maximum, aggregation over lookahead
 * rows and layers exactly as in sp_oracle_score_look (Appendix A.1.1).
 */
int sp_oracle_score_fp8(const uint16_t *q, const uint8_t *const *k8_layers,
                        int64_t k_stride_token, int64_t k_stride_head,
                        int Lyr, int H, int Hkv, int n_q, int d, int64_t L,
                        const double *kscale, double scale, int layer_agg, double *I)
{
    if (!q || !k8_layers || !kscale || !I || Lyr <= 0 || (layer_agg != 0 && layer_agg != 1)) return 1;
    const int64_t rows = (int64_t)H * n_q;
    double *p = (double *)malloc(sizeof(double) * rows * L);
    double *acc = (double *)malloc(sizeof(double) * (int64_t)n_q * L); /* per (n, j) */
    if (!p || !acc) { free(p); free(acc); return 2; }
    for (int64_t i = 0; i < (int64_t)n_q * L; ++i) acc[i] = 0.0;
    for (int l = 0; l < Lyr; ++l) {
        int rc = sp_oracle_logits_layer_fp8(q + (int64_t)l * rows * d, k8_layers[l], k_stride_token, k_stride_head,
                                            H, Hkv, n_q, d, L, kscale + (int64_t)l * Hkv, scale, p);
        if (!rc) rc = sp_oracle_softmax_rows(p, rows, L, NULL, NULL);
        if (rc) { free(p); free(acc); return rc; }
#pragma omp parallel for schedule(static)
        for (int n = 0; n < n_q; ++n) {
            for (int64_t j = 0; j < L; ++j) {
                double mh = 0.0; /* probabilities are positive */
                for (int h = 0; h < H; ++h) {
                    double v = p[((int64_t)h * n_q + n) * L + j];
                    if (v > mh) mh = v;
                }
                double *a = &acc[(int64_t)n * L + j];
                if (layer_agg == 1) { if (mh > *a) *a = mh; }   /* max over layers */
                else                { *a += mh; }               /* sum over layers */
            }
        }
    }
    const double denom = (layer_agg == 1) ? (double)n_q : (double)n_q * (double)Lyr;
    for (int64_t j = 0; j < L; ++j) {
        double sum = 0.0;
        for (int n = 0; n < n_q; ++n) sum += acc[(int64_t)n * L + j];
        I[j] = sum / denom;
    }
    free(p);
    free(acc);
    return 0;
}

/*
 * 1-D average pooling (Algorithm 1 "AvgPool1D"; Appendix A.3: kernel 13).
 * The paper gives only the kernel size. Reading: stride 1, window centred on
 * j, output length L, zeros outside [0, L), and the divisor is always w:
 *   out[j] = (1/w) * sum_{t = j-(w-1)/2}^{j+(w-1)/2} I[t],  I[t] = 0 off the ends.
 * w must be odd.
 */
int sp_oracle_pool(const double *I, int64_t L, int w, double *out)
{
    if (!I || !out || L <= 0 || w < 1 || (w % 2) == 0) return 1;
    const int64_t half = (w - 1) / 2;
    for (int64_t j = 0; j < L; ++j) {
        double sum = 0.0;
        for (int64_t t = j - half; t <= j + half; ++t)
            if (t >= 0 && t < L) sum += I[t];
        out[j] = sum / (double)w;
    }
    return 0;
}

/*
 * Chunk means (Algorithm 1 "PartitionIntoChunks"; Appendix A.1.2): contiguous
 * chunks of c tokens; chunk i covers [i*c, min((i+1)*c, L)). A short last
 * chunk is averaged over its true size. cs has ceil(L/c) entries.
 */
int sp_oracle_chunk_mean(const double *P, int64_t L, int c, double *cs)
{
    if (!P || !cs || L <= 0 || c < 1) return 1;
    const int64_t C = (L + c - 1) / c;
    for (int64_t i = 0; i < C; ++i) {
        int64_t a = i * c, b = a + c;
        if (b > L) b = L;
        double sum = 0.0;
        for (int64_t j = a; j < b; ++j) sum += P[j];
        cs[i] = sum / (double)(b - a);
    }
    return 0;
}

/*
 * Number of chunks to keep for a keep rate rho = num/den (Section 3.1: the
 * top-K chunks are a fraction rho of the draft sequence). Reading:
 * K = clamp(ceil(C * num / den), 1, C) in integer arithmetic.
 */
int64_t sp_oracle_keep_count(int64_t C, int64_t num, int64_t den)
{
    if (C <= 0 || den <= 0 || num < 0) return -1;
    int64_t k = (C * num + den - 1) / den;
    if (k < 1) k = 1;
    if (k > C) k = C;
    return k;
}

typedef struct { double v; int64_t i; } sp_oracle_key;

static int key_cmp(const void *a, const void *b)
{
    const sp_oracle_key *x = (const sp_oracle_key *)a, *y = (const sp_oracle_key *)b;
    if (x->v > y->v) return -1;      /* larger score first */
    if (x->v < y->v) return 1;
    if (x->i < y->i) return -1;      /* equal scores: lower chunk index first */
    if (x->i > y->i) return 1;
    return 0;
}

static int i64_cmp(const void *a, const void *b)
{
    int64_t x = *(const int64_t *)a, y = *(const int64_t *)b;
    return (x > y) - (x < y);
}

/*
 * Top-k chunks (Algorithm 1 "TopKChunks"): full sort on (score descending,
 * index ascending), keep the first k, return their indices in ascending order
 * (the compressed prompt keeps the original token order, Section 2).
 */
int sp_oracle_topk(const double *cs, int64_t C, int64_t k, int64_t *sel)
{
    if (!cs || !sel || C <= 0 || k < 1 || k > C) return 1;
    sp_oracle_key *keys = (sp_oracle_key *)malloc(sizeof(sp_oracle_key) * C);
    if (!keys) return 2;
    for (int64_t i = 0; i < C; ++i) { keys[i].v = cs[i]; keys[i].i = i; }
    qsort(keys, (size_t)C, sizeof(sp_oracle_key), key_cmp);
    for (int64_t i = 0; i < k; ++i) sel[i] = keys[i].i;
    qsort(sel, (size_t)k, sizeof(int64_t), i64_cmp);
    free(keys);
    return 0;
}

/*
 * Merge adjacent kept chunks into draft-token spans (Algorithm 1
 * "MergeAdjacentChunks"; Section 3.2). sel is ascending. A maximal run of
 * consecutive chunk indices i0..i1 becomes [i0*c, min((i1+1)*c, L)).
 * Returns the number of spans; spans holds (begin, end) pairs.
 */
int64_t sp_oracle_merge(const int64_t *sel, int64_t k, int c, int64_t L, int64_t *spans)
{
    if (!sel || !spans || k < 1 || c < 1 || L <= 0) return -1;
    int64_t n = 0;
    int64_t i = 0;
    while (i < k) {
        int64_t j = i;
        while (j + 1 < k && sel[j + 1] == sel[j] + 1) ++j;
        int64_t b = sel[i] * c, e = (sel[j] + 1) * c;
        if (e > L) e = L;
        spans[2 * n] = b;
        spans[2 * n + 1] = e;
        ++n;
        i = j + 1;
    }
    return n;
}

/*
 * Projection of draft-token spans onto the target tokenisation (Algorithm 1
 * "MapDraftChunksToTextSpans" followed by target tokenisation; Section 3.1).
 * Tokenizer-free form: both tokenisations are given as character offsets into
 * the same text (draft_off[L+1], target_off[M+1]). Draft span [a, b) covers
 * characters [draft_off[a], draft_off[b]); target token t is kept iff its
 * character interval overlaps that of some span:
 *      target_off[t] < ce  and  target_off[t+1] > cs.
 * Done by brute force over every (token, span) pair. Maximal runs of kept
 * target tokens are returned as target spans (so target ranges that overlap or
 * touch are merged). mask may be NULL.
 */
int sp_oracle_project(const int64_t *draft_off, int64_t L,
                      const int64_t *target_off, int64_t M,
                      const int64_t *spans, int64_t n_spans,
                      uint8_t *mask, int64_t *tspans, int64_t *n_tspans, int64_t *n_kept)
{
    if (!draft_off || !target_off || !tspans || !n_tspans || !n_kept ||
        L <= 0 || M <= 0 || n_spans < 0 || (n_spans > 0 && !spans))
        return 1;
    uint8_t *mk = mask ? mask : (uint8_t *)malloc((size_t)M);
    if (!mk) return 2;
    for (int64_t t = 0; t < M; ++t) {
        uint8_t keep = 0;
        for (int64_t s = 0; s < n_spans && !keep; ++s) {
            int64_t a = spans[2 * s], b = spans[2 * s + 1];
            if (a < 0 || b > L || a > b) { if (!mask) free(mk); return 1; }
            int64_t cs = draft_off[a], ce = draft_off[b];
            if (target_off[t] < ce && target_off[t + 1] > cs) keep = 1;
        }
        mk[t] = keep;
    }
    int64_t n = 0, kept = 0;
    for (int64_t t = 0; t < M; ++t) {
        if (!mk[t]) continue;
        ++kept;
        if (t == 0 || !mk[t - 1]) tspans[2 * n] = t;
        if (t == M - 1 || !mk[t + 1]) { tspans[2 * n + 1] = t + 1; ++n; }
    }
    *n_tspans = n;
    *n_kept = kept;
    if (!mask) free(mk);
    return 0;
}

/*
 * Compressed target prompt in token-id form (paper: Algorithm 1, "ConcatWithDelim", the target
 * tokenisation of the compressed text and the new contiguous position ids; Section 3.2;
 * Appendix A.3 for the delimiters used). With the target tokenisation of the original text given
 * as ids, the kept ranges [b, e) of target tokens are copied in order and the delimiter's ids are
 * put between consecutive ranges (not before the first, not after the last). out_src[i] is the
 * original target index of output token i, -1 for delimiter tokens; out_pos[i] = i.
 * Buffers must hold sum(e - b) + (n_tspans - 1) * n_delim entries. Returns 0, or 1 on bad arguments.
 */
int sp_oracle_assemble(const int32_t *target_ids, int64_t M, const int64_t *tspans, int64_t n_tspans,
                       const int32_t *delim, int64_t n_delim,
                       int32_t *out_ids, int32_t *out_pos, int64_t *out_src, int64_t *out_len)
{
    if (!target_ids || M <= 0 || n_tspans < 0 || n_delim < 0 || !out_len ||
        (n_tspans > 0 && !tspans) || (n_delim > 0 && !delim))
        return 1;
    int64_t n = 0;
    for (int64_t r = 0; r < n_tspans; ++r) {
        const int64_t b = tspans[2 * r], e = tspans[2 * r + 1];
        if (b < 0 || e > M || b > e) return 1;
        if (r > 0) {
            for (int64_t j = 0; j < n_delim; ++j) {
                if (out_ids) out_ids[n] = delim[j];
                if (out_src) out_src[n] = -1;
                if (out_pos) out_pos[n] = (int32_t)n;
                ++n;
            }
        }
        for (int64_t t = b; t < e; ++t) {
            if (out_ids) out_ids[n] = target_ids[t];
            if (out_src) out_src[n] = t;
            if (out_pos) out_pos[n] = (int32_t)n;
            ++n;
        }
    }
    *out_len = n;
    return 0;
}
