/*
 * lt_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what the LightTransfer hot path computes:
 * decode attention in a hybrid layer stack (full attention / streaming attention
 * over sink + recent tokens), the lazy ratio of a layer, the choice of lazy layers,
 * and the prefill attention whose log-sum-exp the lazy ratio can reuse.  It exists only so that tests, the smoke check and the benchmark's CPU
 * baseline can compare the GPU library against the paper's definitions.  Nothing
 * in the product path may call it, and it shares no code with the GPU path.
 *
 * Every function works positionally on the WHOLE token history of a layer: there
 * is no ring buffer, no splitting of the key axis, no blocking and no fusion here.
 * Inputs are bf16 bit patterns (uint16_t); every product, sum, exponential and
 * logarithm is taken in double precision.
 *
 * Pins (tests/test_oracle_*.py): closed forms for uniform keys, shift invariance,
 * rows of the softmax summing to one, streaming == full when the window covers the
 * history, one dominant key, the identity |s1 - s1~|_1 = 1 - rho and the bound of
 * the paper's streaming-attention lemma, agreement of the probability-sum and the
 * log-sum-exp forms of the lazy ratio, brute force against an explicit N x N masked
 * softmax built from library routines, and queue simulation == sort for selection;
 * prefill rows against the decode function on the truncated history and against the
 * library form of the whole masked softmax, the ratio from a supplied log-sum-exp
 * against the two self-contained forms.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define LTO_OK 0
#define LTO_ERR_ARG 1
#define LTO_ERR_NOMEM 2

#define LTO_MODE_FULL 0
#define LTO_MODE_LAZY 1

#define LTO_RECENT_PER_QUERY 0
#define LTO_RECENT_FIXED 1

static double bf16_bits_to_double(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Appendix "Theoretical Analysis": the causal mask keeps j <= i; the sink mask keeps,
 * for the query at position p, the first w_sink positions and the last w_recent
 * positions ending at p (p itself included).  Both sets are sets: a position that is
 * both an initial and a recent token is counted once. */
static int in_streaming_set(int64_t j, int64_t p, int64_t w_sink, int64_t w_recent)
{
    if (j < 0 || j > p) return 0;
    if (j < w_sink) return 1;
    if (j > p - w_recent) return 1;
    return 0;
}

/* Table 1 reading: the recent tokens are the last w_recent tokens of the prompt
 * (the same for every query), intersected with the causal set of the query. */
static int in_fixed_set(int64_t j, int64_t p, int64_t n, int64_t w_sink, int64_t w_recent)
{
    if (j < 0 || j > p) return 0;
    if (j < w_sink) return 1;
    if (j >= n - w_recent) return 1;
    return 0;
}

static double dot_qk(const uint16_t *q, const uint16_t *k, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += bf16_bits_to_double(q[c]) * bf16_bits_to_double(k[c]);
    return s;
}

/*
 * Decode attention of one layer for the newest token (Preliminary, "Decoding";
 * Appendix "Theoretical Analysis", softmax(q K^T + M) V with M the causal mask for a
 * full layer and the sink mask for a lazy layer).
 *
 *   q      [B, Hq, d]      query of the token at position T-1
 *   K, V   [B, Hkv, T, d]  the layer's whole history, the newest token included
 *   mode   LTO_MODE_FULL: attend to 0..T-1;  LTO_MODE_LAZY: first w_sink and last w_recent
 *   out    [B, Hq, d]      softmax-weighted mean of V
 *   lse    [B, Hq]         log of the softmax denominator (may be NULL)
 *   probs  [B, Hq, T]      attention weights, 0 outside the attended set (may be NULL)
 *
 * Query head h reads KV head h / (Hq / Hkv).
 */
int lto_decode_attn(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                    int B, int Hq, int Hkv, int d, int64_t T,
                    int mode, int64_t w_sink, int64_t w_recent, double scale,
                    double *out, double *lse, double *probs)
{
    if (!q || !K || !V || !out) return LTO_ERR_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || T <= 0) return LTO_ERR_ARG;
    if (Hq % Hkv != 0) return LTO_ERR_ARG;
    if (mode != LTO_MODE_FULL && mode != LTO_MODE_LAZY) return LTO_ERR_ARG;
    if (w_sink < 0 || w_recent < 0) return LTO_ERR_ARG;
    if (mode == LTO_MODE_LAZY && w_sink + w_recent == 0) return LTO_ERR_ARG;
    const int G = Hq / Hkv;
    const int64_t p = T - 1;
    int status = LTO_OK;

#pragma omp parallel for schedule(dynamic)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, g = h / G;
        const uint16_t *qv = q + ((size_t)b * Hq + h) * d;
        const uint16_t *Kb = K + ((size_t)b * Hkv + g) * (size_t)T * d;
        const uint16_t *Vb = V + ((size_t)b * Hkv + g) * (size_t)T * d;
        double *s = (double *)malloc((size_t)T * sizeof(double));
        double *o = out + ((size_t)b * Hq + h) * d;
        if (!s) {
#pragma omp critical
            status = LTO_ERR_NOMEM;
            continue;
        }
        double m = -INFINITY;
        for (int64_t j = 0; j < T; ++j) {
            const int keep = (mode == LTO_MODE_FULL) ? 1 : in_streaming_set(j, p, w_sink, w_recent);
            if (!keep) { s[j] = -INFINITY; continue; }
            s[j] = scale * dot_qk(qv, Kb + (size_t)j * d, d);
            if (s[j] > m) m = s[j];
        }
        double Z = 0.0;
        for (int64_t j = 0; j < T; ++j) if (s[j] != -INFINITY) Z += exp(s[j] - m);
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int64_t j = 0; j < T; ++j) {
            const double pj = (s[j] == -INFINITY) ? 0.0 : exp(s[j] - m) / Z;
            if (probs) probs[((size_t)b * Hq + h) * (size_t)T + j] = pj;
            if (pj == 0.0) continue;
            const uint16_t *vj = Vb + (size_t)j * d;
            for (int c = 0; c < d; ++c) o[c] += pj * bf16_bits_to_double(vj[c]);
        }
        if (lse) lse[(size_t)b * Hq + h] = m + log(Z);
        free(s);
    }
    return status;
}

/*
 * Lazy ratio of one layer, probability-sum form (Eq. 1): for each of the last w
 * prompt positions p = n-w .. n-1 and each head, the causal softmax row of that query
 * is formed over keys 0..p and the weights falling on the initial and recent tokens
 * are added up; the ratio is the mean over queries and heads (the attention weight in
 * Eq. 1 is the head average), then over the sequences of the batch.
 *
 *   q_last [B, Hq, w, d]   queries of prompt positions n-w .. n-1
 *   K      [B, Hkv, n, d]  prompt keys
 *   rho    [B, Hq, w]      per (sequence, head, query) mass (may be NULL)
 *   r_seq  [B]             per-sequence mean (may be NULL)
 *   r      [1]             batch mean
 */
int lto_lazy_ratio(const uint16_t *q_last, const uint16_t *K,
                   int B, int Hq, int Hkv, int d, int64_t n, int w,
                   int64_t w_sink, int64_t w_recent, double scale, int recent_mode,
                   double *rho, double *r_seq, double *r)
{
    if (!q_last || !K || !r) return LTO_ERR_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || n <= 0 || w <= 0 || w > n) return LTO_ERR_ARG;
    if (Hq % Hkv != 0 || w_sink < 0 || w_recent < 0) return LTO_ERR_ARG;
    if (recent_mode != LTO_RECENT_PER_QUERY && recent_mode != LTO_RECENT_FIXED) return LTO_ERR_ARG;
    const int G = Hq / Hkv;
    double *rho_all = (double *)malloc((size_t)B * Hq * w * sizeof(double));
    if (!rho_all) return LTO_ERR_NOMEM;
    int status = LTO_OK;

#pragma omp parallel for schedule(dynamic)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, g = h / G;
        const uint16_t *Kb = K + ((size_t)b * Hkv + g) * (size_t)n * d;
        double *s = (double *)malloc((size_t)n * sizeof(double));
        if (!s) {
#pragma omp critical
            status = LTO_ERR_NOMEM;
            continue;
        }
        for (int t = 0; t < w; ++t) {
            const int64_t p = n - w + t;
            const uint16_t *qv = q_last + (((size_t)b * Hq + h) * w + t) * d;
            double m = -INFINITY;
            for (int64_t j = 0; j <= p; ++j) {
                s[j] = scale * dot_qk(qv, Kb + (size_t)j * d, d);
                if (s[j] > m) m = s[j];
            }
            double Z = 0.0;
            for (int64_t j = 0; j <= p; ++j) Z += exp(s[j] - m);
            double mass = 0.0;
            for (int64_t j = 0; j <= p; ++j) {
                const int keep = (recent_mode == LTO_RECENT_PER_QUERY)
                                     ? in_streaming_set(j, p, w_sink, w_recent)
                                     : in_fixed_set(j, p, n, w_sink, w_recent);
                if (keep) mass += exp(s[j] - m) / Z;
            }
            rho_all[((size_t)b * Hq + h) * w + t] = mass;
        }
        free(s);
    }
    if (status == LTO_OK) {
        double total = 0.0;
        for (int b = 0; b < B; ++b) {
            double acc = 0.0;
            for (int i = 0; i < Hq * w; ++i) acc += rho_all[(size_t)b * Hq * w + i];
            acc /= (double)Hq * (double)w;
            if (r_seq) r_seq[b] = acc;
            total += acc;
        }
        *r = total / (double)B;
        if (rho) memcpy(rho, rho_all, (size_t)B * Hq * w * sizeof(double));
    }
    free(rho_all);
    return status;
}

/* log(sum_j exp(s_j)) over the positions j of 0..p for which keep[j] != 0. */
static double masked_logsumexp(const double *s, const unsigned char *keep, int64_t p)
{
    double m = -INFINITY;
    for (int64_t j = 0; j <= p; ++j) if (keep[j] && s[j] > m) m = s[j];
    if (m == -INFINITY) return -INFINITY;
    double Z = 0.0;
    for (int64_t j = 0; j <= p; ++j) if (keep[j]) Z += exp(s[j] - m);
    return m + log(Z);
}

/*
 * Lazy ratio, log-sum-exp form (Table 1): log rho = LSE over the initial and recent
 * keys minus the LSE of the whole causal row; rho = exp(log rho).  Same arguments and
 * outputs as lto_lazy_ratio; log_rho [B, Hq, w] (may be NULL) returns the differences.
 */
int lto_lazy_ratio_lse(const uint16_t *q_last, const uint16_t *K,
                       int B, int Hq, int Hkv, int d, int64_t n, int w,
                       int64_t w_sink, int64_t w_recent, double scale, int recent_mode,
                       double *log_rho, double *r_seq, double *r)
{
    if (!q_last || !K || !r) return LTO_ERR_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || n <= 0 || w <= 0 || w > n) return LTO_ERR_ARG;
    if (Hq % Hkv != 0 || w_sink < 0 || w_recent < 0) return LTO_ERR_ARG;
    if (recent_mode != LTO_RECENT_PER_QUERY && recent_mode != LTO_RECENT_FIXED) return LTO_ERR_ARG;
    const int G = Hq / Hkv;
    double *lr_all = (double *)malloc((size_t)B * Hq * w * sizeof(double));
    if (!lr_all) return LTO_ERR_NOMEM;
    int status = LTO_OK;

#pragma omp parallel for schedule(dynamic)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, g = h / G;
        const uint16_t *Kb = K + ((size_t)b * Hkv + g) * (size_t)n * d;
        double *s = (double *)malloc((size_t)n * sizeof(double));
        unsigned char *all = (unsigned char *)malloc((size_t)n);
        unsigned char *win = (unsigned char *)malloc((size_t)n);
        if (!s || !all || !win) {
#pragma omp critical
            status = LTO_ERR_NOMEM;
            free(s); free(all); free(win);
            continue;
        }
        for (int t = 0; t < w; ++t) {
            const int64_t p = n - w + t;
            const uint16_t *qv = q_last + (((size_t)b * Hq + h) * w + t) * d;
            for (int64_t j = 0; j <= p; ++j) {
                s[j] = scale * dot_qk(qv, Kb + (size_t)j * d, d);
                all[j] = 1;
                win[j] = (unsigned char)((recent_mode == LTO_RECENT_PER_QUERY)
                                             ? in_streaming_set(j, p, w_sink, w_recent)
                                             : in_fixed_set(j, p, n, w_sink, w_recent));
            }
            lr_all[((size_t)b * Hq + h) * w + t] = masked_logsumexp(s, win, p) - masked_logsumexp(s, all, p);
        }
        free(s); free(all); free(win);
    }
    if (status == LTO_OK) {
        double total = 0.0;
        for (int b = 0; b < B; ++b) {
            double acc = 0.0;
            for (int i = 0; i < Hq * w; ++i) acc += exp(lr_all[(size_t)b * Hq * w + i]);
            acc /= (double)Hq * (double)w;
            if (r_seq) r_seq[b] = acc;
            total += acc;
        }
        *r = total / (double)B;
        if (log_rho) memcpy(log_rho, lr_all, (size_t)B * Hq * w * sizeof(double));
    }
    free(lr_all);
    return status;
}

/*
 * Lazy ratio from a log-sum-exp that the prefill attention already produced (Table 1:
 * the LSE of the window logits minus the prefill kernel's LSE of the whole causal row).
 * Only the initial and recent keys of each query are touched.
 *
 *   lse_rows [B, Hq, w]   natural-log LSE of the causal rows n-w .. n-1 (scale included)
 *
 * Other arguments and outputs as lto_lazy_ratio_lse.
 */
int lto_lazy_ratio_from_lse(const uint16_t *q_last, const uint16_t *K, const double *lse_rows,
                            int B, int Hq, int Hkv, int d, int64_t n, int w,
                            int64_t w_sink, int64_t w_recent, double scale, int recent_mode,
                            double *log_rho, double *r_seq, double *r)
{
    if (!q_last || !K || !lse_rows || !r) return LTO_ERR_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || n <= 0 || w <= 0 || w > n) return LTO_ERR_ARG;
    if (Hq % Hkv != 0 || w_sink < 0 || w_recent < 0) return LTO_ERR_ARG;
    if (recent_mode != LTO_RECENT_PER_QUERY && recent_mode != LTO_RECENT_FIXED) return LTO_ERR_ARG;
    const int G = Hq / Hkv;
    double *lr_all = (double *)malloc((size_t)B * Hq * w * sizeof(double));
    if (!lr_all) return LTO_ERR_NOMEM;

    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, g = h / G;
        const uint16_t *Kb = K + ((size_t)b * Hkv + g) * (size_t)n * d;
        for (int t = 0; t < w; ++t) {
            const int64_t p = n - w + t;
            const uint16_t *qv = q_last + (((size_t)b * Hq + h) * w + t) * d;
            /* logits of the kept keys only, then their log-sum-exp */
            double m = -INFINITY, Z = 0.0;
            for (int pass = 0; pass < 2; ++pass) {
                for (int64_t j = 0; j <= p; ++j) {
                    const int keep = (recent_mode == LTO_RECENT_PER_QUERY)
                                         ? in_streaming_set(j, p, w_sink, w_recent)
                                         : in_fixed_set(j, p, n, w_sink, w_recent);
                    if (!keep) continue;
                    const double sj = scale * dot_qk(qv, Kb + (size_t)j * d, d);
                    if (pass == 0) { if (sj > m) m = sj; }
                    else Z += exp(sj - m);
                }
            }
            const double lse_window = (m == -INFINITY) ? -INFINITY : m + log(Z);
            lr_all[((size_t)b * Hq + h) * w + t] = lse_window - lse_rows[((size_t)b * Hq + h) * w + t];
        }
    }
    double total = 0.0;
    for (int b = 0; b < B; ++b) {
        double acc = 0.0;
        for (int i = 0; i < Hq * w; ++i) acc += exp(lr_all[(size_t)b * Hq * w + i]);
        acc /= (double)Hq * (double)w;
        if (r_seq) r_seq[b] = acc;
        total += acc;
    }
    *r = total / (double)B;
    if (log_rho) memcpy(log_rho, lr_all, (size_t)B * Hq * w * sizeof(double));
    free(lr_all);
    return LTO_OK;
}

/*
 * Prefill attention of one layer over a whole prompt (Preliminary, "Prefilling":
 * every position attends to itself and the positions before it; Appendix "Theoretical
 * Analysis": softmax(Q K^T + M) V with M the causal mask, or the sink mask for a layer
 * that runs streaming attention from the start, as LightTransfer-Train's lazy layers do).
 *
 *   Q      [B, Hq, n, d]    K, V  [B, Hkv, n, d]
 *   mode   LTO_MODE_FULL: row p attends 0..p;  LTO_MODE_LAZY: first w_sink and last w_recent of 0..p
 *   out    [B, Hq, n, d]    softmax-weighted mean of V per row
 *   lse    [B, Hq, n]       log of each row's softmax denominator (may be NULL)
 *   absw   [B, Hq, n, d]    sum_j p_j |V_j| per row and channel (may be NULL): the scale of the
 *                           rounding error of an implementation that rounds the weights
 */
int lto_prefill_attn(const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                     int B, int Hq, int Hkv, int d, int64_t n,
                     int mode, int64_t w_sink, int64_t w_recent, double scale,
                     double *out, double *lse, double *absw)
{
    if (!Q || !K || !V || !out) return LTO_ERR_ARG;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || n <= 0) return LTO_ERR_ARG;
    if (Hq % Hkv != 0) return LTO_ERR_ARG;
    if (mode != LTO_MODE_FULL && mode != LTO_MODE_LAZY) return LTO_ERR_ARG;
    if (w_sink < 0 || w_recent < 0) return LTO_ERR_ARG;
    if (mode == LTO_MODE_LAZY && w_sink + w_recent == 0) return LTO_ERR_ARG;
    const int G = Hq / Hkv;
    int status = LTO_OK;

#pragma omp parallel for schedule(dynamic)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, g = h / G;
        const uint16_t *Kb = K + ((size_t)b * Hkv + g) * (size_t)n * d;
        const uint16_t *Vb = V + ((size_t)b * Hkv + g) * (size_t)n * d;
        double *w = (double *)malloc((size_t)n * sizeof(double));
        if (!w) {
#pragma omp critical
            status = LTO_ERR_NOMEM;
            continue;
        }
        for (int64_t p = 0; p < n; ++p) {
            const uint16_t *qv = Q + (((size_t)b * Hq + h) * (size_t)n + p) * d;
            double *o = out + (((size_t)b * Hq + h) * (size_t)n + p) * d;
            double *a = absw ? absw + (((size_t)b * Hq + h) * (size_t)n + p) * d : NULL;
            /* row p of Q K^T + M, then its softmax */
            double m = -INFINITY;
            for (int64_t j = 0; j <= p; ++j) {
                const int keep = (mode == LTO_MODE_FULL) ? 1 : in_streaming_set(j, p, w_sink, w_recent);
                w[j] = keep ? scale * dot_qk(qv, Kb + (size_t)j * d, d) : -INFINITY;
                if (w[j] > m) m = w[j];
            }
            double Z = 0.0;
            for (int64_t j = 0; j <= p; ++j) { w[j] = exp(w[j] - m); Z += w[j]; }
            for (int c = 0; c < d; ++c) { o[c] = 0.0; if (a) a[c] = 0.0; }
            for (int64_t j = 0; j <= p; ++j) {
                const double pj = w[j] / Z;
                if (pj == 0.0) continue;
                const uint16_t *vj = Vb + (size_t)j * d;
                for (int c = 0; c < d; ++c) {
                    const double v = bf16_bits_to_double(vj[c]);
                    o[c] += pj * v;
                    if (a) a[c] += pj * fabs(v);
                }
            }
            if (lse) lse[((size_t)b * Hq + h) * (size_t)n + p] = m + log(Z);
        }
        free(w);
    }
    return status;
}

/* 1 when layer a is "lazier" than layer b: larger ratio, ties to the lower index. */
static int lazier(const double *r, int a, int b)
{
    if (r[a] != r[b]) return r[a] > r[b];
    return a < b;
}

/*
 * Lazy-layer selection, closed form (Section "LightTransfer-Test"): the n_lazy layers
 * with the largest lazy ratios are lazy, the other P = L - n_lazy keep full attention.
 * order[L] lists the layers from laziest to least lazy (may be NULL).
 */
int lto_select_lazy(const double *r, int L, int n_lazy, unsigned char *is_lazy, int *order)
{
    if (!r || !is_lazy || L <= 0 || n_lazy < 0 || n_lazy > L) return LTO_ERR_ARG;
    for (int i = 0; i < L; ++i) if (r[i] != r[i]) return LTO_ERR_ARG;
    int *idx = (int *)malloc((size_t)L * sizeof(int));
    if (!idx) return LTO_ERR_NOMEM;
    for (int i = 0; i < L; ++i) idx[i] = i;
    for (int i = 1; i < L; ++i) {          /* insertion sort: L is the layer count */
        int v = idx[i], k = i - 1;
        while (k >= 0 && lazier(r, v, idx[k])) { idx[k + 1] = idx[k]; --k; }
        idx[k + 1] = v;
    }
    for (int i = 0; i < L; ++i) is_lazy[i] = 0;
    for (int i = 0; i < n_lazy; ++i) is_lazy[idx[i]] = 1;
    if (order) memcpy(order, idx, (size_t)L * sizeof(int));
    free(idx);
    return LTO_OK;
}

/*
 * Lazy-layer selection as the paper runs it during prefill: a max-priority queue of
 * capacity P = L - n_lazy receives (ratio, layer) after each layer, in layer order;
 * whenever it holds more than P entries the entry with the highest ratio is removed
 * and that layer becomes lazy.  pop_step[i] (may be NULL) is the layer index whose
 * push caused layer i to be removed, or -1 if layer i keeps full attention.
 */
int lto_select_lazy_queue(const double *r, int L, int n_lazy, unsigned char *is_lazy, int *pop_step)
{
    if (!r || !is_lazy || L <= 0 || n_lazy < 0 || n_lazy > L) return LTO_ERR_ARG;
    for (int i = 0; i < L; ++i) if (r[i] != r[i]) return LTO_ERR_ARG;
    const int P = L - n_lazy;
    int *queue = (int *)malloc((size_t)(P + 1) * sizeof(int));
    if (!queue) return LTO_ERR_NOMEM;
    int size = 0;
    for (int i = 0; i < L; ++i) { is_lazy[i] = 0; if (pop_step) pop_step[i] = -1; }
    for (int i = 0; i < L; ++i) {
        queue[size++] = i;
        if (size > P) {
            int top = 0;
            for (int k = 1; k < size; ++k) if (lazier(r, queue[k], queue[top])) top = k;
            const int layer = queue[top];
            queue[top] = queue[--size];
            is_lazy[layer] = 1;
            if (pop_step) pop_step[layer] = i;
        }
    }
    free(queue);
    return LTO_OK;
}

/* Threads the parallel loops above will use (1 when built without OpenMP). */
/*
 * LightTransfer-Train pre-selection: every training sample, fed with question and answer,
 * yields its own set of lazy layers; a layer's frequency is the number of samples that chose
 * it, and the n_lazy most frequent layers become the fixed lazy set (equal frequencies go to
 * the lower layer index, the rule of the priority queue).
 *
 *   sets     [S, L]  1 where sample s chose layer l
 *   count    [L]     frequency of every layer (may be NULL)
 *   is_lazy  [L]     1 for the selected layers
 */
int lto_preselect_lazy(const unsigned char *sets, int S, int L, int n_lazy, int *count, unsigned char *is_lazy)
{
    if (!sets || !is_lazy || S <= 0 || L <= 0 || n_lazy < 0 || n_lazy > L) return LTO_ERR_ARG;
    int *freq = (int *)calloc((size_t)L, sizeof(int));
    if (!freq) return LTO_ERR_NOMEM;
    for (int s = 0; s < S; ++s)
        for (int l = 0; l < L; ++l)
            if (sets[(size_t)s * L + l]) freq[l] += 1;
    memset(is_lazy, 0, (size_t)L);
    for (int pick = 0; pick < n_lazy; ++pick) {
        int best = -1;
        for (int l = 0; l < L; ++l) {
            if (is_lazy[l]) continue;
            if (best < 0 || freq[l] > freq[best]) best = l;     /* strict: the first of equals stays */
        }
        is_lazy[best] = 1;
    }
    if (count) memcpy(count, freq, (size_t)L * sizeof(int));
    free(freq);
    return LTO_OK;
}

#ifdef _OPENMP
#include <omp.h>
int lto_num_threads(void) { return omp_get_max_threads(); }
void lto_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int lto_num_threads(void) { return 1; }
void lto_set_num_threads(int n) { (void)n; }
#endif
