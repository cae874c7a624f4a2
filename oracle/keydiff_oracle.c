/*
 * KeyDiff block-prefill ORACLE -- test infrastructure, not product code.
 *
 * A plain, slow, host-only statement of what one block step computes, written
 * from the paper's equations so that it can be checked against them by eye.
 * Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
 * call it.  It shares no code with the HIP path and is never a fallback for it.
 *
 * Inputs are bf16 bit patterns (uint16_t); every bf16 value is converted to
 * double exactly and all arithmetic is IEEE double (compile with
 * -ffp-contract=off).  One sequence per call; KV heads are independent.
 *
 * Step order per block (Background, Fig. 1: (1) K/V of the block are inputs,
 * (2) attention, (3) eviction score, (4) eviction):
 *   append    Eq. 5   (block prompt processing): C_i <- [K_{i-1} || k_block]
 *   attention Eq. 1-2 : softmax(q K^T / sqrt(d) + M) V over cache || block
 *   anchor    Method, "Efficient Variant": mean of the keys (raw keys: the
 *             variant the paper says it evaluates; unit keys: Eq. 7 literally)
 *   score     Appendix "FLOP count of KeyDiff": s_i = mu.k_i / max(|mu||k_i|, eps)
 *   select    Eq. 6/7 + Fig. 3 (3): keep the N keys with the LOWEST similarity
 *   compact   Eq. 6: K' = gather(K, S), V' = gather(V, S)
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - the anchor is taken over all n = len + Bt rows (Method: "intermediate size n");
 *   - eps = 1e-8 unless given, applied to the product of the norms as printed;
 *   - the score that decides is the double result rounded once to float;
 *     ties in that float keep the LOWER token position;
 *   - survivors are stored in ascending token position;
 *   - nothing is evicted while n <= N (Background, "KV Cache Eviction Methods");
 *   - sliding window: the W highest positions are exempt (Method, "KeyDiff with
 *     Sliding Window"), the rest of the budget goes to the lowest scores;
 *   - unit-key anchor: a zero key contributes a zero vector.
 *
 * Parity pins (tests/test_oracle_*.py): closed-form hand examples, brute-force
 * argsort, the pairwise row-sum identity of Eq. 6 vs Eq. 7, one-shot causal
 * attention for B = T, invariances, the op-count closed form.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KDO_EXPORT __attribute__((visibility("default")))

static double bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* ------------------------------------------------------------------ attention
 * Eq. 1-2.  q [hq][Bt][d]; K, V [hkv][cap][d] with the block already appended at
 * rows [len, len + Bt).  Block query j sees every cached row and block rows
 * 0..j (the mask M "accounting for both the KV cache and" the new tokens).
 * Query head h reads KV head h / (hq / hkv).  out [hq][Bt][d] float.          */
KDO_EXPORT void kdo_attention(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                              int hq, int hkv, int d, int cap, int len, int Bt,
                              double scale, float *out)
{
    const int G = hq / hkv;
    const int n = len + Bt;
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < hq; ++h) {
        for (int j = 0; j < Bt; ++j) {
            const int g = h / G;
            const uint16_t *qr = q + ((size_t)h * Bt + j) * d;
            const uint16_t *Kh = K + (size_t)g * cap * d;
            const uint16_t *Vh = V + (size_t)g * cap * d;
            const int visible = len + j + 1; /* rows [0, visible) */
            double *logit = (double *)malloc(sizeof(double) * (size_t)n);
            double *acc = (double *)calloc((size_t)d, sizeof(double));
            double mx = -INFINITY;
            for (int i = 0; i < visible; ++i) {
                double s = 0.0;
                for (int c = 0; c < d; ++c)
                    s += bf16_to_f64(qr[c]) * bf16_to_f64(Kh[(size_t)i * d + c]);
                logit[i] = s * scale;
                if (logit[i] > mx) mx = logit[i];
            }
            double denom = 0.0;
            for (int i = 0; i < visible; ++i) {
                logit[i] = exp(logit[i] - mx);
                denom += logit[i];
            }
            for (int i = 0; i < visible; ++i) {
                const double p = logit[i] / denom;
                for (int c = 0; c < d; ++c)
                    acc[c] += p * bf16_to_f64(Vh[(size_t)i * d + c]);
            }
            float *o = out + ((size_t)h * Bt + j) * d;
            for (int c = 0; c < d; ++c) o[c] = (float)acc[c];
            free(acc);
            free(logit);
        }
    }
}

/* --------------------------------------------------------------------- anchor
 * One KV head, rows Kh [n][d].  mode 0: mu = (1/n) sum k_i (mean of the keys,
 * Fig. 3 (1)).  mode 1: mu = (1/n) sum k_i / |k_i| (Eq. 7).                    */
KDO_EXPORT void kdo_anchor(const uint16_t *Kh, int n, int d, int mode, double *mu)
{
    for (int c = 0; c < d; ++c) mu[c] = 0.0;
    for (int i = 0; i < n; ++i) {
        double inv = 1.0;
        if (mode == 1) {
            double k2 = 0.0;
            for (int c = 0; c < d; ++c) {
                const double x = bf16_to_f64(Kh[(size_t)i * d + c]);
                k2 += x * x;
            }
            const double nk = sqrt(k2);
            inv = nk > 0.0 ? 1.0 / nk : 0.0;
        }
        for (int c = 0; c < d; ++c) {
            const double x = bf16_to_f64(Kh[(size_t)i * d + c]);
            mu[c] += (mode == 1) ? x * inv : x;
        }
    }
    for (int c = 0; c < d; ++c) mu[c] /= (double)n;
}

/* ---------------------------------------------------------------------- score
 * s_i = (mu . k_i) / max(|mu| * |k_i|, eps), for every row.  s64 (nullable)
 * receives the double, s32 that double rounded once to float -- the value the
 * selection is decided on.                                                     */
KDO_EXPORT void kdo_scores(const uint16_t *Kh, int n, int d, const double *mu, double eps,
                           double *s64, float *s32)
{
    double mu2 = 0.0;
    for (int c = 0; c < d; ++c) mu2 += mu[c] * mu[c];
    const double nmu = sqrt(mu2);
    for (int i = 0; i < n; ++i) {
        double dot = 0.0, k2 = 0.0;
        for (int c = 0; c < d; ++c) {
            const double x = bf16_to_f64(Kh[(size_t)i * d + c]);
            dot += mu[c] * x;
            k2 += x * x;
        }
        double den = nmu * sqrt(k2);
        if (den < eps) den = eps;
        const double s = dot / den;
        if (s64) s64[i] = s;
        if (s32) s32[i] = (float)s;
    }
}

/* --------------------------------------------------------------------- select
 * Keep `keep` of the n rows: the W rows with the highest position are exempt
 * (always kept); of the others the keep - W with the lowest score are kept,
 * ties broken towards the lower position.  kept[] receives the kept row indices
 * ordered by ascending position.                                               */
typedef struct {
    float s;
    int32_t pos;
    int32_t row;
} kdo_item;

static int cmp_score_then_pos(const void *a, const void *b)
{
    const kdo_item *x = (const kdo_item *)a, *y = (const kdo_item *)b;
    if (x->s < y->s) return -1;
    if (x->s > y->s) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

static int cmp_pos(const void *a, const void *b)
{
    const kdo_item *x = (const kdo_item *)a, *y = (const kdo_item *)b;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

KDO_EXPORT void kdo_select(const float *s32, const int32_t *pos, int n, int keep, int window_W,
                           int32_t *kept)
{
    kdo_item *it = (kdo_item *)malloc(sizeof(kdo_item) * (size_t)n);
    for (int i = 0; i < n; ++i) {
        it[i].s = s32[i];
        it[i].pos = pos[i];
        it[i].row = i;
    }
    if (keep >= n) {
        qsort(it, (size_t)n, sizeof *it, cmp_pos);
        for (int i = 0; i < n; ++i) kept[i] = it[i].row;
        free(it);
        return;
    }
    if (window_W > keep) window_W = keep;
    /* the window: the W highest positions go to the tail of the array */
    qsort(it, (size_t)n, sizeof *it, cmp_pos);
    const int cand = n - window_W;
    /* among the candidates, lowest score first (then lower position) */
    qsort(it, (size_t)cand, sizeof *it, cmp_score_then_pos);
    const int from_cand = keep - window_W;
    /* survivors = first from_cand candidates + the window */
    memmove(it + from_cand, it + cand, sizeof(kdo_item) * (size_t)window_W);
    qsort(it, (size_t)keep, sizeof *it, cmp_pos);
    for (int i = 0; i < keep; ++i) kept[i] = it[i].row;
    free(it);
}

/* ------------------------------------------------------------ one sequence's state */
typedef struct {
    int hq, hkv, d, N, B, mode, W;
    double eps, scale;
    int len;
    uint16_t *K, *V; /* [hkv][N + B][d] */
    int32_t *pos;    /* [hkv][N + B]    */
} kdo_state;

KDO_EXPORT kdo_state *kdo_new(int hq, int hkv, int d, int N, int B, int mode, int W, double eps,
                              double scale)
{
    kdo_state *s = (kdo_state *)calloc(1, sizeof *s);
    s->hq = hq; s->hkv = hkv; s->d = d; s->N = N; s->B = B; s->mode = mode; s->W = W;
    s->eps = eps > 0.0 ? eps : 1e-8;
    s->scale = scale > 0.0 ? scale : 1.0 / sqrt((double)d);
    s->len = 0; /* C_0 is empty (Eq. 5) */
    const size_t cap = (size_t)N + (size_t)B;
    s->K = (uint16_t *)calloc((size_t)hkv * cap * d, sizeof(uint16_t));
    s->V = (uint16_t *)calloc((size_t)hkv * cap * d, sizeof(uint16_t));
    s->pos = (int32_t *)calloc((size_t)hkv * cap, sizeof(int32_t));
    return s;
}

KDO_EXPORT void kdo_free(kdo_state *s)
{
    if (!s) return;
    free(s->K); free(s->V); free(s->pos); free(s);
}

KDO_EXPORT int kdo_len(const kdo_state *s) { return s->len; }
KDO_EXPORT const uint16_t *kdo_K(const kdo_state *s) { return s->K; }
KDO_EXPORT const uint16_t *kdo_V(const kdo_state *s) { return s->V; }
KDO_EXPORT const int32_t *kdo_pos(const kdo_state *s) { return s->pos; }

/* Overwrite the state (teacher forcing): K, V [hkv][len][d], pos [hkv][len]. */
KDO_EXPORT int kdo_load(kdo_state *s, const uint16_t *K, const uint16_t *V, const int32_t *pos,
                        int len)
{
    if (len < 0 || len > s->N) return -1;
    const size_t cap = (size_t)s->N + s->B;
    for (int g = 0; g < s->hkv; ++g) {
        memcpy(s->K + (size_t)g * cap * s->d, K + (size_t)g * len * s->d, sizeof(uint16_t) * (size_t)len * s->d);
        memcpy(s->V + (size_t)g * cap * s->d, V + (size_t)g * len * s->d, sizeof(uint16_t) * (size_t)len * s->d);
        memcpy(s->pos + (size_t)g * cap, pos + (size_t)g * len, sizeof(int32_t) * (size_t)len);
    }
    s->len = len;
    return 0;
}

/* One block step.  q [hq][Bt][d] (nullable together with out: attention is then
 * skipped -- the eviction trace does not depend on queries or values);
 * k_new, v_new [hkv][Bt][d]; out [hq][Bt][d] float; scores_out (nullable)
 * [hkv][len + Bt] float, written only when this step evicts, in row order
 * before eviction.  Returns the number of rows evicted per head (>= 0) or a
 * negative value on a bad argument.                                            */
KDO_EXPORT int kdo_prefill_block(kdo_state *s, const uint16_t *q, const uint16_t *k_new,
                                 const uint16_t *v_new, int Bt, int64_t pos0, float *out,
                                 float *scores_out)
{
    if (Bt < 1 || Bt > s->B) return -1;
    const int d = s->d, hkv = s->hkv;
    const size_t cap = (size_t)s->N + s->B;
    const int len = s->len, n = len + Bt;

    /* append (Eq. 5) */
    for (int g = 0; g < hkv; ++g) {
        memcpy(s->K + ((size_t)g * cap + len) * d, k_new + (size_t)g * Bt * d, sizeof(uint16_t) * (size_t)Bt * d);
        memcpy(s->V + ((size_t)g * cap + len) * d, v_new + (size_t)g * Bt * d, sizeof(uint16_t) * (size_t)Bt * d);
        for (int j = 0; j < Bt; ++j) s->pos[(size_t)g * cap + len + j] = (int32_t)(pos0 + j);
    }

    /* attention before eviction (Fig. 1, step 2 precedes 3-4) */
    if (q && out)
        kdo_attention(q, s->K, s->V, s->hq, hkv, d, (int)cap, len, Bt, s->scale, out);

    if (n <= s->N) { /* budget not exceeded: nothing to evict */
        s->len = n;
        return 0;
    }

    double *mu = (double *)malloc(sizeof(double) * (size_t)d);
    float *sc = (float *)malloc(sizeof(float) * (size_t)n);
    int32_t *kept = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->N);
    uint16_t *tk = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)s->N * d);
    uint16_t *tv = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)s->N * d);
    int32_t *tp = (int32_t *)malloc(sizeof(int32_t) * (size_t)s->N);
    for (int g = 0; g < hkv; ++g) {
        uint16_t *Kh = s->K + (size_t)g * cap * d, *Vh = s->V + (size_t)g * cap * d;
        int32_t *ph = s->pos + (size_t)g * cap;
        kdo_anchor(Kh, n, d, s->mode, mu);
        kdo_scores(Kh, n, d, mu, s->eps, NULL, sc);
        if (scores_out) memcpy(scores_out + (size_t)g * n, sc, sizeof(float) * (size_t)n);
        kdo_select(sc, ph, n, s->N, s->W, kept);
        /* gather (Eq. 6), survivors in ascending position */
        for (int r = 0; r < s->N; ++r) {
            memcpy(tk + (size_t)r * d, Kh + (size_t)kept[r] * d, sizeof(uint16_t) * (size_t)d);
            memcpy(tv + (size_t)r * d, Vh + (size_t)kept[r] * d, sizeof(uint16_t) * (size_t)d);
            tp[r] = ph[kept[r]];
        }
        memcpy(Kh, tk, sizeof(uint16_t) * (size_t)s->N * d);
        memcpy(Vh, tv, sizeof(uint16_t) * (size_t)s->N * d);
        memcpy(ph, tp, sizeof(int32_t) * (size_t)s->N);
    }
    free(tp); free(tv); free(tk); free(kept); free(sc); free(mu);
    s->len = s->N;
    return n - s->N;
}

/* Scores of the rows currently cached, no mutation: out [hkv][len]. */
KDO_EXPORT void kdo_scores_of_cache(const kdo_state *s, float *out)
{
    const size_t cap = (size_t)s->N + s->B;
    double *mu = (double *)malloc(sizeof(double) * (size_t)s->d);
    for (int g = 0; g < s->hkv; ++g) {
        const uint16_t *Kh = s->K + (size_t)g * cap * s->d;
        kdo_anchor(Kh, s->len, s->d, s->mode, mu);
        kdo_scores(Kh, s->len, s->d, mu, s->eps, NULL, out + (size_t)g * s->len);
    }
    free(mu);
}

/* ------------------------------------------------------------------- pairwise
 * Eq. 6: row sums of the pairwise cosine-similarity matrix, O(n^2 d).  A key of
 * zero norm has similarity 0 to everything.  Used to pin the anchor form.      */
KDO_EXPORT void kdo_pairwise_rowsum(const uint16_t *Kh, int n, int d, double *rowsum)
{
    double *nrm = (double *)malloc(sizeof(double) * (size_t)n);
    for (int i = 0; i < n; ++i) {
        double k2 = 0.0;
        for (int c = 0; c < d; ++c) {
            const double x = bf16_to_f64(Kh[(size_t)i * d + c]);
            k2 += x * x;
        }
        nrm[i] = sqrt(k2);
    }
    for (int i = 0; i < n; ++i) {
        double acc = 0.0;
        for (int j = 0; j < n; ++j) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c)
                dot += bf16_to_f64(Kh[(size_t)i * d + c]) * bf16_to_f64(Kh[(size_t)j * d + c]);
            const double den = nrm[i] * nrm[j];
            acc += den > 0.0 ? dot / den : 0.0;
        }
        rowsum[i] = acc;
    }
    free(nrm);
}
