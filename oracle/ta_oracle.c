/*
 * CPU oracle for the Transactional Attention (TA) KV-cache eviction pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, single-threaded
 * restatement of what the eviction pass computes, written from the paper's
 * definitions.  It shares no code, header, table or constant with the GPU
 * library; only tests, the smoke check and the benchmark's CPU-baseline leg
 * may call it.  Every pointer is host memory, every array is contiguous.
 *
 * Conventions: positions p are 0-based (the paper's i = p + 1).  bf16 values
 * are passed as their 16 raw bits (uint16_t) and widened exactly.
 *
 * Parity pins live in tests/ (printed voucher values, the budget-partition
 * example, softmax row sums, closed forms, brute force on tiny inputs,
 * numpy/torch library routines).  Unpinned: nothing in this file; the values
 * of A on a trained model and the paper's accuracy tables are not reproduced.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- bf16 -> double, exact ------------------------------------------- */
static double bf16_to_double(uint16_t h)
{
    uint32_t bits = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * Step 1 - anchor detection (Sec. 3.2 "Anchor detection"; Alg. 1, detection
 * step; Eq. 1 term S_i).  The pattern set P is a table of token-ID n-grams.
 * Position p is an anchor iff some entry e of length len[e] equals the tokens
 * ending at p; the anchor is the LAST token of the n-gram, so that the
 * sponsored span starts right after the pattern.  Every position is tested on
 * its own: overlapping and nested matches all count, and a position matched by
 * several entries is still one anchor (S_i is an indicator).
 *
 * tab_ids is [E][tab_stride]; only the first len[e] IDs of a row are read.
 */
void ta_oracle_match(const int32_t *tok, int32_t n,
                     const int32_t *tab_ids, int32_t tab_stride,
                     const int32_t *tab_len, int32_t E,
                     uint8_t *anchor)
{
    for (int32_t p = 0; p < n; ++p) {
        uint8_t hit = 0;
        for (int32_t e = 0; e < E; ++e) {
            int32_t len = tab_len[e];
            if (len < 1 || p - len + 1 < 0)
                continue;
            int ok = 1;
            for (int32_t t = 0; t < len; ++t)
                if (tok[p - len + 1 + t] != tab_ids[(size_t)e * tab_stride + t])
                    ok = 0;
            if (ok)
                hit = 1;
        }
        anchor[p] = hit;
    }
}

/*
 * Step 2 - voucher allocation (Eq. 2; Alg. 1, the double loop over anchors
 * and j = i+1..i+L; Fig. 2 caption).  V_j = sum over anchors i with
 * i < j <= i+L of B_i * rho^(j-i).  Spans are clipped at the end of the
 * sequence, overlapping spans add, a later anchor never truncates a span.
 * spons[j] = 1 iff at least one anchor lies in [j-L, j-1].
 *
 * Arithmetic: pw[k] = (float) rho^k with rho^k evaluated in double; each term
 * B_i * pw[k] is rounded to fp32; terms are added in fp32 in order of
 * increasing distance k.  anchor_B (nullable) gives a per-anchor budget B_i;
 * when NULL every anchor has budget B.
 */
void ta_oracle_expand(const uint8_t *anchor, const float *anchor_B, int32_t n,
                      int32_t L, float B, double rho,
                      uint8_t *spons, float *V)
{
    float *pw = (float *)malloc(sizeof(float) * (size_t)(L + 1));
    for (int32_t k = 0; k <= L; ++k)
        pw[k] = (float)pow(rho, (double)k);
    for (int32_t j = 0; j < n; ++j) {
        float v = 0.0f;
        uint8_t s = 0;
        for (int32_t k = 1; k <= L; ++k) {
            int32_t i = j - k;
            if (i < 0 || !anchor[i])
                continue;
            float Bi = anchor_B ? anchor_B[i] : B;
            float term = Bi * pw[k];
            v = v + term;
            s = 1;
        }
        V[j] = v;
        spons[j] = s;
    }
    free(pw);
}

/*
 * Step 3 - attention term A_i (Eq. 1 "cumulative attention across heads and
 * steps"; dormant-token definition in App. A: A_i = sum_s sum_h a_{h,i}^(s)).
 * The "steps" of a one-shot pass are the last W positions of the context (the
 * observation window), the heads are the G query heads that share this KV
 * head.  Row (h, w) is the query at absolute position P_w = n - W + w; under
 * the causal mask it sees keys 0..P_w.  a = softmax over visible keys of
 * q.k / sqrt(d).  Everything is evaluated in double from the exact bf16
 * inputs; the result is rounded to fp32 once.
 *
 * Q is [G][W][d] (the heads of this group), K is [n][d].
 */
void ta_oracle_score(const uint16_t *Q, const uint16_t *K,
                     int32_t n, int32_t G, int32_t W, int32_t d,
                     int32_t causal, float *A)
{
    double *acc = (double *)calloc((size_t)n, sizeof(double));
    double *s = (double *)malloc(sizeof(double) * (size_t)n);
    double *q = (double *)malloc(sizeof(double) * (size_t)d);
    const double scale = 1.0 / sqrt((double)d);
    for (int32_t h = 0; h < G; ++h) {
        for (int32_t w = 0; w < W; ++w) {
            const uint16_t *qrow = Q + ((size_t)h * W + w) * d;
            for (int32_t c = 0; c < d; ++c)
                q[c] = bf16_to_double(qrow[c]);
            int32_t last = causal ? (n - W + w) : (n - 1); /* last visible key */
            if (last < 0)
                continue; /* query sees nothing: contributes nothing */
            double m = -INFINITY;
            for (int32_t i = 0; i <= last; ++i) {
                const uint16_t *krow = K + (size_t)i * d;
                double dot = 0.0;
                for (int32_t c = 0; c < d; ++c)
                    dot += q[c] * bf16_to_double(krow[c]);
                s[i] = dot * scale;
                if (s[i] > m)
                    m = s[i];
            }
            double Z = 0.0;
            for (int32_t i = 0; i <= last; ++i)
                Z += exp(s[i] - m);
            for (int32_t i = 0; i <= last; ++i)
                acc[i] += exp(s[i] - m) / Z;
        }
    }
    for (int32_t i = 0; i < n; ++i)
        A[i] = (float)acc[i];
    free(q);
    free(s);
    free(acc);
}

/*
 * Step 4 - utility and protected top-K (Eq. 1; Eq. 3 for TA-Fast; Alg. 1
 * utility and top-K steps; Sec. 3.3 budget partition; Thm. 2-4 and the
 * budget-partition table of App. D).
 *
 *   u_p = alpha*A_p + beta*(p+1)/n + gamma*S_p + V_p        (delta=lambda=0:
 *         the pension and frequency terms have no definition in the paper)
 *
 * evaluated in fp32, every product and sum rounded, left to right.
 * Classes: 2 = attention sink (p < n_sink) or recent window (p >= n-n_recent),
 * 1 = sponsored and not class 2, 0 = everything else.  The retained set is
 * the first min(K, n) positions under the total order (class descending,
 * u descending, position descending), reported in ascending position order.
 * With alpha == 0 the array A is not read (may be NULL).
 */
typedef struct {
    int32_t cls;
    float u;
    int32_t pos;
} ta_oracle_key;

static int key_before(const void *pa, const void *pb)
{
    const ta_oracle_key *a = (const ta_oracle_key *)pa;
    const ta_oracle_key *b = (const ta_oracle_key *)pb;
    if (a->cls != b->cls)
        return a->cls > b->cls ? -1 : 1;
    if (a->u != b->u)
        return a->u > b->u ? -1 : 1;
    if (a->pos != b->pos)
        return a->pos > b->pos ? -1 : 1;
    return 0;
}

static int int_ascending(const void *pa, const void *pb)
{
    int32_t a = *(const int32_t *)pa, b = *(const int32_t *)pb;
    return (a > b) - (a < b);
}

void ta_oracle_utility(const float *A, const uint8_t *anchor, const float *V,
                       int32_t n, float alpha, float beta, float gamma,
                       float *u)
{
    for (int32_t p = 0; p < n; ++p) {
        float r = (float)(p + 1) / (float)n;
        float t = (alpha != 0.0f) ? alpha * A[p] : 0.0f;
        float b = beta * r;
        t = t + b;
        float g = gamma * (float)anchor[p];
        t = t + g;
        t = t + V[p];
        u[p] = t;
    }
}

int32_t ta_oracle_select(const float *A, const uint8_t *anchor,
                         const uint8_t *spons, const float *V,
                         int32_t n, int32_t K, int32_t n_sink, int32_t n_recent,
                         float alpha, float beta, float gamma,
                         int32_t *idx)
{
    int32_t cnt = K < n ? K : n;
    if (cnt <= 0)
        return 0;
    float *u = (float *)malloc(sizeof(float) * (size_t)n);
    ta_oracle_key *keys = (ta_oracle_key *)malloc(sizeof(ta_oracle_key) * (size_t)n);
    ta_oracle_utility(A, anchor, V, n, alpha, beta, gamma, u);
    for (int32_t p = 0; p < n; ++p) {
        int32_t cls = 0;
        if (p < n_sink || p >= n - n_recent)
            cls = 2;
        else if (spons[p])
            cls = 1;
        keys[p].cls = cls;
        keys[p].u = u[p];
        keys[p].pos = p;
    }
    qsort(keys, (size_t)n, sizeof(ta_oracle_key), key_before);
    for (int32_t r = 0; r < cnt; ++r)
        idx[r] = keys[r].pos;
    qsort(idx, (size_t)cnt, sizeof(int32_t), int_ascending);
    free(keys);
    free(u);
    return cnt;
}

/*
 * Step 5 - eviction (Sec. 3.2 "Token selection": index_select on the KV
 * tensors along the sequence dimension; Alg. 1 eviction step).
 * out[r,:] = in[idx[r],:], rows of row_elems 16-bit elements.
 */
void ta_oracle_compact(const uint16_t *in, const int32_t *idx, int32_t cnt,
                       int32_t row_elems, uint16_t *out)
{
    for (int32_t r = 0; r < cnt; ++r)
        memcpy(out + (size_t)r * row_elems, in + (size_t)idx[r] * row_elems,
               sizeof(uint16_t) * (size_t)row_elems);
}
