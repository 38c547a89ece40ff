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
 * numpy/torch library routines; the incremental form: sliding-window reduction,
 * decay closed form, softmax sums, tuple-order arg-min; the learned detector:
 * GELU and logistic closed forms, a linear special case, torch's float64 ops;
 * embedding cosine: identical / orthogonal / opposite vectors, scale invariance,
 * numpy float64; policy options: torch max_pool1d, the partition against the
 * elastic selection, a plain top-K and brute force, the budget-partition table,
 * sum / endpoints / monotonicity of the layer budgets; scores from a given
 * log-sum-exp: torch.logsumexp, agreement with the two-pass scores, row sums;
 * paged gather and scatter: numpy fancy indexing on both common page layouts,
 * gather after scatter returns the rows; margin of the cut: hand-read cases, and
 * the minimum / maximum restated on the selection's own output).
 * Unpinned: nothing in this file; the values
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
 * Margin of the cut that ta_oracle_select makes (a diagnostic of the total order of
 * Sec. 3.3 / Eq. 1, not a quantity of the paper): with the positions ranked as above, the
 * first evicted one is ranked min(K, n); its class c is the class the cut falls in (every
 * higher class is kept whole).
 *   margin[0] = smallest u among the retained positions of class c, +inf if none is retained
 *   margin[1] = largest u among the evicted positions of class c  (the first evicted one's)
 * Nothing evicted (n <= K): (+inf, -inf).  margin[0] == margin[1] means positions tie at the
 * cut and the position order decided; a small gap means a selection that rounding can flip.
 */
void ta_oracle_select_margin(const float *A, const uint8_t *anchor,
                             const uint8_t *spons, const float *V,
                             int32_t n, int32_t K, int32_t n_sink, int32_t n_recent,
                             float alpha, float beta, float gamma, float *margin)
{
    margin[0] = INFINITY;
    margin[1] = -INFINITY;
    if (n <= K || K <= 0)
        return;
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
    margin[1] = keys[K].u;
    if (keys[K - 1].cls == keys[K].cls)
        margin[0] = keys[K - 1].u;
    free(keys);
    free(u);
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

/* ======================================================================
 * Incremental (per generation step) form of the same pass
 * ("a retention policy selects a subset ... after each generation step",
 * Sec. 3.1; Alg. 1 run once per step, including its last step: the budget
 * decay B_i <- 0.9 B_i of Sec. 3.2 "Token selection").
 *
 * Per sequence the state is the token stream, the anchor flags and the
 * CURRENT budget of every anchor (0 where there is no anchor).  Per unit the
 * cache holds K+1 slots: K occupied and one free.  One step appends one
 * token: the new k/v row goes into the free slot, the decode queries of the
 * group add their softmax weights over the K+1 cached rows to the cumulative
 * attention A of each slot (H2O-style accumulation, Eq. 1 "cumulative
 * attention across heads and steps"), the slot that ranks last under the
 * (class, u, position) order is evicted and becomes the free slot, and
 * finally every budget decays.  Vouchers are recomputed from the current
 * budgets each step (Alg. 1 rebuilds V from B_i every time it runs); classes
 * and the recency term use absolute positions and the current length.
 * ====================================================================== */

/* Append one token to a sequence: anchor flag of the new position (same rule
 * as ta_oracle_match, evaluated at the new position only) and its budget. */
void ta_oracle_decode_append(int32_t *tok, uint8_t *anchor, float *budget, int32_t len,
                             int32_t new_tok,
                             const int32_t *tab_ids, int32_t tab_stride,
                             const int32_t *tab_len, int32_t E, float B)
{
    tok[len] = new_tok;
    uint8_t hit = 0;
    for (int32_t e = 0; e < E; ++e) {
        int32_t l = tab_len[e];
        if (l < 1 || len - l + 1 < 0)
            continue;
        int ok = 1;
        for (int32_t t = 0; t < l; ++t)
            if (tok[len - l + 1 + t] != tab_ids[(size_t)e * tab_stride + t])
                ok = 0;
        if (ok)
            hit = 1;
    }
    anchor[len] = hit;
    budget[len] = hit ? B : 0.0f;
}

/* Voucher and sponsor flag of position p from the current budgets (Eq. 2). */
void ta_oracle_decode_vouch(const uint8_t *anchor, const float *budget, int32_t p,
                            int32_t L, double rho, float *V, uint8_t *spons)
{
    float v = 0.0f;
    uint8_t s = 0;
    for (int32_t k = 1; k <= L; ++k) {
        int32_t i = p - k;
        if (i < 0 || !anchor[i])
            continue;
        float pw = (float)pow(rho, (double)k);
        float term = budget[i] * pw;
        v = v + term;
        s = 1;
    }
    *V = v;
    *spons = s;
}

/* Budget decay at the end of a step (Alg. 1, last step). */
void ta_oracle_decode_decay(float *budget, int32_t len, float decay)
{
    for (int32_t i = 0; i < len; ++i)
        budget[i] = decay * budget[i];
}

/*
 * One step of one unit.  Kc/Vc: [slots][d] bf16 bits, pos[slots] (absolute
 * position, -1 = free; at least one slot is free on entry), A[slots].
 * q: [G][d] decode queries of the group, k_new/v_new: [d].
 * The new row takes the lowest-numbered free slot.  Attention runs over the
 * occupied slots.  If no slot is free afterwards (the cache holds more than
 * its budget of slots-1 rows) the slot ranking last is evicted, otherwise
 * nothing is.
 * rank_A (nullable): attention values to rank with instead of the unit's own
 * updated A (lets a caller impose scores computed elsewhere, in the same
 * precision on both sides of a comparison).
 * last_query != 0: the attention term of a slot is the mass that THIS step's
 * queries give it, not the running sum over the steps - the step-wise
 * minimum-attention eviction that the corollary of Thm. 1 ascribes to TOVA
 * (Sec. 2).  A[s] of every occupied slot is then replaced by this step's
 * mass.
 * Returns the evicted slot or -1; u_out (nullable, [slots]) receives the
 * utilities of the occupied slots.
 */
int32_t ta_oracle_decode_unit(uint16_t *Kc, uint16_t *Vc, int32_t *pos, float *A,
                              int32_t slots, int32_t d,
                              const uint16_t *q, int32_t G,
                              const uint16_t *k_new, const uint16_t *v_new, int32_t p_new,
                              const uint8_t *anchor, const float *budget, int32_t len_new,
                              int32_t n_sink, int32_t n_recent, int32_t L, double rho,
                              float alpha, float beta, float gamma,
                              const float *rank_A, float *u_out, int32_t last_query)
{
    int32_t f = -1;
    for (int32_t s = slots - 1; s >= 0; --s)
        if (pos[s] < 0)
            f = s;
    if (f < 0)
        return -1;
    memcpy(Kc + (size_t)f * d, k_new, sizeof(uint16_t) * (size_t)d);
    memcpy(Vc + (size_t)f * d, v_new, sizeof(uint16_t) * (size_t)d);
    pos[f] = p_new;
    A[f] = 0.0f;

    /* attention of the decode queries over every cached row */
    if (alpha != 0.0f) {
        double *add = (double *)calloc((size_t)slots, sizeof(double));
        double *sc = (double *)malloc(sizeof(double) * (size_t)slots);
        const double scale = 1.0 / sqrt((double)d);
        for (int32_t h = 0; h < G; ++h) {
            double m = -INFINITY;
            for (int32_t s = 0; s < slots; ++s) {
                if (pos[s] < 0)
                    continue;
                double dot = 0.0;
                for (int32_t c = 0; c < d; ++c)
                    dot += bf16_to_double(q[(size_t)h * d + c]) * bf16_to_double(Kc[(size_t)s * d + c]);
                sc[s] = dot * scale;
                if (sc[s] > m)
                    m = sc[s];
            }
            double Z = 0.0;
            for (int32_t s = 0; s < slots; ++s)
                if (pos[s] >= 0)
                    Z += exp(sc[s] - m);
            for (int32_t s = 0; s < slots; ++s)
                if (pos[s] >= 0)
                    add[s] += exp(sc[s] - m) / Z;
        }
        for (int32_t s = 0; s < slots; ++s)
            if (pos[s] >= 0)
                A[s] = last_query ? (float)add[s] : (float)((double)A[s] + add[s]);
        free(sc);
        free(add);
    }

    /* rank every occupied slot; if the cache is over budget the last one under the order goes */
    ta_oracle_key worst;
    int32_t worst_slot = -1, nfree = 0;
    for (int32_t s = 0; s < slots; ++s) {
        int32_t p = pos[s];
        if (p < 0) {
            ++nfree;
            continue;
        }
        float V;
        uint8_t sp;
        ta_oracle_decode_vouch(anchor, budget, p, L, rho, &V, &sp);
        float a = rank_A ? rank_A[s] : A[s];
        float r = (float)(p + 1) / (float)len_new;
        float t = (alpha != 0.0f) ? alpha * a : 0.0f;
        float b = beta * r;
        t = t + b;
        float g = gamma * (float)anchor[p];
        t = t + g;
        t = t + V;
        if (u_out)
            u_out[s] = t;
        ta_oracle_key k;
        k.cls = (p < n_sink || p >= len_new - n_recent) ? 2 : (sp ? 1 : 0);
        k.u = t;
        k.pos = p;
        if (worst_slot < 0 || key_before(&worst, &k) < 0) { /* worst ranks before k: k is worse */
            worst = k;
            worst_slot = s;
        }
    }
    if (nfree > 0)
        return -1;
    pos[worst_slot] = -1;
    return worst_slot;
}


/* ======================================================================
 * Learned anchor detection and confidence-weighted sponsorship
 * (Sec. 5.1 "Learned Anchor Detection": the detector equation and the
 * TA-Learned / TA-LearnRank rules).
 * ====================================================================== */

/*
 * Detector f(h) = sigmoid(W2 . GELU(W1 . h)) on one sequence of hidden states
 * (Sec. 5.1, detector equation).  h is [n][dm], W1 is [m][dm], W2 is [m], all bf16
 * bit patterns; no bias terms (the equation has none); GELU is the exact form
 * x * Phi(x) of the cited definition.  Everything is evaluated in double and the
 * confidence is returned rounded to fp32.
 */
void ta_oracle_detect(const uint16_t *h, const uint16_t *W1, const uint16_t *W2,
                      int32_t n, int32_t dm, int32_t m, float *conf)
{
    for (int32_t p = 0; p < n; ++p) {
        double out = 0.0;
        for (int32_t j = 0; j < m; ++j) {
            double z = 0.0;
            for (int32_t c = 0; c < dm; ++c)
                z += bf16_to_double(h[(size_t)p * dm + c]) * bf16_to_double(W1[(size_t)j * dm + c]);
            const double gelu = 0.5 * z * (1.0 + erf(z / sqrt(2.0)));
            out += bf16_to_double(W2[j]) * gelu;
        }
        conf[p] = (float)(1.0 / (1.0 + exp(-out)));
    }
}

/*
 * Anchors and their budgets from confidences (Sec. 5.1).  A position is an
 * anchor iff conf > thr (strictly; 0.5 for TA-Learned, 0.3 for TA-LearnRank).
 * rank == 0: every anchor gets the fixed budget B (TA-Learned: the sponsorship of
 * Eq. 2 applied after confident predictions).  rank != 0: the budget is the
 * confidence itself times `scale` (TA-LearnRank equation: V_j sums f(h_i) rho^(j-i);
 * scale = 1 is the printed form).  The product is one fp32 multiplication.
 * Vouchers then follow from ta_oracle_expand with these per-anchor budgets.
 */
void ta_oracle_confidence_anchors(const float *conf, int32_t n, float thr, int32_t rank,
                                  float B, float scale, uint8_t *anchor, float *anchor_B)
{
    for (int32_t p = 0; p < n; ++p) {
        const int is_anchor = conf[p] > thr;
        anchor[p] = (uint8_t)is_anchor;
        anchor_B[p] = is_anchor ? (rank ? scale * conf[p] : B) : 0.0f;
    }
}

/*
 * Embedding-based anchor detection (Sec. 3.2 "Anchor detection", third instantiation;
 * TA-Fast-Embedding of Sec. 3.4 and of the multilingual experiment): the similarity of
 * an input embedding x to a set of anchor-concept embeddings c_0 .. c_{E-1} is the
 * largest cosine
 *     sim = max_e  (x . c_e) / (|x| |c_e|),
 * a cosine with a zero vector on either side counting as 0.  x is [n][dm], C is
 * [E][dm], bf16 bit patterns, E >= 1; evaluated in double, returned rounded to fp32.
 * The paper gives no threshold: a position is an anchor iff sim > tau (strictly),
 * tau a parameter.  Budgets are the fixed B of Eq. 2, so the flags feed
 * ta_oracle_expand unchanged.
 */
void ta_oracle_cosine_sim(const uint16_t *x, const uint16_t *C, int32_t n, int32_t dm, int32_t E, float *sim)
{
    for (int32_t p = 0; p < n; ++p) {
        double xx = 0.0;
        for (int32_t c = 0; c < dm; ++c) {
            const double v = bf16_to_double(x[(size_t)p * dm + c]);
            xx += v * v;
        }
        double best = 0.0;
        for (int32_t e = 0; e < E; ++e) {
            double dot = 0.0, cc = 0.0;
            for (int32_t c = 0; c < dm; ++c) {
                const double v = bf16_to_double(C[(size_t)e * dm + c]);
                dot += bf16_to_double(x[(size_t)p * dm + c]) * v;
                cc += v * v;
            }
            const double cosine = (xx > 0.0 && cc > 0.0) ? dot / (sqrt(xx) * sqrt(cc)) : 0.0;
            if (e == 0 || cosine > best) best = cosine;
        }
        sim[p] = (float)best;
    }
}

void ta_oracle_threshold_anchors(const float *sim, int32_t n, float tau, uint8_t *anchor)
{
    for (int32_t p = 0; p < n; ++p) anchor[p] = (uint8_t)(sim[p] > tau);
}

/*
 * Input embeddings depend on the token ID only, so embedding-based detection can be run
 * over the vocabulary once and looked up per position: anchor[p] = vocab_anchor[tok[p]].
 * IDs outside [0, V) are never anchors.
 */
void ta_oracle_lookup_anchors(const int32_t *tok, int32_t n, const uint8_t *vocab_anchor, int32_t V, uint8_t *anchor)
{
    for (int32_t p = 0; p < n; ++p)
        anchor[p] = (uint8_t)((tok[p] >= 0 && tok[p] < V) ? (vocab_anchor[tok[p]] != 0) : 0);
}

/* ======================================================================
 * Policy options around the same selection (Sec. 3.3 budget partition; Sec. 2 /
 * Sec. 4 baselines as settings; Sec. 5.2 robustness).
 * ====================================================================== */

/*
 * Max-pooling of the attention scores before the selection, the clustering step
 * of the SnapKV baseline (Sec. 2 "clusters attention patterns"): window of k
 * positions (k odd) centred on p, clipped to the sequence:
 *   out[p] = max { A[q] : |q - p| <= (k-1)/2, 0 <= q < n }.
 */
void ta_oracle_maxpool(const float *A, int32_t n, int32_t k, float *out)
{
    const int32_t r = (k - 1) / 2;
    for (int32_t p = 0; p < n; ++p) {
        float m = A[p];
        for (int32_t q = p - r; q <= p + r; ++q)
            if (q >= 0 && q < n && A[q] > m)
                m = A[q];
        out[p] = m;
    }
}

/*
 * Selection with a fixed budget partition (Sec. 3.3): K = K_main + K_protected.
 * The protected pool holds the k_protected sponsored tokens that rank first under
 * (u, position) - all of them if there are fewer; the main pool holds the mandatory
 * tokens (sinks, recent window) and fills its remaining K - mandatory - protected
 * slots with the best of ALL other tokens under (u, position), sponsored or not
 * ("selected by utility score").  Unused protected slots return to the main pool.
 * k_protected = 0 is the strict configuration of the ablation (K_main = K);
 * k_protected >= number of sponsored tokens is the elastic reading of
 * ta_oracle_select whenever the sponsored tokens fit.
 */
int32_t ta_oracle_select_partition(const float *A, const uint8_t *anchor,
                                   const uint8_t *spons, const float *V,
                                   int32_t n, int32_t K, int32_t k_protected,
                                   int32_t n_sink, int32_t n_recent,
                                   float alpha, float beta, float gamma, int32_t *idx)
{
    int32_t cnt = K < n ? K : n;
    if (cnt <= 0)
        return 0;
    float *u = (float *)malloc(sizeof(float) * (size_t)n);
    ta_oracle_key *keys = (ta_oracle_key *)malloc(sizeof(ta_oracle_key) * (size_t)n);
    ta_oracle_utility(A, anchor, V, n, alpha, beta, gamma, u);
    /* pass 1: mandatory tokens first, then sponsored by (u, position), then the rest */
    int32_t mandatory = 0;
    for (int32_t p = 0; p < n; ++p) {
        int32_t cls = 0;
        if (p < n_sink || p >= n - n_recent) {
            cls = 2;
            ++mandatory;
        } else if (spons[p])
            cls = 1;
        keys[p].cls = cls;
        keys[p].u = u[p];
        keys[p].pos = p;
    }
    qsort(keys, (size_t)n, sizeof(ta_oracle_key), key_before);
    int32_t sponsored = 0;
    for (int32_t r = mandatory; r < n && keys[r].cls == 1; ++r)
        ++sponsored;
    int32_t prot = k_protected < sponsored ? k_protected : sponsored;
    if (prot > cnt - mandatory)
        prot = cnt - mandatory > 0 ? cnt - mandatory : 0;
    /* pass 2: everything after the mandatory and protected tokens competes by (u, position) alone */
    for (int32_t r = mandatory + prot; r < n; ++r)
        keys[r].cls = 0;
    if (mandatory + prot < n)
        qsort(keys + mandatory + prot, (size_t)(n - mandatory - prot), sizeof(ta_oracle_key), key_before);
    for (int32_t r = 0; r < cnt; ++r)
        idx[r] = keys[r].pos;
    qsort(idx, (size_t)cnt, sizeof(int32_t), int_ascending);
    free(keys);
    free(u);
    return cnt;
}

/*
 * Margin of the main-pool cut of ta_oracle_select_partition (a diagnostic, as
 * ta_oracle_select_margin): among the positions that are neither mandatory nor protected,
 *   margin[0] = smallest u among the retained ones, +inf if the main pool has no slot for them
 *   margin[1] = largest u among the evicted ones
 * Nothing evicted (n <= K): (+inf, -inf).
 */
void ta_oracle_select_partition_margin(const float *A, const uint8_t *anchor,
                                       const uint8_t *spons, const float *V,
                                       int32_t n, int32_t K, int32_t k_protected,
                                       int32_t n_sink, int32_t n_recent,
                                       float alpha, float beta, float gamma, float *margin)
{
    margin[0] = INFINITY;
    margin[1] = -INFINITY;
    if (n <= K || K <= 0)
        return;
    float *u = (float *)malloc(sizeof(float) * (size_t)n);
    ta_oracle_key *keys = (ta_oracle_key *)malloc(sizeof(ta_oracle_key) * (size_t)n);
    ta_oracle_utility(A, anchor, V, n, alpha, beta, gamma, u);
    int32_t mandatory = 0;
    for (int32_t p = 0; p < n; ++p) {
        int32_t cls = 0;
        if (p < n_sink || p >= n - n_recent) {
            cls = 2;
            ++mandatory;
        } else if (spons[p])
            cls = 1;
        keys[p].cls = cls;
        keys[p].u = u[p];
        keys[p].pos = p;
    }
    qsort(keys, (size_t)n, sizeof(ta_oracle_key), key_before);
    int32_t sponsored = 0;
    for (int32_t r = mandatory; r < n && keys[r].cls == 1; ++r)
        ++sponsored;
    int32_t prot = k_protected < sponsored ? k_protected : sponsored;
    if (prot > K - mandatory)
        prot = K - mandatory > 0 ? K - mandatory : 0;
    const int32_t first = mandatory + prot;          /* rank of the main pool's best candidate */
    for (int32_t r = first; r < n; ++r)
        keys[r].cls = 0;
    if (first < n)
        qsort(keys + first, (size_t)(n - first), sizeof(ta_oracle_key), key_before);
    if (K >= first) {                                /* else the mandatory tokens alone overflow K */
        margin[1] = keys[K].u;
        if (K - 1 >= first)
            margin[0] = keys[K - 1].u;
    }
    free(keys);
    free(u);
}

/*
 * Per-layer budgets of the PyramidKV baseline (Sec. 2 "allocates budgets pyramidally
 * across transformer layers"): an arithmetic progression that falls from the first
 * layer to the last, ends at k_min and has mean K, i.e. starts at 2K - k_min:
 *   K_l = round-to-nearest( (2K - k_min) - l * (2K - 2 k_min) / (layers - 1) ),
 * with the rounding residue added to layer 0 so that the budgets sum to layers * K.
 * One layer: K.  Requires 1 <= k_min <= K.
 */
void ta_oracle_layer_budgets(int32_t layers, int32_t K, int32_t k_min, int32_t *out)
{
    if (layers == 1) {
        out[0] = K;
        return;
    }
    const double top = 2.0 * K - k_min, step = (2.0 * K - 2.0 * k_min) / (layers - 1);
    int64_t sum = 0;
    for (int32_t l = 0; l < layers; ++l) {
        out[l] = (int32_t)floor(top - l * step + 0.5);
        sum += out[l];
    }
    out[0] += (int32_t)((int64_t)layers * K - sum);
}

/*
 * Allowlist filtering (Sec. 5.2: adversarial anchor injection is answered by an
 * allowlist): an anchor only counts where allow[p] != 0 - positions of untrusted
 * spans can neither be anchors nor sponsor anything.
 */
void ta_oracle_allow_filter(const uint8_t *anchor, const uint8_t *allow, int32_t n, uint8_t *out)
{
    for (int32_t p = 0; p < n; ++p)
        out[p] = (uint8_t)(anchor[p] != 0 && allow[p] != 0);
}

/*
 * Scoring fused with the prefill attention (Sec. 3.4 / Sec. 4.7: TA must live with
 * SDPA / FlashAttention backends that never materialise the attention matrix).  Such a
 * kernel already sweeps the keys for the window's queries and leaves, per query row, the
 * log-sum-exp of its scaled logits,
 *     lse[h][w] = log sum_{i visible} exp(q_{h,w} . k_i / sqrt(d)),
 * from which the attention weight of a key is exp(s - lse) without a second reduction:
 *     A[i] = sum_{h,w : i visible} exp(q_{h,w} . k_i / sqrt(d) - lse[h][w]).
 * ta_oracle_row_lse is the definition of that by-product (double, rounded to fp32; -inf
 * for a row that sees no key); ta_oracle_score_lse evaluates the sum above in double from
 * the fp32 lse it is given.
 */
void ta_oracle_row_lse(const uint16_t *Q, const uint16_t *K, int32_t n, int32_t G, int32_t W, int32_t d,
                       int32_t causal, float *lse)
{
    const double scale = 1.0 / sqrt((double)d);
    double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    for (int32_t h = 0; h < G; ++h)
        for (int32_t w = 0; w < W; ++w) {
            const uint16_t *qrow = Q + ((size_t)h * W + w) * d;
            const int32_t last = causal ? (n - W + w) : (n - 1);
            double m = -INFINITY;
            for (int32_t i = 0; i <= last; ++i) {
                double dot = 0.0;
                for (int32_t c = 0; c < d; ++c)
                    dot += bf16_to_double(qrow[c]) * bf16_to_double(K[(size_t)i * d + c]);
                s[i] = dot * scale;
                if (s[i] > m)
                    m = s[i];
            }
            double Z = 0.0;
            for (int32_t i = 0; i <= last; ++i)
                Z += exp(s[i] - m);
            lse[(size_t)h * W + w] = last < 0 ? -INFINITY : (float)(m + log(Z));
        }
    free(s);
}

void ta_oracle_score_lse(const uint16_t *Q, const uint16_t *K, const float *lse,
                         int32_t n, int32_t G, int32_t W, int32_t d, int32_t causal, float *A)
{
    const double scale = 1.0 / sqrt((double)d);
    double *acc = (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double));
    for (int32_t h = 0; h < G; ++h)
        for (int32_t w = 0; w < W; ++w) {
            const uint16_t *qrow = Q + ((size_t)h * W + w) * d;
            const int32_t last = causal ? (n - W + w) : (n - 1);
            const double l = (double)lse[(size_t)h * W + w];
            for (int32_t i = 0; i <= last; ++i) {
                double dot = 0.0;
                for (int32_t c = 0; c < d; ++c)
                    dot += bf16_to_double(qrow[c]) * bf16_to_double(K[(size_t)i * d + c]);
                acc[i] += exp(dot * scale - l);
            }
        }
    for (int32_t i = 0; i < n; ++i)
        A[i] = (float)acc[i];
    free(acc);
}

/*
 * Paged (block-table) caches, the layout of serving engines: the rows of one sequence live in
 * pages of page_size positions scattered over a pool; table[j] is the page that holds
 * positions [j * page_size, (j + 1) * page_size).  Row p of head `head` starts at element
 *     table[p / page_size] * stride_page + (p % page_size) * stride_pos + head * stride_head
 * of the pool (one layer).  This function is the whole of the oracle's paged support: it
 * lays the n rows of a (sequence, head) out densely, [n][d], after which every other
 * function of this file applies unchanged.
 */
void ta_oracle_paged_gather(const uint16_t *pool, const int32_t *table, int32_t n, int32_t page_size,
                            int64_t stride_page, int64_t stride_pos, int64_t stride_head, int32_t head,
                            int32_t d, uint16_t *out)
{
    for (int32_t p = 0; p < n; ++p) {
        const uint16_t *row = pool + (int64_t)table[p / page_size] * stride_page +
                              (int64_t)(p % page_size) * stride_pos + (int64_t)head * stride_head;
        memcpy(out + (size_t)p * d, row, sizeof(uint16_t) * (size_t)d);
    }
}

/*
 * The inverse of the gather: rows [cnt][d] of one (sequence, head) are written to slots
 * 0 .. cnt-1 of a paged cache - compaction straight into the page pool, and the layout of a
 * generation-step cache whose K+1 slots live in pages (slot s of the unit is "position" s of
 * the addressing above).  Nothing else in the pool is touched.
 */
void ta_oracle_paged_scatter(const uint16_t *rows, int32_t cnt, const int32_t *table, int32_t page_size,
                             int64_t stride_page, int64_t stride_pos, int64_t stride_head, int32_t head,
                             int32_t d, uint16_t *pool)
{
    for (int32_t r = 0; r < cnt; ++r) {
        uint16_t *dst = pool + (int64_t)table[r / page_size] * stride_page +
                        (int64_t)(r % page_size) * stride_pos + (int64_t)head * stride_head;
        memcpy(dst, rows + (size_t)r * d, sizeof(uint16_t) * (size_t)d);
    }
}
