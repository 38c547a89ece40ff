/*
 * libta - Transactional Attention KV-cache eviction pass for AMD gfx950.
 *
 * C ABI.  One call evicts a KV cache down to a budget of K tokens per
 * (layer, sequence, KV head) "unit":
 *
 *   1. ta_match_anchors  anchor n-gram match over token IDs + voucher expansion
 *   2. ta_score          attention column sums of an observation window
 *   3. ta_select         protected top-K under the (class, utility, position) order
 *   4. ta_compact        gather of the retained K/V rows
 *      ta_detect_anchors /  anchors from a learned detector on hidden states instead of the
 *      ta_expand_vouchers   table match, with confidence-weighted budgets (Sec. 5.1)
 *      ta_embed_anchors /   anchors from cosine similarity to anchor-concept embeddings
 *      ta_lookup_anchors    (Sec. 3.2), per position or once per vocabulary entry
 *      ta_score_lse /    scores in one sweep from the prefill attention's row log-sum-exps
 *      ta_evict_lse
 *      ta_score_paged /  steps 3 and 5, and the whole pass, over paged (block-table) caches
 *      ta_compact_paged / ta_evict_paged
 *      ta_compact_into_pages  step 5 writing its rows into the pages of a block table
 *      ta_evict          all of the above in one call
 *      ta_evict_layers / the same over caches that are one tensor (or one page pool)
 *      ta_evict_layers_paged  per layer
 *      ta_decode_init /  the same policy applied after every generation step
 *      ta_decode_step    (append, accumulate attention, evict one row, decay budgets),
 *                        over dense slots or slots in a page pool
 *      ta_evict_static / ta_evict with its scratch in a static device buffer, for callers
 *      ta_init           that cannot allocate
 *
 * Conventions shared by every entry point
 *   - Pointers marked DEVICE are GPU global memory owned by the caller;
 *     pointers marked HOST are ordinary host memory read during the call.
 *     Inputs are never written; outputs must not alias inputs (ta_compact and the passes
 *     built on it refuse K/V outputs whose address equals an input's or each other's: SHAPE).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls only enqueue work on it: they never synchronise, allocate or free.
 *   - Positions are 0-based; the paper's token i is position p = i - 1.
 *   - K, V, Q are bf16.  The head dimension d must be 128.
 *   - Sequences of a batch are padded to a common length n; `seq_len`
 *     (DEVICE int32 [B], nullable) gives the valid length of each sequence,
 *     clamped to [0, n] on the device.  NULL means every sequence has length n.
 *   - Return value: TA_OK or a negative ta_status.  All argument validation
 *     happens on the host before anything is launched, so an error code other
 *     than TA_ERR_HIP means no work was enqueued.
 */
#ifndef TA_H
#define TA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TA_MAX_TABLE 64   /* anchor-table entries                       */
#define TA_MAX_GRAM 4     /* tokens per anchor n-gram                   */
#define TA_MAX_SPAN 64    /* sponsor span L                             */
#define TA_MAX_LAYER_PTRS 96 /* layers of a per-layer pointer table       */
#define TA_LAYER_WS_BYTES 4096 /* workspace share of such a table         */
#define TA_HEAD_DIM 128   /* the only supported head dimension          */
#define TA_MAX_ROWS 512   /* (query heads per KV head) * window rows    */

typedef enum ta_status {
    TA_OK = 0,
    TA_ERR_NULL = -1,      /* a required pointer is NULL                                   */
    TA_ERR_SHAPE = -2,     /* a size, stride or table entry is outside the supported range */
    TA_ERR_BUDGET = -3,    /* K < 1 or K < n_sink + n_recent                               */
    TA_ERR_WORKSPACE = -4, /* workspace missing or smaller than ta_workspace_bytes()       */
    TA_ERR_ALIGN = -5,     /* a pointer or stride is not aligned as documented (K/V/Q: 16 bytes) */
    TA_ERR_HIP = -6,       /* a launch failed; see ta_last_hip_error()                     */
    TA_ERR_SCRATCH = -7    /* ta_evict_static: the layout needs more scratch than
                              TA_STATIC_SCRATCH_BYTES                                      */
} ta_status;

/*
 * Hyper-parameters of the retention policy (Eq. 1, Eq. 2, Eq. 3, Sec. 3.3).
 * The pension and frequency terms of Eq. 1 have no definition in the paper and
 * are not part of the utility (delta = lambda = 0).
 */
typedef struct ta_params {
    int32_t n_sink;     /* first n_sink positions are always retained (attention sinks)   */
    int32_t n_recent;   /* last n_recent positions are always retained (recent window)    */
    int32_t span_L;     /* sponsor span L of Eq. 2 (paper default 6), 0..TA_MAX_SPAN      */
    float sponsor_B;    /* sponsor budget B of Eq. 2 (paper default 15)                   */
    double rho;         /* voucher decay base of Eq. 2 (paper: 0.8)                       */
    float alpha;        /* weight of the attention term A_i (1.0; 0 = TA-Fast, Eq. 3)     */
    float beta;         /* weight of the recency term R_i = (p+1)/n (0.5)                 */
    float gamma;        /* weight of the anchor indicator S_i (0.3)                       */
    int32_t causal;     /* 1: window query w sees keys 0..n-W+w; 0: every key             */
    float budget_decay; /* per-step decay of sponsor budgets (paper: 0.9); decode steps   */
    /* Options around the same selection (baselines of Sec. 2 / Sec. 4 and the partition of
     * Sec. 3.3 as settings).  Defaults: 1, -1, 0, NULL, NULL, NULL.  The per-step form accepts only the
     * defaults of pool_k and k_protected and ignores layer_K and allow; the one-shot pass ignores
     * last_query. */
    int32_t pool_k;      /* odd window (1, 3, 5, 7 or 9) of a max-pool applied to A along the sequence
                            before the utility - the clustering step of SnapKV; 1 = none            */
    int32_t k_protected; /* K_protected of Sec. 3.3: the protected pool holds the k_protected best
                            sponsored tokens under (u, position); all other tokens that are not
                            mandatory compete for the K_main = K - k_protected slots by (u, position)
                            alone, mandatory tokens count against K_main, unused protected slots
                            return to the main pool.  Negative: the elastic pool (every sponsored
                            token outranks every plain one).  0: the strict configuration           */
    int32_t last_query;  /* per-step form only (0 or 1).  0: a slot's attention term is its cumulative mass
                            over the steps (H2O-style, Eq. 1).  1: it is the mass the CURRENT step's
                            queries give it - the step-wise minimum-attention eviction of TOVA (Sec. 2;
                            corollary of Thm. 1): the state's A array then holds the last step's
                            attention of every slot instead of a running sum                        */
    const int32_t *layer_K; /* DEVICE int32 [layers] or NULL: budget of each layer (PyramidKV-style
                            schedules, see ta_layer_budgets), clamped on the device to
                            [max(1, n_sink + n_recent), K]; idx rows keep K entries, cnt says how
                            many are valid                                                         */
    const uint8_t *allow;   /* DEVICE uint8 [B][n] or NULL: allowlist of positions (Sec. 5.2): an
                            anchor only counts where allow != 0                                    */
    float *margin;          /* DEVICE float [units][2] (out) or NULL: the margin of every selection the
                            call makes - units as the idx rows of that call.  With the positions in
                            the order of ta_select, the cut falls in one class (the highest that
                            loses a member; with k_protected >= 0: among the tokens that are neither
                            mandatory nor protected):
                              margin[unit][0] = smallest u among its retained members, +inf if none
                              margin[unit][1] = largest u among its evicted members
                            and (+inf, -inf) when nothing is evicted.  Equal values: positions tie
                            at the cut and the position decided; a relative gap within the rounding
                            of A names the units whose retained set another summation order of A
                            may change (the near-ties a parity check excuses).  The per-step form
                            does not write it.  4-byte aligned (else ALIGN)                        */
} ta_params;

/*
 * Per-layer budgets of a pyramidal schedule (the PyramidKV baseline, Sec. 2): an arithmetic
 * progression falling from layer 0 to the last layer, ending at k_min, with mean K:
 *   K_l = round((2K - k_min) - l (2K - 2 k_min) / (layers - 1)), the rounding residue added
 *   to layer 0 so that the budgets sum to layers * K.  One layer: K.
 *   out HOST int32 [layers].  Pass max_l K_l (= out[0]) as K and a DEVICE copy as layer_K.
 * Errors: NULL, SHAPE (layers < 1, k_min < 1, k_min > K).
 */
int32_t ta_layer_budgets(int32_t layers, int32_t K, int32_t k_min, int32_t *out);

/*
 * Shapes and strides of the cache tensors.  Strides are in ELEMENTS (bf16).
 * The innermost dimension d is contiguous everywhere.
 *   K, V : [layers][batch][hkv][n][d]     strides kv_stride = {layer, batch, head, position}
 *   Q    : [layers][batch][hq][window][d] strides q_stride  = {layer, batch, head}; rows of a
 *          head are contiguous ([window][d]).  Row w of sequence b is the query at
 *          position seq_len[b] - window + w (the last `window` positions).
 * Query head h belongs to KV head h / (hq / hkv).
 */
typedef struct ta_layout {
    int32_t layers, batch, hq, hkv;
    int32_t n;          /* padded sequence length                                   */
    int32_t window;     /* observation-window rows W (ignored when alpha == 0)      */
    int32_t d;          /* must equal TA_HEAD_DIM                                   */
    int64_t kv_stride[4];
    int64_t q_stride[3];
} ta_layout;

/* Bytes of DEVICE scratch that ta_score / ta_evict need for this layout (0 when
 * no attention term is computed).  The workspace holds per-chunk softmax row
 * statistics; its contents are meaningless between calls. */
size_t ta_workspace_bytes(const ta_layout *lay, const ta_params *prm);

/*
 * Steps 1+2 - anchor detection (Sec. 3.2; Alg. 1, detection step; S_i of Eq. 1)
 * and voucher allocation (Eq. 2; Alg. 1, voucher loops; Fig. 2).
 *
 * anchor[b][p] = 1 iff some table entry e equals tok[b][p-len[e]+1 .. p]; the
 * anchor is the last token of the n-gram, matches never cross a sequence start.
 * vouch[b][j]  = sum over anchors i with i < j <= i+L of B_i * rho^(j-i),
 *                each term B_i * (float)rho^k rounded to fp32 and added in fp32
 *                in order of increasing k = j - i; spans are clipped at seq_len.
 * spons[b][j]  = 1 iff an anchor lies in [j-L, j-1]  (<=> vouch > 0 for B > 0).
 * Positions >= seq_len[b] get 0 in all three outputs.  With prm->allow set, a
 * match only counts where allow[b][p] != 0.
 *
 *   tok       DEVICE int32 [B][n]
 *   seq_len   DEVICE int32 [B] or NULL
 *   tab_ids   HOST   int32 [E][TA_MAX_GRAM]; row e holds tab_len[e] token IDs (>= 0), rest ignored
 *   tab_len   HOST   int32 [E], each in 1..TA_MAX_GRAM;  0 <= E <= TA_MAX_TABLE
 *   anchor_B  DEVICE float [B][n] or NULL: per-anchor budget B_i read at anchor
 *             positions (confidence-weighted sponsorship, Sec. 5.1); NULL = prm->sponsor_B
 *   anchor, spons  DEVICE uint8 [B][n] (out);  vouch DEVICE float [B][n] (out)
 * Errors: NULL, SHAPE (B,n < 1; E, lengths, ids, span_L out of range).
 */
int32_t ta_match_anchors(const int32_t *tok, const int32_t *seq_len, int32_t B, int32_t n,
                         const int32_t *tab_ids, const int32_t *tab_len, int32_t E,
                         const float *anchor_B, const ta_params *prm,
                         uint8_t *anchor, uint8_t *spons, float *vouch, void *stream);

/*
 * Learned anchor detection (Sec. 5.1 "Learned Anchor Detection": detector
 * f(h) = sigmoid(W2 . GELU(W1 . h)) on the hidden state of each position, and
 * the two ways the paper feeds it into the policy).
 *   conf[b][p]     = f(h[b][p])  (bf16 inputs, fp32 accumulation, exact-erf GELU, no biases)
 *   anchor[b][p]   = 1 iff conf > thr  (strict; TA-Learned uses 0.5, TA-LearnRank 0.3)
 *   anchor_B[b][p] = at anchors: prm->sponsor_B when rank == 0 (TA-Learned, fixed budget),
 *                    scale * conf when rank != 0 (TA-LearnRank, budget proportional to the
 *                    confidence; scale = 1 gives vouchers conf * rho^k); 0 elsewhere
 * Positions >= seq_len[b] get 0 in all three outputs.  The outputs feed
 * ta_expand_vouchers (then ta_select) in place of the table match.
 *
 *   h        DEVICE bf16 [B][n][d_model], rows h_row_stride elements apart (>= d_model,
 *            multiple of 8), sequences n * h_row_stride apart; 16-byte aligned
 *   W1       DEVICE bf16 [m][d_model] contiguous, 16-byte aligned;  W2 DEVICE bf16 [m]
 *   d_model  multiple of 32, 32..32768;  m one of 32, 64, 128, 256
 *   conf, anchor_B DEVICE float [B][n] (out);  anchor DEVICE uint8 [B][n] (out)
 * Errors: NULL, SHAPE (sizes outside the ranges above, thr or scale not finite,
 *         256 * h_row_stride * 2 bytes >= 2^31), ALIGN.
 */
int32_t ta_detect_anchors(const void *h, int64_t h_row_stride, const void *W1, const void *W2,
                          const int32_t *seq_len, int32_t B, int32_t n, int32_t d_model, int32_t m,
                          float thr, int32_t rank, float scale, const ta_params *prm,
                          float *conf, uint8_t *anchor, float *anchor_B, void *stream);

/*
 * Embedding-based anchor detection (Sec. 3.2 "Anchor detection", third
 * instantiation; TA-Fast-Embedding of Sec. 3.4 and Sec. 5.3): similarity of an
 * input embedding to a set of anchor-concept embeddings,
 *   sim[b][p]    = max over e < E of  (x . c_e) / (|x| |c_e|)   (a cosine with a zero
 *                  vector on either side counts as 0; bf16 inputs, fp32 accumulation)
 *   anchor[b][p] = 1 iff sim > tau  (strict; the paper gives no value for tau)
 * Positions >= seq_len[b] get 0 in both outputs.  Input embeddings depend on the
 * token ID only: run this over the embedding table once (B = 1, n = vocabulary
 * size) and use ta_lookup_anchors per sequence, or run it per position.
 *
 *   x        DEVICE bf16 [B][n][d_model], rows x_row_stride elements apart (>= d_model,
 *            multiple of 8), sequences n * x_row_stride apart; 16-byte aligned
 *   C        DEVICE bf16 [E][d_model] contiguous, 16-byte aligned;  1 <= E <= 256
 *   d_model  multiple of 32, 32..32768
 *   sim      DEVICE float [B][n] (out);  anchor DEVICE uint8 [B][n] (out)
 * Errors: NULL, SHAPE (as ta_detect_anchors; E out of range; tau not finite), ALIGN.
 */
int32_t ta_embed_anchors(const void *x, int64_t x_row_stride, const void *C, int32_t E,
                         const int32_t *seq_len, int32_t B, int32_t n, int32_t d_model, float tau,
                         float *sim, uint8_t *anchor, void *stream);

/*
 * Anchor flags of token IDs from per-vocabulary flags (the output of
 * ta_embed_anchors over the embedding table):
 *   anchor[b][p] = 1 iff p < seq_len[b], 0 <= tok[b][p] < V and vocab_anchor[tok[b][p]] != 0.
 *   tok DEVICE int32 [B][n]; vocab_anchor DEVICE uint8 [V]; anchor DEVICE uint8 [B][n] (out)
 * Errors: NULL, SHAPE (B, n, V < 1).
 */
int32_t ta_lookup_anchors(const int32_t *tok, const int32_t *seq_len, int32_t B, int32_t n,
                          const uint8_t *vocab_anchor, int32_t V, uint8_t *anchor, void *stream);

/*
 * Step 2 alone - voucher allocation (Eq. 2; Alg. 1, voucher loops) from anchor
 * flags that were not produced by the table match (learned detection, Sec. 5.1).
 * vouch and spons exactly as defined under ta_match_anchors, with
 * anchor[b][i] != 0 marking the anchors (flags at positions >= seq_len are ignored).
 *   anchor    DEVICE uint8 [B][n] (in);  anchor_B DEVICE float [B][n] or NULL (= prm->sponsor_B)
 *   spons     DEVICE uint8 [B][n] (out); vouch DEVICE float [B][n] (out)
 * Errors: NULL, SHAPE (B, n < 1; span_L out of range).
 */
int32_t ta_expand_vouchers(const uint8_t *anchor, const float *anchor_B, const int32_t *seq_len,
                           int32_t B, int32_t n, const ta_params *prm,
                           uint8_t *spons, float *vouch, void *stream);

/*
 * Step 3 - attention term A_i of Eq. 1 (cumulative attention over heads and
 * steps; dormant-token definition, App. A), computed SnapKV/H2O style over an
 * observation window: for every unit (layer, b, g)
 *   A[i] = sum over the hq/hkv query heads h of group g and rows w < W of
 *          softmax_i( q_{h,w} . k_i / sqrt(d) ) over the keys visible to row w.
 * bf16 inputs, fp32 accumulation and softmax.  A[i] = 0 for i >= seq_len[b].
 *
 *   Q, K   DEVICE bf16, laid out per `lay`
 *   A      DEVICE float [layers][batch][hkv][n] (out, contiguous)
 *   ws     DEVICE scratch of at least ta_workspace_bytes() bytes, 16-byte aligned
 * Errors: NULL, SHAPE (d != 128, hq % hkv != 0, W < 1, W > n,
 *         (hq/hkv)*W > TA_MAX_ROWS), ALIGN, WORKSPACE.
 */
int32_t ta_score(const void *Q, const void *K, const ta_layout *lay, const int32_t *seq_len,
                 const ta_params *prm, float *A, void *ws, size_t ws_bytes, void *stream);

/*
 * Step 3 fused with the prefill attention (Sec. 3.4, Sec. 4.7: SDPA / FlashAttention
 * backends never materialise the attention matrix).  Such a kernel already sweeps the keys
 * for the window's queries and leaves the log-sum-exp of every row's scaled logits,
 *   lse[l][b][h][w] = log sum over the keys visible to row w of exp(q_{h,w} . k_i / sqrt(d))
 * (natural logarithm; -inf for a row that sees no key).  Given it, the attention weight of
 * a key is exp(s - lse) and A needs ONE sweep over K instead of two:
 *   A[i] = sum over the group's heads h and rows w of exp(q_{h,w} . k_i / sqrt(d) - lse).
 * Same inputs, output, masking and errors as ta_score; no workspace.
 *   lse  DEVICE float [layers][batch][hq][window], contiguous
 */
int32_t ta_score_lse(const void *Q, const void *K, const ta_layout *lay, const int32_t *seq_len,
                     const ta_params *prm, const float *lse, float *A, void *stream);

/*
 * Step 4 - utility and protected top-K (Eq. 1 / Eq. 3; Alg. 1, utility and
 * top-K steps; Sec. 3.3; Thm. 2-4; budget-partition table, App. D).
 *   u_p   = alpha*A_p + beta*(p+1)/len + gamma*anchor_p + vouch_p   (fp32, each product
 *           and sum rounded, left to right; A is not read when alpha == 0)
 *   class = 2 if p < n_sink or p >= len - n_recent; 1 if sponsored; else 0
 * The retained set of a unit is the first min(K, len) positions under the total
 * order (class descending, u descending, position descending), written in
 * ascending position order.  NaN utilities are not supported.
 *
 *   A       DEVICE float [layers][batch][hkv][n], or NULL when alpha == 0
 *   anchor, spons DEVICE uint8 [batch][n]; vouch DEVICE float [batch][n]
 *   idx     DEVICE int32 [layers][batch][hkv][K] (out; entries >= cnt are left untouched)
 *   cnt     DEVICE int32 [layers][batch][hkv]    (out; = min(K, len))
 * The retained set of TA-Fast does not depend on layer or head: call with
 * layers = hkv = 1 and share idx across units (see ta_compact).
 * prm->pool_k, prm->k_protected and prm->layer_K modify the selection as described
 * at ta_params; prm->margin, if set, receives the margin of every unit's cut.
 * Errors: NULL, SHAPE (also pool_k not in {1,3,5,7,9}), BUDGET.
 */
int32_t ta_select(const float *A, const uint8_t *anchor, const uint8_t *spons, const float *vouch,
                  const int32_t *seq_len, int32_t layers, int32_t batch, int32_t hkv, int32_t n,
                  int32_t K, const ta_params *prm, int32_t *idx, int32_t *cnt, void *stream);

/*
 * Step 5 - eviction (Sec. 3.2 "Token selection": index_select on the KV tensors
 * along the sequence dimension; Alg. 1, eviction step).
 *   Kout[unit][r][:] = Kin[unit][idx[r]][:],  Vout likewise,  for r < cnt.
 * Rows r >= cnt of the outputs are left untouched.
 *
 *   Kin, Vin   DEVICE bf16 per `lay` (kv_stride)
 *   idx, cnt   DEVICE int32: [layers][batch][hkv][K] / [layers][batch][hkv], or, when
 *              idx_shared != 0, [batch][K] / [batch] used by every layer and head
 *   Kout, Vout DEVICE bf16 [layers][batch][hkv][K][d] (out, contiguous)
 * Every idx entry below cnt must be a valid position (< n); entries are clamped
 * to [0, n-1] on the device so a corrupt index cannot fault.
 * Errors: NULL, SHAPE, ALIGN.
 */
int32_t ta_compact(const void *Kin, const void *Vin, const int32_t *idx, const int32_t *cnt,
                   const ta_layout *lay, int32_t K, int32_t idx_shared,
                   void *Kout, void *Vout, void *stream);

/*
 * The whole pass (Alg. 1 without the budget-decay step, which only matters
 * between decode steps): match + vouchers once per sequence, then score,
 * select and compact for every unit.  Arguments as in the four calls above.
 * With prm->alpha == 0 (TA-Fast, Eq. 3) Q, A and ws may be NULL, the retained
 * set is computed once per sequence and idx / cnt have the shared shapes
 * [batch][K] / [batch]; otherwise they are per unit.
 */
int32_t ta_evict(const int32_t *tok, const int32_t *seq_len,
                 const int32_t *tab_ids, const int32_t *tab_len, int32_t E, const float *anchor_B,
                 const void *Q, const void *Kin, const void *Vin,
                 const ta_layout *lay, const ta_params *prm, int32_t K,
                 uint8_t *anchor, uint8_t *spons, float *vouch, float *A,
                 int32_t *idx, int32_t *cnt, void *Kout, void *Vout,
                 void *ws, size_t ws_bytes, void *stream);

/*
 * Paged (block-table) caches, the layout of serving engines: K and V rows of a sequence
 * live in pages of page_size positions scattered over a pool; entry j of a sequence's row
 * of the block table is the page that holds its positions [j*page_size, (j+1)*page_size).
 * Row p of KV head g of sequence b in layer l starts at element
 *   l*stride[0] + block_table[b][p / page_size]*stride[1] + (p % page_size)*stride[2] + g*stride[3]
 * of the pool ([pages][page_size][heads][d] and [pages][heads][page_size][d] are both
 * expressible).  Table entries are clamped to [0, num_pages - 1] on the device, so a
 * corrupt table cannot fault.  With a paged cache, ta_layout gives the sizes and the query
 * strides; its kv_stride is not used.
 */
typedef struct ta_paged_kv {
    int32_t page_size;          /* positions per page; scoring needs a multiple of 64           */
    int32_t max_pages;          /* block-table entries per sequence; max_pages*page_size >= n   */
    int32_t num_pages;          /* pages in the pool                                            */
    const int32_t *block_table; /* DEVICE int32 [batch][max_pages]                              */
    int64_t stride[4];          /* ELEMENTS: {layer, page, position, head}; multiples of 8      */
} ta_paged_kv;

/*
 * Steps 3 and 5 over a paged cache: ta_score / ta_score_lse (lse != NULL: one sweep, ws
 * not used) and ta_compact with the rows addressed through the block table.  Outputs as in
 * the dense calls (A [layers][batch][hkv][n]; Kout, Vout dense [layers][batch][hkv][K][d]).
 * Errors: as the dense calls; SHAPE also for page_size < 1 (scoring: not a multiple of 64),
 * max_pages*page_size < n, num_pages < 1, negative strides; ALIGN for strides that are
 * not multiples of 8 or pools that are not 16-byte aligned; NULL for a missing table.
 */
int32_t ta_score_paged(const void *Q, const void *Kpool, const ta_paged_kv *pg, const ta_layout *lay,
                       const int32_t *seq_len, const ta_params *prm, const float *lse,
                       float *A, void *ws, size_t ws_bytes, void *stream);
int32_t ta_compact_paged(const void *Kpool, const void *Vpool, const ta_paged_kv *pg,
                         const int32_t *idx, const int32_t *cnt, const ta_layout *lay, int32_t K,
                         int32_t idx_shared, void *Kout, void *Vout, void *stream);

/*
 * Step 5 straight into a page pool (Sec. 3.2 "Token selection" on the block-table caches of serving
 * engines): the r-th retained row of unit (l, b, g) is written to slot r of sequence b's pages in the
 * destination pool,
 *   Kdst[l*dst->stride[0] + dst->block_table[b][r / ps]*dst->stride[1] + (r % ps)*dst->stride[2] + g*dst->stride[3]]
 * (ps = dst->page_size, dst->max_pages * ps >= K), Vdst likewise: the layout a paged ta_decode_state
 * reads, so the generation steps can start from these pages without another copy.
 * The source is dense (`src` NULL, strides from lay->kv_stride) or paged (`src`).  Source and
 * destination may be the same pool as long as no destination page holds source rows of the call:
 * pages are read and written in no fixed order.
 * Errors: as ta_compact_paged for both descriptions; SHAPE if dst->max_pages * ps < K.
 */
int32_t ta_compact_into_pages(const void *Kin, const void *Vin, const ta_paged_kv *src,
                              const int32_t *idx, const int32_t *cnt, const ta_layout *lay, int32_t K,
                              int32_t idx_shared, void *Kdst, void *Vdst, const ta_paged_kv *dst, void *stream);

/*
 * The whole pass with the one-sweep score of ta_score_lse: as ta_evict for prm->alpha != 0,
 * with the row log-sum-exps of the prefill attention kernel in place of the workspace.
 * Errors: as ta_evict; SHAPE when prm->alpha == 0.
 */
int32_t ta_evict_lse(const int32_t *tok, const int32_t *seq_len,
                     const int32_t *tab_ids, const int32_t *tab_len, int32_t E, const float *anchor_B,
                     const void *Q, const void *Kin, const void *Vin, const float *lse,
                     const ta_layout *lay, const ta_params *prm, int32_t K,
                     uint8_t *anchor, uint8_t *spons, float *vouch, float *A,
                     int32_t *idx, int32_t *cnt, void *Kout, void *Vout, void *stream);

/*
 * The whole pass over a paged cache: as ta_evict (lse == NULL; ws as there) or ta_evict_lse
 * (lse != NULL; ws unused), with K and V addressed through the block table of `pg`.
 * Outputs as in the dense calls.  Errors: as ta_evict / ta_score_paged / ta_compact_paged.
 */
int32_t ta_evict_paged(const int32_t *tok, const int32_t *seq_len,
                       const int32_t *tab_ids, const int32_t *tab_len, int32_t E, const float *anchor_B,
                       const void *Q, const void *Kpool, const void *Vpool, const ta_paged_kv *pg,
                       const float *lse, const ta_layout *lay, const ta_params *prm, int32_t K,
                       uint8_t *anchor, uint8_t *spons, float *vouch, float *A,
                       int32_t *idx, int32_t *cnt, void *Kout, void *Vout,
                       void *ws, size_t ws_bytes, void *stream);

/*
 * Caches kept as one tensor per layer (the `past_key_values` order that Sec. 3.2 "Token
 * selection" applies index_select to is a list of per-layer K and V tensors): HOST arrays of
 * lay->layers DEVICE pointers, read during the call.  Layer l of K and V is a
 * [batch][hkv][n][d] tensor with the strides kv_stride[1..3] of `lay`, layer l of Q a
 * [batch][hq][window][d] tensor with q_stride[1..2]; Kout[l], Vout[l] are dense
 * [batch][hkv][K][d].  kv_stride[0] and q_stride[0] are not used.
 */
typedef struct ta_layer_ptrs {
    const void *const *Q;     /* HOST [layers] of DEVICE bf16; may be NULL when prm->alpha == 0 */
    const void *const *K;     /* HOST [layers] of DEVICE bf16 */
    const void *const *V;     /* HOST [layers] of DEVICE bf16 */
    void *const *Kout;        /* HOST [layers] of DEVICE bf16 */
    void *const *Vout;        /* HOST [layers] of DEVICE bf16 */
} ta_layer_ptrs;

/*
 * ta_evict over per-layer tensors: the same kernels in the same launches (one pass over all
 * layers, not one per layer), each layer's base address taken from `lp` instead of
 * base + l * layer stride.  Every other argument and output as in ta_evict, except
 *   ws   DEVICE, at least ta_workspace_bytes(lay, prm) rounded up to a multiple of 256, plus
 *        TA_LAYER_WS_BYTES (needed when prm->alpha == 0 too): the table is validated on the
 *        host and then kept there for the kernels.
 * Errors: as ta_evict; SHAPE also for lay->layers > TA_MAX_LAYER_PTRS; NULL for a missing
 * array or entry; ALIGN for an entry that is not 16-byte aligned; SHAPE for an output entry
 * equal to an input entry of the same layer.
 */
int32_t ta_evict_layers(const int32_t *tok, const int32_t *seq_len,
                        const int32_t *tab_ids, const int32_t *tab_len, int32_t E, const float *anchor_B,
                        const ta_layer_ptrs *lp, const ta_layout *lay, const ta_params *prm, int32_t K,
                        uint8_t *anchor, uint8_t *spons, float *vouch, float *A,
                        int32_t *idx, int32_t *cnt, void *ws, size_t ws_bytes, void *stream);

/*
 * ta_evict_paged over one page pool per layer (serving engines allocate the pools of a layer
 * on their own and share the block table between the layers): lp->K[l], lp->V[l] are the
 * pools of layer l, addressed through pg->block_table with the strides pg->stride[1..3]
 * (pg->stride[0] is not used: pass 0); lp->Q, lp->Kout, lp->Vout as in ta_evict_layers; lse as in
 * ta_evict_paged (NULL: two sweeps).  ws as in ta_evict_layers (with lse != NULL only the
 * TA_LAYER_WS_BYTES of the table are needed).
 * Errors: as ta_evict_paged and ta_evict_layers.
 */
int32_t ta_evict_layers_paged(const int32_t *tok, const int32_t *seq_len,
                              const int32_t *tab_ids, const int32_t *tab_len, int32_t E, const float *anchor_B,
                              const ta_layer_ptrs *lp, const ta_paged_kv *pg, const float *lse,
                              const ta_layout *lay, const ta_params *prm, int32_t K,
                              uint8_t *anchor, uint8_t *spons, float *vouch, float *A,
                              int32_t *idx, int32_t *cnt, void *ws, size_t ws_bytes, void *stream);

/*
 * Incremental form: the same retention policy applied after every generation
 * step (Sec. 3.1 "after each generation step"; Alg. 1 including its last step,
 * the budget decay B_i <- decay * B_i of Sec. 3.2 "Token selection").
 *
 * State (all DEVICE memory owned by the caller, sized by the fields below):
 *   per sequence  tok    int32 [batch][cap]   token stream
 *                 len    int32 [batch]        current length
 *                 anchor uint8 [batch][cap]   anchor flags
 *                 budget float [batch][cap]   CURRENT budget B_i of each anchor, 0 elsewhere
 *                 vouch  float [batch][cap]   scratch of a step: voucher of each position from the
 *                 spons  uint8 [batch][cap]   current budgets (Eq. 2), and its flags (bit 0: sponsored,
 *                                             bit 1: an anchor itself, except at the position just
 *                                             appended); rewritten by every ta_decode_step
 *                 stepped int32 [batch]       scratch of a step: 0 if the sequence was at capacity and
 *                                             left alone, else its new length in bits 0-29 and, in
 *                                             bit 30, whether the appended token is an anchor
 *   per unit      Kc, Vc bf16  [layers][batch][hkv][K+1][d]  cache slots
 *                 pos    int32 [layers][batch][hkv][K+1]     absolute position of a slot, -1 = free
 *                 A      float [layers][batch][hkv][K+1]     cumulative attention of a slot
 * A unit keeps at most K rows; the extra slot receives the next token.  Slots
 * are stable: an evicted slot is reused, rows are never moved (keys are stored
 * with their positional encoding, so slot order does not matter to attention).
 *
 * `pages` (HOST pointer, NULL = the dense layout above) keeps the K/V slots in a paged pool, the
 * cache layout of serving engines (see ta_paged_kv): Kc and Vc are then the pools, and slot s of
 * KV head g of sequence b in layer l starts at element
 *   l*stride[0] + block_table[b][s / page_size]*stride[1] + (s % page_size)*stride[2] + g*stride[3];
 * max_pages * page_size >= K + 1; table entries are clamped to the pool on the device.  pos and A
 * stay dense.  Every sequence needs pages of its own (a page shared by two sequences would be
 * written by both).
 */
typedef struct ta_decode_state {
    int32_t layers, batch, hq, hkv, d;
    int32_t K;       /* budget per unit; slots per unit = K + 1, 1 <= K <= TA_MAX_DECODE_K */
    int32_t cap;     /* positions the per-sequence arrays can hold                        */
    int32_t *tok;
    int32_t *len;
    uint8_t *anchor;
    float *budget;
    float *vouch;
    uint8_t *spons;
    void *Kc, *Vc;
    int32_t *pos;
    float *A;
    int32_t *stepped;
    const ta_paged_kv *pages;
} ta_decode_state;

#define TA_MAX_DECODE_K 2047

/*
 * Fills a decode state from the outputs of a prefill eviction (ta_evict /
 * ta_match_anchors + ta_score + ta_select + ta_compact with per-unit idx):
 * tokens, anchor flags and budgets (anchor_B, or prm->sponsor_B at anchors) are
 * copied for positions < seq_len; slot r < cnt of a unit gets row r of
 * Kout/Vout, position idx[r] and attention A[idx[r]] (0 when A is NULL); the
 * remaining slots are free.
 *   tok int32 [batch][n], seq_len int32 [batch] or NULL, anchor uint8 [batch][n],
 *   anchor_B float [batch][n] or NULL, A float [layers][batch][hkv][n] or NULL,
 *   idx int32 [layers][batch][hkv][K], cnt int32 [layers][batch][hkv],
 *   Kout, Vout bf16 [layers][batch][hkv][K][d]           (all DEVICE)
 * With a paged state (st->pages) Kout and Vout may both be NULL: the retained rows are then taken
 * to be in place already - row r of a unit in its slot r, as ta_compact_into_pages leaves them -
 * and only positions and attention are filled in.
 * Errors: NULL, SHAPE (n > cap, K out of range, d != 128, hq % hkv != 0, more than 16 query
 * heads per KV head, (hq/hkv) * (K + 1) > 15360; paged: sizes and strides as in ta_paged_kv,
 * max_pages * page_size < K + 1), ALIGN.
 */
int32_t ta_decode_init(const ta_decode_state *st, const int32_t *tok, const int32_t *seq_len, int32_t n,
                       const uint8_t *anchor, const float *anchor_B, const float *A,
                       const int32_t *idx, const int32_t *cnt, const void *Kout, const void *Vout,
                       const ta_params *prm, void *stream);

/*
 * One generation step for every sequence and unit:
 *   1. append new_tok[b] at position p = len[b]; the anchor flag of p follows the
 *      rule of ta_match_anchors evaluated at p only; its budget is sponsor_B; len += 1
 *   2. per unit: the new k/v row goes into the lowest-numbered free slot with A = 0;
 *      with alpha != 0 each of the hq/hkv decode queries of the group adds its
 *      softmax weights over the occupied slots (q.k/sqrt(d), fp32) to A
 *      (prm->last_query: A of every occupied slot is REPLACED by this step's weights)
 *   3. per unit, if no slot is free: the slot ranking last under the order of
 *      ta_select - classes and the recency term taken from absolute positions and
 *      the new length, vouchers recomputed from the current budgets - is freed
 *   4. every budget is multiplied by prm->budget_decay
 *   new_tok int32 [batch]; q_new bf16 [layers][batch][hq][d] (NULL when alpha == 0);
 *   k_new, v_new bf16 [layers][batch][hkv][d]; table as in ta_match_anchors (HOST);
 *   evicted int32 [layers][batch][hkv] or NULL: position freed in step 3, -1 if none.
 * The caller keeps len[b] < cap; a sequence at capacity (len[b] >= cap) is left unchanged:
 * nothing is appended, no attention is added, nothing is evicted (evicted = -1 for its
 * units) and its budgets do not decay.
 * Errors: NULL, SHAPE, BUDGET (K < n_sink + n_recent), ALIGN.
 */
int32_t ta_decode_step(const ta_decode_state *st, const int32_t *new_tok, const void *q_new,
                       const void *k_new, const void *v_new,
                       const int32_t *tab_ids, const int32_t *tab_len, int32_t E,
                       const ta_params *prm, int32_t *evicted, void *stream);

/*
 * One-time set-up of the library on the CURRENT device: kernel attributes (dynamic LDS sizes)
 * and the device address of the static scratch buffer of ta_evict_static.  Every entry point
 * performs the part it needs on its first call on a device, so calling ta_init is optional -
 * except before a stream capture or inside code that must not touch the runtime beyond
 * launches: call it once per device beforehand.  Allocates nothing.  Returns TA_OK or TA_ERR_HIP.
 */
int32_t ta_init(void);

/*
 * ta_evict for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * outputs, kernels and errors as ta_evict, minus `ws` / `ws_bytes`: the per-chunk softmax row
 * statistics of the score step go to a static device buffer of TA_STATIC_SCRATCH_BYTES that
 * lives inside the library (one copy per GPU, held until the process ends).  The call
 * allocates and frees nothing and calls no allocating routine.
 *   - A layout whose ta_workspace_bytes() exceeds TA_STATIC_SCRATCH_BYTES is refused with
 *     TA_ERR_SCRATCH before anything is launched (the full-model, long-context and agentic
 *     prefill shapes need 0.5, 2 and 16 MiB).
 *   - `stream` must belong to the current device.
 *   - Every call on a GPU uses that GPU's one buffer: calls that may overlap on one GPU
 *     (different streams, different threads) race on it and must be serialised by the caller.
 *     Nothing in the buffer has to start at zero (every statistic is written by the first
 *     sweep before the second reads it), so the previous call's contents do no harm.
 *   - The first call on a device looks up the buffer's address (ta_init does the same ahead
 *     of time).
 */
#define TA_STATIC_SCRATCH_BYTES (32u << 20)
int32_t ta_evict_static(const int32_t *tok, const int32_t *seq_len,
                        const int32_t *tab_ids, const int32_t *tab_len, int32_t E, const float *anchor_B,
                        const void *Q, const void *Kin, const void *Vin,
                        const ta_layout *lay, const ta_params *prm, int32_t K,
                        uint8_t *anchor, uint8_t *spons, float *vouch, float *A,
                        int32_t *idx, int32_t *cnt, void *Kout, void *Vout, void *stream);

/* Text for a ta_status value (static storage). */
const char *ta_strerror(int32_t status);
/* Raw hipError_t of the most recent TA_ERR_HIP on this thread (0 if none). */
int32_t ta_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TA_H */
