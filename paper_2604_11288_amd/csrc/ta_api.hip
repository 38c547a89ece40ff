// C-ABI front end: argument validation on the host, then launches.  Every
// check happens before the first launch, so any status other than TA_ERR_HIP
// means nothing was enqueued.
#include <math.h>
#include <string.h>

#include "ta_internal.h"

// Scratch of ta_evict_static: per-chunk softmax row statistics of the score step.  Host code
// never uses this name as an address (it is a host-side stand-in): the device address is looked
// up once per device with hipGetSymbolAddress and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[TA_STATIC_SCRATCH_BYTES];

namespace {

ta::DeviceOnce g_scratch_once;
void* g_scratch_ptr[64];                                   // per device, valid once g_scratch_once has run there

// (a plain host function: the compiler gives the array a symbol the runtime can find only when
// it sees host code name it, and the call operator of a lambda does not count as host code)
hipError_t scratch_address(void** p) { return hipGetSymbolAddress(p, HIP_SYMBOL(scratch)); }

hipError_t scratch_setup()
{
    return g_scratch_once.run([](int dev) {
        void* p = nullptr;
        const hipError_t e = scratch_address(&p);
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
        return hipSuccess;
    });
}

thread_local int32_t t_last_hip_error = 0;

int32_t hip_status(hipError_t e)
{
    if (e == hipSuccess) return TA_OK;
    t_last_hip_error = (int32_t)e;
    return TA_ERR_HIP;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

int32_t check_params(const ta_params* prm)
{
    if (!prm) return TA_ERR_NULL;
    if (prm->n_sink < 0 || prm->n_recent < 0) return TA_ERR_SHAPE;
    if (prm->span_L < 0 || prm->span_L > TA_MAX_SPAN) return TA_ERR_SHAPE;
    if (!(prm->rho >= 0.0) || !isfinite(prm->rho)) return TA_ERR_SHAPE;
    if (!isfinite(prm->alpha) || !isfinite(prm->beta) || !isfinite(prm->gamma) ||
        !isfinite(prm->sponsor_B))
        return TA_ERR_SHAPE;
    if (prm->pool_k != 0 && prm->pool_k != 1 && prm->pool_k != 3 && prm->pool_k != 5 && prm->pool_k != 7 &&
        prm->pool_k != 9)
        return TA_ERR_SHAPE;
    if (prm->last_query != 0 && prm->last_query != 1) return TA_ERR_SHAPE;
    if (((uintptr_t)prm->margin & 3u) != 0) return TA_ERR_ALIGN;
    return TA_OK;
}

int32_t check_budget(const ta_params* prm, int32_t K)
{
    if (K < 1) return TA_ERR_BUDGET;
    if ((int64_t)prm->n_sink + prm->n_recent > K) return TA_ERR_BUDGET;
    return TA_OK;
}

// Shapes shared by score / compact / evict.
int32_t check_layout(const ta_layout* lay, bool need_q)
{
    if (!lay) return TA_ERR_NULL;
    if (lay->layers < 1 || lay->batch < 1 || lay->hkv < 1 || lay->n < 1) return TA_ERR_SHAPE;
    if (lay->d != TA_HEAD_DIM) return TA_ERR_SHAPE;
    if (lay->batch > 65535) return TA_ERR_SHAPE;
    if ((int64_t)lay->layers * lay->batch * lay->hkv > (1 << 24)) return TA_ERR_SHAPE;
    for (int i = 0; i < 4; ++i)
        if (lay->kv_stride[i] < 0) return TA_ERR_SHAPE;
    if (lay->kv_stride[3] < lay->d) return TA_ERR_SHAPE;
    if ((lay->kv_stride[3] / 8) * (int64_t)lay->n >= 0x7FFFFFFFll) return TA_ERR_SHAPE;   // 32-bit row offsets
    for (int i = 0; i < 4; ++i)
        if (lay->kv_stride[i] % 8 != 0) return TA_ERR_ALIGN;
    if (need_q) {
        if (lay->hq < 1 || lay->hq % lay->hkv != 0) return TA_ERR_SHAPE;
        if (lay->window < 1 || lay->window > lay->n) return TA_ERR_SHAPE;
        if ((int64_t)(lay->hq / lay->hkv) * lay->window > TA_MAX_ROWS) return TA_ERR_SHAPE;
        for (int i = 0; i < 3; ++i) {
            if (lay->q_stride[i] < 0) return TA_ERR_SHAPE;
            if (lay->q_stride[i] % 8 != 0) return TA_ERR_ALIGN;
        }
        if (lay->q_stride[2] < (int64_t)lay->window * lay->d) return TA_ERR_SHAPE;
    }
    return TA_OK;
}

int32_t build_table(const int32_t* tab_ids, const int32_t* tab_len, int32_t E, const ta_params* prm,
                    ta::MatchTable* out)
{
    if (E < 0 || E > TA_MAX_TABLE) return TA_ERR_SHAPE;
    if (E > 0 && (!tab_ids || !tab_len)) return TA_ERR_NULL;
    memset(out, 0, sizeof(*out));
    for (int e = 0; e < E; ++e) {
        const int32_t len = tab_len[e];
        if (len < 1 || len > TA_MAX_GRAM) return TA_ERR_SHAPE;
        for (int t = 0; t < len; ++t) {
            const int32_t id = tab_ids[e * TA_MAX_GRAM + t];
            if (id < 0) return TA_ERR_SHAPE;
            out->rid[e][len - 1 - t] = id;                  // reversed: last token first
        }
        for (int t = len; t < TA_MAX_GRAM; ++t) out->rid[e][t] = -1;
        out->len[e] = len;
    }
    out->E = E;
    out->L = prm->span_L;
    out->B = prm->sponsor_B;
    for (int k = 0; k <= TA_MAX_SPAN; ++k) out->pw[k] = (float)pow(prm->rho, (double)k);
    return TA_OK;
}

size_t workspace_bytes(const ta_layout* lay) { return ta::score_workspace_bytes(*lay); }

int32_t check_match(const int32_t* tok, int32_t B, int32_t n, const ta_params* prm,
                    const uint8_t* anchor, const uint8_t* spons, const float* vouch)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    if (!tok || !anchor || !spons || !vouch) return TA_ERR_NULL;
    if (B < 1 || n < 1 || B > 65535) return TA_ERR_SHAPE;
    return TA_OK;
}

int32_t check_score(const void* Q, const void* K, const ta_layout* lay, const ta_params* prm,
                    const float* A, const void* ws, size_t ws_bytes)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    rc = check_layout(lay, true);
    if (rc != TA_OK) return rc;
    if (!Q || !K || !A) return TA_ERR_NULL;
    if (!aligned16(Q) || !aligned16(K)) return TA_ERR_ALIGN;
    if (!ws || ws_bytes < workspace_bytes(lay)) return TA_ERR_WORKSPACE;
    if (!aligned16(ws)) return TA_ERR_ALIGN;
    if (ta::score_grid_blocks(*lay) > 0x7FFFFFFFll) return TA_ERR_SHAPE;
    return TA_OK;
}

int32_t check_select(const float* A, const uint8_t* anchor, const uint8_t* spons, const float* vouch,
                     int32_t layers, int32_t batch, int32_t hkv, int32_t n, int32_t K,
                     const ta_params* prm, const int32_t* idx, const int32_t* cnt)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    if (!anchor || !spons || !vouch || !idx || !cnt) return TA_ERR_NULL;
    if (prm->alpha != 0.0f && !A) return TA_ERR_NULL;
    if (layers < 1 || batch < 1 || hkv < 1 || n < 1) return TA_ERR_SHAPE;
    if ((int64_t)layers * batch * hkv > (1 << 24)) return TA_ERR_SHAPE;
    return check_budget(prm, K);
}

// `same_pool_ok`: the outputs are page pools that may be the input pools (the caller keeps source and
// destination pages apart); otherwise outputs must not alias the inputs.
int32_t check_compact(const void* Kin, const void* Vin, const int32_t* idx, const int32_t* cnt,
                      const ta_layout* lay, int32_t K, const void* Kout, const void* Vout, bool same_pool_ok = false)
{
    int32_t rc = check_layout(lay, false);
    if (rc != TA_OK) return rc;
    if (!Kin || !Vin || !idx || !cnt || !Kout || !Vout) return TA_ERR_NULL;
    if (K < 1) return TA_ERR_SHAPE;
    if (!aligned16(Kin) || !aligned16(Vin) || !aligned16(Kout) || !aligned16(Vout)) return TA_ERR_ALIGN;
    // outputs must not alias the inputs or each other: workgroups read and write rows in no fixed order
    if (Kout == Vout || Kout == Vin || Vout == Kin) return TA_ERR_SHAPE;
    if (!same_pool_ok && (Kout == Kin || Vout == Vin)) return TA_ERR_SHAPE;
    const int64_t units = (int64_t)lay->layers * lay->batch * lay->hkv;
    if (units * ((K + 63) / 64) > 0x7FFFFFFFll) return TA_ERR_SHAPE;
    return TA_OK;
}

int32_t check_decode_state(const ta_decode_state* st)
{
    if (!st) return TA_ERR_NULL;
    if (!st->tok || !st->len || !st->anchor || !st->budget || !st->vouch || !st->spons || !st->Kc || !st->Vc ||
        !st->pos || !st->A || !st->stepped)
        return TA_ERR_NULL;
    if (st->layers < 1 || st->batch < 1 || st->hkv < 1 || st->hq < 1 || st->hq % st->hkv != 0) return TA_ERR_SHAPE;
    if (st->hq / st->hkv > 16) return TA_ERR_SHAPE;        // the heads of a group are the 16 columns of an MFMA tile
    if (st->d != TA_HEAD_DIM) return TA_ERR_SHAPE;
    if (st->K < 1 || st->K > TA_MAX_DECODE_K) return TA_ERR_SHAPE;
    if ((int64_t)(st->hq / st->hkv) * (st->K + 1) > 15360) return TA_ERR_SHAPE;      // logits of a unit sit in LDS
    if (st->cap < 1 || st->cap >= (1 << 30) || st->batch > 65535) return TA_ERR_SHAPE;
    if ((int64_t)st->layers * st->batch * st->hkv > (1 << 24)) return TA_ERR_SHAPE;
    // one launch holds the units and one workgroup per 256 positions of every sequence
    if ((int64_t)st->batch * ((st->cap + 255) / 256) > 0x7F000000ll - (1 << 24)) return TA_ERR_SHAPE;
    if (!aligned16(st->Kc) || !aligned16(st->Vc)) return TA_ERR_ALIGN;
    if (st->pages) {                                       // K/V slots in a paged pool
        const ta_paged_kv* pg = st->pages;
        if (!pg->block_table) return TA_ERR_NULL;
        if (pg->page_size < 1 || pg->max_pages < 1 || pg->num_pages < 1) return TA_ERR_SHAPE;
        if ((int64_t)pg->max_pages * pg->page_size < (int64_t)st->K + 1) return TA_ERR_SHAPE;
        for (int i = 0; i < 4; ++i) {
            if (pg->stride[i] < 0) return TA_ERR_SHAPE;
            if (pg->stride[i] % 8 != 0) return TA_ERR_ALIGN;
        }
        if (pg->stride[2] < st->d) return TA_ERR_SHAPE;
    }
    return TA_OK;
}

}  // namespace

extern "C" {

size_t ta_workspace_bytes(const ta_layout* lay, const ta_params* prm)
{
    if (!lay || !prm) return 0;
    if (prm->alpha == 0.0f) return 0;
    if (check_layout(lay, true) != TA_OK) return 0;
    return workspace_bytes(lay);
}

int32_t ta_layer_budgets(int32_t layers, int32_t K, int32_t k_min, int32_t* out)
{
    if (!out) return TA_ERR_NULL;
    if (layers < 1 || k_min < 1 || k_min > K) return TA_ERR_SHAPE;
    if (layers == 1) {
        out[0] = K;
        return TA_OK;
    }
    const double first = 2.0 * K - k_min, fall = (2.0 * K - 2.0 * k_min) / (layers - 1);
    int64_t total = 0;
    for (int32_t l = 0; l < layers; ++l) {
        out[l] = (int32_t)floor(first - fall * l + 0.5);
        total += out[l];
    }
    out[0] += (int32_t)((int64_t)layers * K - total);        // rounding residue
    return TA_OK;
}

int32_t ta_match_anchors(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                         const int32_t* tab_ids, const int32_t* tab_len, int32_t E,
                         const float* anchor_B, const ta_params* prm,
                         uint8_t* anchor, uint8_t* spons, float* vouch, void* stream)
{
    int32_t rc = check_match(tok, B, n, prm, anchor, spons, vouch);
    if (rc != TA_OK) return rc;
    ta::MatchTable tab;
    rc = build_table(tab_ids, tab_len, E, prm, &tab);
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_match(tok, seq_len, B, n, tab, anchor_B, prm->allow, anchor, spons, vouch,
                                       (hipStream_t)stream));
}

int32_t ta_detect_anchors(const void* h, int64_t h_row_stride, const void* W1, const void* W2,
                          const int32_t* seq_len, int32_t B, int32_t n, int32_t d_model, int32_t m,
                          float thr, int32_t rank, float scale, const ta_params* prm,
                          float* conf, uint8_t* anchor, float* anchor_B, void* stream)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    if (!h || !W1 || !W2 || !conf || !anchor || !anchor_B) return TA_ERR_NULL;
    if (B < 1 || n < 1) return TA_ERR_SHAPE;
    if (d_model < 32 || d_model > 32768 || d_model % 32 != 0) return TA_ERR_SHAPE;
    if (m != 32 && m != 64 && m != 128 && m != 256) return TA_ERR_SHAPE;
    if (h_row_stride < d_model) return TA_ERR_SHAPE;
    if (256 * h_row_stride * 2 >= 0x7FFFFFFFll) return TA_ERR_SHAPE;      // 32-bit offsets inside a tile
    if (((int64_t)B * n + 255) / 256 > 0x7FFFFFFFll) return TA_ERR_SHAPE;
    if (!isfinite(thr) || !isfinite(scale)) return TA_ERR_SHAPE;
    if (h_row_stride % 8 != 0 || !aligned16(h) || !aligned16(W1)) return TA_ERR_ALIGN;
    return hip_status(ta::launch_detect(h, h_row_stride, W1, W2, seq_len, B, n, d_model, m, thr, rank,
                                        prm->sponsor_B, scale, conf, anchor, anchor_B, (hipStream_t)stream));
}

int32_t ta_embed_anchors(const void* x, int64_t x_row_stride, const void* C, int32_t E,
                         const int32_t* seq_len, int32_t B, int32_t n, int32_t d_model, float tau,
                         float* sim, uint8_t* anchor, void* stream)
{
    if (!x || !C || !sim || !anchor) return TA_ERR_NULL;
    if (B < 1 || n < 1) return TA_ERR_SHAPE;
    if (d_model < 32 || d_model > 32768 || d_model % 32 != 0) return TA_ERR_SHAPE;
    if (E < 1 || E > 256) return TA_ERR_SHAPE;
    if (x_row_stride < d_model) return TA_ERR_SHAPE;
    if (256 * x_row_stride * 2 >= 0x7FFFFFFFll) return TA_ERR_SHAPE;      // 32-bit offsets inside a tile
    if (((int64_t)B * n + 255) / 256 > 0x7FFFFFFFll) return TA_ERR_SHAPE;
    if (!isfinite(tau)) return TA_ERR_SHAPE;
    if (x_row_stride % 8 != 0 || !aligned16(x) || !aligned16(C)) return TA_ERR_ALIGN;
    return hip_status(ta::launch_cosine(x, x_row_stride, C, E, (int64_t)B * n, d_model, seq_len, n, tau, sim, anchor,
                                        (hipStream_t)stream));
}

int32_t ta_lookup_anchors(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                          const uint8_t* vocab_anchor, int32_t V, uint8_t* anchor, void* stream)
{
    if (!tok || !vocab_anchor || !anchor) return TA_ERR_NULL;
    if (B < 1 || n < 1 || V < 1 || B > 65535) return TA_ERR_SHAPE;
    return hip_status(ta::launch_lookup(tok, seq_len, B, n, vocab_anchor, V, anchor, (hipStream_t)stream));
}

int32_t ta_expand_vouchers(const uint8_t* anchor, const float* anchor_B, const int32_t* seq_len,
                           int32_t B, int32_t n, const ta_params* prm,
                           uint8_t* spons, float* vouch, void* stream)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    if (!anchor || !spons || !vouch) return TA_ERR_NULL;
    if (B < 1 || n < 1 || B > 65535) return TA_ERR_SHAPE;
    ta::MatchTable tab;
    rc = build_table(nullptr, nullptr, 0, prm, &tab);
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_expand(anchor, anchor_B, prm->allow, seq_len, B, n, tab, spons, vouch, (hipStream_t)stream));
}

int32_t ta_score(const void* Q, const void* K, const ta_layout* lay, const int32_t* seq_len,
                 const ta_params* prm, float* A, void* ws, size_t ws_bytes, void* stream)
{
    int32_t rc = check_score(Q, K, lay, prm, A, ws, ws_bytes);
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_score(Q, K, *lay, seq_len, prm->causal, A, (float*)ws, nullptr, nullptr, nullptr,
                                       nullptr, (hipStream_t)stream));
}

int32_t ta_score_lse(const void* Q, const void* K, const ta_layout* lay, const int32_t* seq_len,
                     const ta_params* prm, const float* lse, float* A, void* stream)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    rc = check_layout(lay, true);
    if (rc != TA_OK) return rc;
    if (!Q || !K || !A || !lse) return TA_ERR_NULL;
    if (!aligned16(Q) || !aligned16(K)) return TA_ERR_ALIGN;
    if (ta::score_grid_blocks(*lay) > 0x7FFFFFFFll) return TA_ERR_SHAPE;
    return hip_status(ta::launch_score(Q, K, *lay, seq_len, prm->causal, A, nullptr, lse, nullptr, nullptr,
                                       nullptr, (hipStream_t)stream));
}

int32_t ta_select(const float* A, const uint8_t* anchor, const uint8_t* spons, const float* vouch,
                  const int32_t* seq_len, int32_t layers, int32_t batch, int32_t hkv, int32_t n,
                  int32_t K, const ta_params* prm, int32_t* idx, int32_t* cnt, void* stream)
{
    int32_t rc = check_select(A, anchor, spons, vouch, layers, batch, hkv, n, K, prm, idx, cnt);
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_select(A, anchor, spons, vouch, seq_len, layers, batch, hkv, n, K,
                                        *prm, idx, cnt, (hipStream_t)stream));
}

int32_t ta_compact(const void* Kin, const void* Vin, const int32_t* idx, const int32_t* cnt,
                   const ta_layout* lay, int32_t K, int32_t idx_shared,
                   void* Kout, void* Vout, void* stream)
{
    int32_t rc = check_compact(Kin, Vin, idx, cnt, lay, K, Kout, Vout);
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_compact(Kin, Vin, idx, cnt, *lay, K, idx_shared, Kout, Vout, nullptr,
                                         nullptr, (hipStream_t)stream));
}

namespace {

// A dense layout whose kv strides pass the shared checks; the real addressing of a paged cache is in `pg`.
int32_t check_paged(const ta_paged_kv* pg, const ta_layout* lay, ta_layout* dense, bool scoring)
{
    if (!pg || !lay) return TA_ERR_NULL;
    if (!pg->block_table) return TA_ERR_NULL;
    if (pg->page_size < 1 || pg->max_pages < 1 || pg->num_pages < 1) return TA_ERR_SHAPE;
    if (scoring && pg->page_size % 64 != 0) return TA_ERR_SHAPE;
    if ((int64_t)pg->max_pages * pg->page_size < lay->n) return TA_ERR_SHAPE;
    for (int i = 0; i < 4; ++i) {
        if (pg->stride[i] < 0) return TA_ERR_SHAPE;
        if (pg->stride[i] % 8 != 0) return TA_ERR_ALIGN;
    }
    if (pg->stride[2] < lay->d) return TA_ERR_SHAPE;
    if ((pg->stride[2] / 8) * (int64_t)pg->page_size >= 0x7FFFFFFFll) return TA_ERR_SHAPE;   // 32-bit offsets in a page
    *dense = *lay;
    dense->kv_stride[0] = dense->kv_stride[1] = dense->kv_stride[2] = 0;
    dense->kv_stride[3] = lay->d;
    return TA_OK;
}

// Copies a per-layer pointer table after checking every entry that the pass will use.
int32_t check_layer_ptrs(const ta_layer_ptrs* lp, const ta_layout* lay, bool scored, ta::LayerPtrs* out)
{
    if (lay->layers < 1 || lay->layers > TA_MAX_LAYER_PTRS) return TA_ERR_SHAPE;
    if (!lp->K || !lp->V || !lp->Kout || !lp->Vout || (scored && !lp->Q)) return TA_ERR_NULL;
    memset(out, 0, sizeof(*out));
    for (int32_t l = 0; l < lay->layers; ++l) {
        const void* q = scored ? lp->Q[l] : nullptr;
        const void *k = lp->K[l], *v = lp->V[l];
        void *ko = lp->Kout[l], *vo = lp->Vout[l];
        if (!k || !v || !ko || !vo || (scored && !q)) return TA_ERR_NULL;
        if (!aligned16(k) || !aligned16(v) || !aligned16(ko) || !aligned16(vo) || !aligned16(q)) return TA_ERR_ALIGN;
        if (ko == k || ko == v || vo == k || vo == v || ko == vo) return TA_ERR_SHAPE;
        out->Q[l] = q;
        out->K[l] = k;
        out->V[l] = v;
        out->Kout[l] = ko;
        out->Vout[l] = vo;
    }
    return TA_OK;
}

// The whole pass; `lse` != NULL selects the one-sweep score (then ws is not used).
int32_t evict_pass(const int32_t* tok, const int32_t* seq_len,
                   const int32_t* tab_ids, const int32_t* tab_len, int32_t E, const float* anchor_B,
                   const void* Q, const void* Kin, const void* Vin,
                   const ta_layout* lay, const ta_params* prm, int32_t K,
                   uint8_t* anchor, uint8_t* spons, float* vouch, float* A,
                   int32_t* idx, int32_t* cnt, void* Kout, void* Vout,
                   void* ws, size_t ws_bytes, const float* lse, const ta_paged_kv* pg, const ta_layer_ptrs* lp,
                   void* stream)
{
    // one tensor per layer: the shared checks see layer 0's addresses and no layer stride
    ta::LayerPtrs layer_ptrs;
    ta_layout lay_of_layers;
    if (lp) {
        if (!lay || !prm) return TA_ERR_NULL;
        const int32_t prc = check_layer_ptrs(lp, lay, prm->alpha != 0.0f, &layer_ptrs);
        if (prc != TA_OK) return prc;
        lay_of_layers = *lay;
        lay_of_layers.kv_stride[0] = lay_of_layers.q_stride[0] = 0;
        lay = &lay_of_layers;
        Q = layer_ptrs.Q[0];
        Kin = layer_ptrs.K[0];
        Vin = layer_ptrs.V[0];
        Kout = layer_ptrs.Kout[0];
        Vout = layer_ptrs.Vout[0];
    }
    ta_layout dense_of_paged;
    if (pg) {                                              // sizes from lay, addressing from pg
        int32_t prc = check_paged(pg, lay, &dense_of_paged, prm && prm->alpha != 0.0f);
        if (prc != TA_OK) return prc;
        lay = &dense_of_paged;
    }
    // validate every stage first: nothing runs unless all of them can
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    if (!lay) return TA_ERR_NULL;
    const bool scored = prm->alpha != 0.0f;
    rc = check_match(tok, lay->batch, lay->n, prm, anchor, spons, vouch);
    if (rc != TA_OK) return rc;
    ta::MatchTable tab;
    rc = build_table(tab_ids, tab_len, E, prm, &tab);
    if (rc != TA_OK) return rc;
    if (scored && lse) {
        rc = check_layout(lay, true);
        if (rc != TA_OK) return rc;
        if (!Q || !Kin || !A) return TA_ERR_NULL;
        if (!aligned16(Q) || !aligned16(Kin)) return TA_ERR_ALIGN;
        if (ta::score_grid_blocks(*lay) > 0x7FFFFFFFll) return TA_ERR_SHAPE;
    } else if (scored) {
        rc = check_score(Q, Kin, lay, prm, A, ws, ws_bytes);
        if (rc != TA_OK) return rc;
    }
    if (!scored && prm->layer_K) return TA_ERR_SHAPE;       // one shared retained set cannot have per-layer sizes
    const int32_t sel_layers = scored ? lay->layers : 1;
    const int32_t sel_hkv = scored ? lay->hkv : 1;
    rc = check_select(A, anchor, spons, vouch, sel_layers, lay->batch, sel_hkv, lay->n, K, prm, idx, cnt);
    if (rc != TA_OK) return rc;
    rc = check_compact(Kin, Vin, idx, cnt, lay, K, Kout, Vout);
    if (rc != TA_OK) return rc;
    // the table of per-layer addresses goes to the workspace, behind what the score step uses of it
    ta::LayerPtrs* lptr = nullptr;
    if (lp) {
        static_assert(sizeof(ta::LayerPtrs) <= TA_LAYER_WS_BYTES, "table must fit its share of the workspace");
        const size_t table_off = ((scored && !lse ? workspace_bytes(lay) : 0) + 255) & ~(size_t)255;
        if (!ws || ws_bytes < table_off + TA_LAYER_WS_BYTES) return TA_ERR_WORKSPACE;
        if (!aligned16(ws)) return TA_ERR_ALIGN;
        lptr = reinterpret_cast<ta::LayerPtrs*>(static_cast<char*>(ws) + table_off);
    }

    hipStream_t st = (hipStream_t)stream;
    if (lp) {
        rc = hip_status(ta::launch_layer_table(layer_ptrs, lptr, lay->layers, st));
        if (rc != TA_OK) return rc;
    }
    if (scored) {
        // the match rides along with the first sweep over the keys (one launch fewer in front of them)
        const ta::MatchRider rider = {tok, anchor_B, prm->allow, anchor, spons, vouch, &tab};
        rc = hip_status(ta::launch_score(Q, Kin, *lay, seq_len, prm->causal, A, (float*)ws, lse, &rider, pg, lptr, st));
        if (rc != TA_OK) return rc;
    } else {
        rc = hip_status(ta::launch_match(tok, seq_len, lay->batch, lay->n, tab, anchor_B, prm->allow, anchor, spons, vouch, st));
        if (rc != TA_OK) return rc;
    }
    rc = hip_status(ta::launch_select(A, anchor, spons, vouch, seq_len, sel_layers, lay->batch, sel_hkv,
                                      lay->n, K, *prm, idx, cnt, st));
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_compact(Kin, Vin, idx, cnt, *lay, K, scored ? 0 : 1, Kout, Vout, pg, lptr, st));
}

}  // namespace

int32_t ta_score_paged(const void* Q, const void* Kpool, const ta_paged_kv* pg, const ta_layout* lay,
                       const int32_t* seq_len, const ta_params* prm, const float* lse,
                       float* A, void* ws, size_t ws_bytes, void* stream)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    ta_layout dense;
    rc = check_paged(pg, lay, &dense, true);
    if (rc != TA_OK) return rc;
    if (lse) {
        rc = check_layout(&dense, true);
        if (rc != TA_OK) return rc;
        if (!Q || !Kpool || !A) return TA_ERR_NULL;
        if (!aligned16(Q) || !aligned16(Kpool)) return TA_ERR_ALIGN;
        if (ta::score_grid_blocks(dense) > 0x7FFFFFFFll) return TA_ERR_SHAPE;
    } else {
        rc = check_score(Q, Kpool, &dense, prm, A, ws, ws_bytes);
        if (rc != TA_OK) return rc;
    }
    return hip_status(ta::launch_score(Q, Kpool, dense, seq_len, prm->causal, A, (float*)ws, lse, nullptr, pg,
                                       nullptr, (hipStream_t)stream));
}

int32_t ta_compact_paged(const void* Kpool, const void* Vpool, const ta_paged_kv* pg,
                         const int32_t* idx, const int32_t* cnt, const ta_layout* lay, int32_t K,
                         int32_t idx_shared, void* Kout, void* Vout, void* stream)
{
    ta_layout dense;
    int32_t rc = check_paged(pg, lay, &dense, false);
    if (rc != TA_OK) return rc;
    rc = check_compact(Kpool, Vpool, idx, cnt, &dense, K, Kout, Vout);
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_compact(Kpool, Vpool, idx, cnt, dense, K, idx_shared, Kout, Vout, pg,
                                         nullptr, (hipStream_t)stream));
}

int32_t ta_compact_into_pages(const void* Kin, const void* Vin, const ta_paged_kv* src,
                              const int32_t* idx, const int32_t* cnt, const ta_layout* lay, int32_t K,
                              int32_t idx_shared, void* Kdst, void* Vdst, const ta_paged_kv* dst, void* stream)
{
    if (!dst || !lay) return TA_ERR_NULL;
    ta_layout dense = *lay;
    int32_t rc = TA_OK;
    if (src) {
        rc = check_paged(src, lay, &dense, false);
        if (rc != TA_OK) return rc;
    }
    ta_layout dst_sized = *lay;                             // the destination holds K slots per unit, not n positions
    dst_sized.n = K < 1 ? 1 : K;
    ta_layout unused;
    rc = check_paged(dst, &dst_sized, &unused, false);
    if (rc != TA_OK) return rc;
    // the shared checks of step 5; a destination pool may be the source pool (distinct pages: the caller's contract)
    rc = check_compact(Kin, Vin, idx, cnt, &dense, K, Kdst, Vdst, src != nullptr);
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_compact(Kin, Vin, idx, cnt, dense, K, idx_shared, Kdst, Vdst, src, nullptr,
                                         (hipStream_t)stream, dst));
}

int32_t ta_evict(const int32_t* tok, const int32_t* seq_len,
                 const int32_t* tab_ids, const int32_t* tab_len, int32_t E, const float* anchor_B,
                 const void* Q, const void* Kin, const void* Vin,
                 const ta_layout* lay, const ta_params* prm, int32_t K,
                 uint8_t* anchor, uint8_t* spons, float* vouch, float* A,
                 int32_t* idx, int32_t* cnt, void* Kout, void* Vout,
                 void* ws, size_t ws_bytes, void* stream)
{
    return evict_pass(tok, seq_len, tab_ids, tab_len, E, anchor_B, Q, Kin, Vin, lay, prm, K, anchor, spons, vouch, A,
                      idx, cnt, Kout, Vout, ws, ws_bytes, nullptr, nullptr, nullptr, stream);
}

int32_t ta_init(void)
{
    hipError_t e = ta::select_setup();
    if (e == hipSuccess) e = ta::decode_setup();
    if (e == hipSuccess) e = scratch_setup();
    return hip_status(e);
}

int32_t ta_evict_static(const int32_t* tok, const int32_t* seq_len,
                        const int32_t* tab_ids, const int32_t* tab_len, int32_t E, const float* anchor_B,
                        const void* Q, const void* Kin, const void* Vin,
                        const ta_layout* lay, const ta_params* prm, int32_t K,
                        uint8_t* anchor, uint8_t* spons, float* vouch, float* A,
                        int32_t* idx, int32_t* cnt, void* Kout, void* Vout, void* stream)
{
    if (!lay || !prm) return TA_ERR_NULL;
    if (ta_workspace_bytes(lay, prm) > (size_t)TA_STATIC_SCRATCH_BYTES) return TA_ERR_SCRATCH;
    hipError_t e = scratch_setup();
    int dev = 0;
    if (e == hipSuccess) e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_status(e);
    return evict_pass(tok, seq_len, tab_ids, tab_len, E, anchor_B, Q, Kin, Vin, lay, prm, K, anchor, spons, vouch, A,
                      idx, cnt, Kout, Vout, g_scratch_ptr[dev], (size_t)TA_STATIC_SCRATCH_BYTES, nullptr, nullptr, nullptr,
                      stream);
}

int32_t ta_evict_lse(const int32_t* tok, const int32_t* seq_len,
                     const int32_t* tab_ids, const int32_t* tab_len, int32_t E, const float* anchor_B,
                     const void* Q, const void* Kin, const void* Vin, const float* lse,
                     const ta_layout* lay, const ta_params* prm, int32_t K,
                     uint8_t* anchor, uint8_t* spons, float* vouch, float* A,
                     int32_t* idx, int32_t* cnt, void* Kout, void* Vout, void* stream)
{
    if (!prm || !lse) return TA_ERR_NULL;
    if (prm->alpha == 0.0f) return TA_ERR_SHAPE;            // nothing to fuse in the attention-free setting
    return evict_pass(tok, seq_len, tab_ids, tab_len, E, anchor_B, Q, Kin, Vin, lay, prm, K, anchor, spons, vouch, A,
                      idx, cnt, Kout, Vout, nullptr, 0, lse, nullptr, nullptr, stream);
}

int32_t ta_evict_paged(const int32_t* tok, const int32_t* seq_len,
                       const int32_t* tab_ids, const int32_t* tab_len, int32_t E, const float* anchor_B,
                       const void* Q, const void* Kpool, const void* Vpool, const ta_paged_kv* pg, const float* lse,
                       const ta_layout* lay, const ta_params* prm, int32_t K,
                       uint8_t* anchor, uint8_t* spons, float* vouch, float* A,
                       int32_t* idx, int32_t* cnt, void* Kout, void* Vout,
                       void* ws, size_t ws_bytes, void* stream)
{
    if (!pg) return TA_ERR_NULL;
    return evict_pass(tok, seq_len, tab_ids, tab_len, E, anchor_B, Q, Kpool, Vpool, lay, prm, K, anchor, spons, vouch, A,
                      idx, cnt, Kout, Vout, ws, ws_bytes, lse, pg, nullptr, stream);
}

int32_t ta_evict_layers(const int32_t* tok, const int32_t* seq_len,
                        const int32_t* tab_ids, const int32_t* tab_len, int32_t E, const float* anchor_B,
                        const ta_layer_ptrs* lp, const ta_layout* lay, const ta_params* prm, int32_t K,
                        uint8_t* anchor, uint8_t* spons, float* vouch, float* A,
                        int32_t* idx, int32_t* cnt, void* ws, size_t ws_bytes, void* stream)
{
    if (!lp) return TA_ERR_NULL;
    return evict_pass(tok, seq_len, tab_ids, tab_len, E, anchor_B, nullptr, nullptr, nullptr, lay, prm, K, anchor, spons,
                      vouch, A, idx, cnt, nullptr, nullptr, ws, ws_bytes, nullptr, nullptr, lp, stream);
}

int32_t ta_evict_layers_paged(const int32_t* tok, const int32_t* seq_len,
                              const int32_t* tab_ids, const int32_t* tab_len, int32_t E, const float* anchor_B,
                              const ta_layer_ptrs* lp, const ta_paged_kv* pg, const float* lse,
                              const ta_layout* lay, const ta_params* prm, int32_t K,
                              uint8_t* anchor, uint8_t* spons, float* vouch, float* A,
                              int32_t* idx, int32_t* cnt, void* ws, size_t ws_bytes, void* stream)
{
    if (!lp || !pg) return TA_ERR_NULL;
    return evict_pass(tok, seq_len, tab_ids, tab_len, E, anchor_B, nullptr, nullptr, nullptr, lay, prm, K, anchor, spons,
                      vouch, A, idx, cnt, nullptr, nullptr, ws, ws_bytes, lse, pg, lp, stream);
}

int32_t ta_decode_init(const ta_decode_state* st, const int32_t* tok, const int32_t* seq_len, int32_t n,
                       const uint8_t* anchor, const float* anchor_B, const float* A,
                       const int32_t* idx, const int32_t* cnt, const void* Kout, const void* Vout,
                       const ta_params* prm, void* stream)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    rc = check_decode_state(st);
    if (rc != TA_OK) return rc;
    if (!tok || !anchor || !idx || !cnt) return TA_ERR_NULL;
    if ((!Kout || !Vout) && !(st->pages && !Kout && !Vout)) return TA_ERR_NULL;   // both, or (paged, rows in place) neither
    if (n < 1 || n > st->cap) return TA_ERR_SHAPE;
    if (!aligned16(Kout) || !aligned16(Vout)) return TA_ERR_ALIGN;
    return hip_status(ta::launch_decode_init(*st, tok, seq_len, n, anchor, anchor_B, A, idx, cnt, Kout, Vout,
                                             prm->sponsor_B, (hipStream_t)stream));
}

int32_t ta_decode_step(const ta_decode_state* st, const int32_t* new_tok, const void* q_new,
                       const void* k_new, const void* v_new,
                       const int32_t* tab_ids, const int32_t* tab_len, int32_t E,
                       const ta_params* prm, int32_t* evicted, void* stream)
{
    int32_t rc = check_params(prm);
    if (rc != TA_OK) return rc;
    rc = check_decode_state(st);
    if (rc != TA_OK) return rc;
    if (!new_tok || !k_new || !v_new) return TA_ERR_NULL;
    if (prm->alpha != 0.0f && !q_new) return TA_ERR_NULL;
    if (!isfinite(prm->budget_decay)) return TA_ERR_SHAPE;
    if (prm->pool_k > 1 || prm->k_protected >= 0) return TA_ERR_SHAPE;   // options of the one-shot selection only
    if (!aligned16(k_new) || !aligned16(v_new) || (q_new && !aligned16(q_new))) return TA_ERR_ALIGN;
    rc = check_budget(prm, st->K);
    if (rc != TA_OK) return rc;
    ta::MatchTable tab;
    rc = build_table(tab_ids, tab_len, E, prm, &tab);
    if (rc != TA_OK) return rc;
    return hip_status(ta::launch_decode_step(*st, new_tok, q_new, k_new, v_new, tab, *prm, evicted,
                                             (hipStream_t)stream));
}

const char* ta_strerror(int32_t status)
{
    switch (status) {
        case TA_OK: return "ok";
        case TA_ERR_NULL: return "a required pointer is NULL";
        case TA_ERR_SHAPE: return "a size, stride or table entry is outside the supported range";
        case TA_ERR_BUDGET: return "budget K is below 1 or below n_sink + n_recent";
        case TA_ERR_WORKSPACE: return "workspace missing or too small";
        case TA_ERR_ALIGN: return "a pointer or stride is not aligned as the header requires";
        case TA_ERR_HIP: return "a HIP launch failed";
        case TA_ERR_SCRATCH: return "the layout needs more scratch than the static buffer of ta_evict_static holds";
        default: return "unknown status";
    }
}

int32_t ta_last_hip_error(void) { return t_last_hip_error; }

}  // extern "C"
