// Internal launcher interface between the C-ABI front end (ta_api.hip) and the
// kernels.  Launchers assume validated arguments and only enqueue work.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/ta.h"

namespace ta {

// Set-up that has to happen once per device before a kernel's first launch there (kernel
// attributes, symbol addresses).  `run` calls `f` with that device current until it has
// succeeded once on it: a failure is returned to the caller and tried again by the next call,
// so nothing is ever launched without its set-up.
class DeviceOnce {
public:
    template <typename F>
    hipError_t run(F&& f)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        std::lock_guard<std::mutex> guard(mu_);
        if ((done_ >> dev) & 1ull) return hipSuccess;
        e = f(dev);
        if (e == hipSuccess) done_ |= 1ull << dev;
        return e;
    }

private:
    std::mutex mu_;
    uint64_t done_ = 0;
};

// Kernel attributes of the select and decode kernels (dynamic LDS above 64 KB) for the current
// device; called by their launchers and by ta_init.
hipError_t select_setup();
hipError_t decode_setup();

// ---- match + voucher expansion -------------------------------------------
struct MatchTable {
    int32_t rid[TA_MAX_TABLE][TA_MAX_GRAM];  // n-gram reversed: rid[e][0] is its last token
    int32_t len[TA_MAX_TABLE];
    int32_t E;
    int32_t L;
    float B;
    float pw[TA_MAX_SPAN + 1];               // pw[k] = (float) rho^k
};

hipError_t launch_match(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                        const MatchTable& tab, const float* anchor_B, const uint8_t* allow,
                        uint8_t* anchor, uint8_t* spons, float* vouch, hipStream_t st);

// Step 2 alone from given anchor flags (read, not written); tab supplies L, B and the powers only.
hipError_t launch_expand(const uint8_t* anchor, const float* anchor_B, const uint8_t* allow, const int32_t* seq_len,
                         int32_t B, int32_t n, const MatchTable& tab, uint8_t* spons, float* vouch, hipStream_t st);

// ---- learned anchor detection -------------------------------------------------
// conf = sigmoid(W2 . GELU(W1 . h)) per position, anchor = conf > thr, budget B or scale * conf.
// m is one of 32, 64, 128, 256; dm a multiple of 32; h rows h_row_stride elements apart.
hipError_t launch_detect(const void* h, int64_t h_row_stride, const void* W1, const void* W2,
                         const int32_t* seq_len, int32_t batch, int32_t n, int32_t dm, int32_t m,
                         float thr, int32_t rank, float B, float scale,
                         float* conf, uint8_t* anchor, float* anchor_B, hipStream_t st);

// sim = largest cosine between a row of x and the E rows of C; anchor = sim > tau.
hipError_t launch_cosine(const void* x, int64_t x_row_stride, const void* C, int32_t E, int64_t rows, int32_t dm,
                         const int32_t* seq_len, int32_t n, float tau, float* sim, uint8_t* anchor, hipStream_t st);
// anchor[b][p] = vocab_anchor[tok[b][p]] != 0 for valid positions and IDs.
hipError_t launch_lookup(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                         const uint8_t* vocab_anchor, int32_t V, uint8_t* anchor, hipStream_t st);

// Arguments of a match that rides along with the first sweep of the score step.
struct MatchRider {
    const int32_t* tok;
    const float* anchor_B;
    const uint8_t* allow;
    uint8_t* anchor;
    uint8_t* spons;
    float* vouch;
    const MatchTable* tab;
};

// Per-layer base addresses in place of base + l * layer stride (entries past the layer count unused).
// The launchers below take such a table in DEVICE memory (written there by launch_layer_table).
struct LayerPtrs {
    const void* Q[TA_MAX_LAYER_PTRS];
    const void* K[TA_MAX_LAYER_PTRS];
    const void* V[TA_MAX_LAYER_PTRS];
    void* Kout[TA_MAX_LAYER_PTRS];
    void* Vout[TA_MAX_LAYER_PTRS];
};

// writes the first `layers` entries of each table (the kernels read no others)
hipError_t launch_layer_table(const LayerPtrs& host_table, LayerPtrs* dev_table, int32_t layers, hipStream_t st);

// ---- score ------------------------------------------------------------------
// Scratch bytes and grid size of the score step for a validated layout.
size_t score_workspace_bytes(const ta_layout& lay);
int64_t score_grid_blocks(const ta_layout& lay);
// With `rider` set, the match + voucher expansion of all sequences runs as trailing workgroups
// of the first sweep's launch (it depends on the tokens only and is needed after the score).
// With `lse` set (row log-sum-exps from a prefill attention kernel, [layers][batch][hq][W]) only the
// column-sum sweep runs and ws is not used.
// `pg` != null: K is a paged pool addressed through pg->block_table (lay.kv_stride unused).
// `lp` != null: Q and K of layer l start at lp->Q[l], lp->K[l] (Q, K and the layer strides unused).
hipError_t launch_score(const void* Q, const void* K, const ta_layout& lay, const int32_t* seq_len,
                        int causal, float* A, float* ws, const float* lse, const MatchRider* rider,
                        const ta_paged_kv* pg, const LayerPtrs* lp, hipStream_t st);

// ---- select -----------------------------------------------------------------
hipError_t launch_select(const float* A, const uint8_t* anchor, const uint8_t* spons,
                         const float* vouch, const int32_t* seq_len,
                         int32_t layers, int32_t batch, int32_t hkv, int32_t n, int32_t K,
                         const ta_params& prm, int32_t* idx, int32_t* cnt, hipStream_t st);

// ---- compact ----------------------------------------------------------------
// `lp` != null: layer l reads lp->K[l], lp->V[l] and writes lp->Kout[l], lp->Vout[l].
// `dst_pg` != null: the outputs are page pools, row r of a unit goes to slot r of its sequence's pages.
hipError_t launch_compact(const void* Kin, const void* Vin, const int32_t* idx, const int32_t* cnt,
                          const ta_layout& lay, int32_t K, int32_t idx_shared,
                          void* Kout, void* Vout, const ta_paged_kv* pg, const LayerPtrs* lp, hipStream_t st,
                          const ta_paged_kv* dst_pg = nullptr);

// ---- incremental (decode) form ------------------------------------------------
hipError_t launch_decode_init(const ta_decode_state& st, const int32_t* tok, const int32_t* seq_len, int32_t n,
                              const uint8_t* anchor, const float* anchor_B, const float* A,
                              const int32_t* idx, const int32_t* cnt, const void* Kout, const void* Vout,
                              float B, hipStream_t s);
hipError_t launch_decode_step(const ta_decode_state& st, const int32_t* new_tok, const void* q_new,
                              const void* k_new, const void* v_new, const MatchTable& tab,
                              const ta_params& prm, int32_t* evicted, hipStream_t s);

}  // namespace ta
