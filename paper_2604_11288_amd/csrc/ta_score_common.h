// Types and launch arguments of the score kernels.
#pragma once
#include "ta_internal.h"

namespace ta {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));


struct ScoreArgs {
    const uint4* Q;
    const uint4* K;
    const int32_t* seq_len;
    float* A;
    float* ws;
    const int32_t* table;              // paged K: block table [batch][max_pages], or null (dense K)
    int64_t k_spage;                   // paged K: page stride in 16-byte units
    int32_t page_size, max_pages, num_pages;
    int32_t page_shift;                // log2(page_size) when it is a power of two, else -1
    const float* lse;                  // given row log-sum-exps [layers][batch][hq][W] (natural log), or null
    int64_t q_sl, q_sb, q_sh;          // Q strides (layer, batch, head) in 16-byte units
    int64_t k_sl, k_sb, k_sh;          // K strides (layer, batch, head) in 16-byte units
    int32_t k_sp;                      // K position stride in 16-byte units (n * k_sp < 2^31)
    int32_t batch, hkv, G, W, n;
    int32_t rows, rows_pad;            // M = G*W and M rounded up to 64*RG
    int32_t chunk_keys, nchunks;
    int32_t units, units_per_xcd;      // units in total and per XCD (block -> unit mapping)
    int32_t causal;
    float scale_log2;                  // log2(e) / sqrt(d)
    // one tensor per layer: DEVICE tables of per-layer base addresses (layer l starts at Ql[l], Kl[l]
    // instead of Q + l*q_sl, K + l*k_sl), or null
    const uint4* const* Ql;
    const uint4* const* Kl;
};

__device__ __forceinline__ bf16x8 as_frag(uint4 v)
{
    union { uint4 u; bf16x8 b; } c;
    c.u = v;
    return c.b;
}

// A pointer to global memory that is the same in every lane, moved to scalar registers (a value
// loaded from device memory sits in vector registers even when its address is uniform) and marked
// as a global address (a pointer read from memory is otherwise accessed with flat instructions).
template <typename T>
__device__ __forceinline__ T* uniform_global_ptr(T* p)
{
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    typedef __attribute__((address_space(1))) T* global_ptr;
    return (T*)(global_ptr)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

}  // namespace ta
