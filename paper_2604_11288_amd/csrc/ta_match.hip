// Steps 1+2 of the eviction pass as a kernel of their own: anchor n-gram match over token
// IDs and voucher / sponsor-mask expansion (Sec. 3.2; Eq. 2; Alg. 1, detection and voucher
// loops).  One pass over the tokens, once per sequence: the result does not depend on layer
// or head.  The per-tile work is in ta_match_device.h.
#include "ta_match_device.h"

namespace ta {

namespace {

#ifndef TA_MATCH_MAX_TILES_PER_WG
#define TA_MATCH_MAX_TILES_PER_WG 16
#endif
constexpr int32_t MATCH_MAX_TILES_PER_WG = TA_MATCH_MAX_TILES_PER_WG;
constexpr int64_t MATCH_MIN_WORKGROUPS = 8192;             // 32 per compute unit before tiles are grouped

// `tpw` consecutive tiles per workgroup (the last workgroup of a sequence may have fewer)
__global__ void __launch_bounds__(MATCH_THREADS)
match_expand_kernel(MatchArgs a, MatchTable tab, int32_t tpw)
{
    __shared__ __align__(16) MatchLds lds;
    const int32_t first = (int32_t)blockIdx.x * tpw;
    const int32_t count = a.tiles - first < tpw ? a.tiles - first : tpw;
    match_expand_tiles(a, tab, first, count, (int32_t)blockIdx.y, (int)threadIdx.x, lds);
}

// Step 2 alone, for anchors that do not come from the n-gram table (learned detection,
// Sec. 5.1): the anchor flags are an input; their bytes for [tile0 - MATCH_MARGIN, tile end)
// become the bit string the expansion reads.
__global__ void __launch_bounds__(MATCH_THREADS)
expand_mask_kernel(MatchArgs a, MatchTable tab)
{
    constexpr int WORDS = (MATCH_TILE + MATCH_MARGIN) / 32 + 2;
    __shared__ uint32_t s_bits[WORDS];
    const int tid = (int)threadIdx.x;
    const int32_t tile = (int32_t)blockIdx.x, b = (int32_t)blockIdx.y;
    const int32_t n = a.n;
    int32_t nb = a.seq_len ? a.seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);
    const int32_t first = tile * MATCH_TILE - MATCH_MARGIN;
    const uint8_t* flags = a.anchor + (size_t)b * (size_t)n;
    const uint8_t* allow = a.allow ? a.allow + (size_t)b * (size_t)n : nullptr;
    if (tid < WORDS) s_bits[tid] = 0u;
    __syncthreads();
    for (int g = tid; g < (MATCH_TILE + MATCH_MARGIN) / 4; g += MATCH_THREADS) {
        const int32_t q0 = first + 4 * g;
        uint32_t nib = 0u;
        if (q0 >= 0 && q0 + 3 < nb && a.vec_ok) {
            const uchar4 f = *reinterpret_cast<const uchar4*>(flags + q0);
            nib = (f.x ? 1u : 0u) | (f.y ? 2u : 0u) | (f.z ? 4u : 0u) | (f.w ? 8u : 0u);
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int32_t q = q0 + c;
                if (q >= 0 && q < nb && flags[q]) nib |= 1u << c;
            }
        }
        if (nib && allow) {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if ((nib >> c) & 1u) nib &= ~((allow[q0 + c] ? 0u : 1u) << c);   // set bits are inside [0, nb)
        }
        if (nib) atomicOr(&s_bits[(4 * g) >> 5], nib << ((4 * g) & 31));
    }
    __syncthreads();
    expand_tile(a, tab, tile, b, tid, s_bits, false);
}

// Anchor flags by token ID (embedding-based detection evaluated once per vocabulary entry).
__global__ void __launch_bounds__(256)
lookup_kernel(const int32_t* tok, const int32_t* seq_len, int32_t n, const uint8_t* vocab_anchor, int32_t V,
              uint8_t* anchor)
{
    const int32_t b = (int32_t)blockIdx.y;
    const int32_t p = (int32_t)(blockIdx.x * 256 + threadIdx.x);
    if (p >= n) return;
    int32_t nb = seq_len ? seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);
    const size_t at = (size_t)b * (size_t)n + (size_t)p;
    uint8_t f = 0;
    if (p < nb) {
        const int32_t t = tok[at];
        if (t >= 0 && t < V) f = vocab_anchor[t] ? 1 : 0;
    }
    anchor[at] = f;
}

}  // namespace

MatchArgs make_match_args(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                          const float* anchor_B, const uint8_t* allow, uint8_t* anchor, uint8_t* spons, float* vouch)
{
    MatchArgs a;
    a.tok = tok;
    a.seq_len = seq_len;
    a.anchor_B = anchor_B;
    a.allow = allow;
    a.anchor = anchor;
    a.spons = spons;
    a.vouch = vouch;
    a.n = n;
    a.vec_ok = (n % 4 == 0) && ((uintptr_t)anchor % 4 == 0) && ((uintptr_t)spons % 4 == 0) &&
               ((uintptr_t)vouch % 16 == 0);
    a.tiles = (n + MATCH_TILE - 1) / MATCH_TILE;
    a.batch = B;
    return a;
}

hipError_t launch_match(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                        const MatchTable& tab, const float* anchor_B, const uint8_t* allow,
                        uint8_t* anchor, uint8_t* spons, float* vouch, hipStream_t st)
{
    const MatchArgs a = make_match_args(tok, seq_len, B, n, anchor_B, allow, anchor, spons, vouch);
    // Several tiles per workgroup once there are far more tiles than the chip holds workgroups: the
    // filter is then built once per workgroup instead of once per 1024 tokens.
    const int64_t total = (int64_t)a.tiles * B;
    int32_t tpw = 1;
    while (tpw < MATCH_MAX_TILES_PER_WG && total / (2 * tpw) >= MATCH_MIN_WORKGROUPS) tpw *= 2;
    dim3 grid((unsigned)((a.tiles + tpw - 1) / tpw), (unsigned)B);
    hipLaunchKernelGGL(match_expand_kernel, grid, dim3(MATCH_THREADS), 0, st, a, tab, tpw);
    return hipGetLastError();
}

hipError_t launch_expand(const uint8_t* anchor, const float* anchor_B, const uint8_t* allow, const int32_t* seq_len,
                         int32_t B, int32_t n, const MatchTable& tab, uint8_t* spons, float* vouch, hipStream_t st)
{
    const MatchArgs a = make_match_args(nullptr, seq_len, B, n, anchor_B, allow, const_cast<uint8_t*>(anchor), spons, vouch);
    dim3 grid((unsigned)a.tiles, (unsigned)B);
    hipLaunchKernelGGL(expand_mask_kernel, grid, dim3(MATCH_THREADS), 0, st, a, tab);
    return hipGetLastError();
}

hipError_t launch_lookup(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                         const uint8_t* vocab_anchor, int32_t V, uint8_t* anchor, hipStream_t st)
{
    dim3 grid((unsigned)((n + 255) / 256), (unsigned)B);
    hipLaunchKernelGGL(lookup_kernel, grid, dim3(256), 0, st, tok, seq_len, n, vocab_anchor, V, anchor);
    return hipGetLastError();
}

}  // namespace ta
