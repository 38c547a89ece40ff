// Steps 1+2 of the eviction pass as a kernel of their own: anchor n-gram match over token
// IDs and voucher / sponsor-mask expansion (Sec. 3.2; Eq. 2; Alg. 1, detection and voucher
// loops).  One pass over the tokens, once per sequence: the result does not depend on layer
// or head.  The per-tile work is in ta_match_device.h.
#include "ta_match_device.h"

namespace ta {

namespace {

__global__ void __launch_bounds__(MATCH_THREADS)
match_expand_kernel(MatchArgs a, MatchTable tab)
{
    __shared__ __align__(16) MatchLds lds;
    match_expand_tile(a, tab, (int32_t)blockIdx.x, (int32_t)blockIdx.y, (int)threadIdx.x, lds);
}

}  // namespace

MatchArgs make_match_args(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                          const float* anchor_B, uint8_t* anchor, uint8_t* spons, float* vouch)
{
    MatchArgs a;
    a.tok = tok;
    a.seq_len = seq_len;
    a.anchor_B = anchor_B;
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
                        const MatchTable& tab, const float* anchor_B,
                        uint8_t* anchor, uint8_t* spons, float* vouch, hipStream_t st)
{
    const MatchArgs a = make_match_args(tok, seq_len, B, n, anchor_B, anchor, spons, vouch);
    dim3 grid((unsigned)a.tiles, (unsigned)B);
    hipLaunchKernelGGL(match_expand_kernel, grid, dim3(MATCH_THREADS), 0, st, a, tab);
    return hipGetLastError();
}

}  // namespace ta
