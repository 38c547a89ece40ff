// Device side of steps 1+2 of the eviction pass (anchor n-gram match over token IDs and
// voucher / sponsor-mask expansion: Sec. 3.2; Eq. 2; Alg. 1, detection and voucher loops),
// shared by the stand-alone match kernel and by the statistics sweep of the score step, which
// can carry the match tiles as trailing workgroups of its own launch.
//
// MATCH_THREADS threads own a tile of MATCH_TILE consecutive positions of one sequence.
//   phase 0  build a 32768-bit filter of the table's last-token IDs in LDS
//   phase 1  stage the tile's tokens plus a left halo of L + 3 tokens in LDS
//   phase 2  anchor flag for every position of [tile - L, tile end): one LDS
//            filter probe per position, full n-gram compare only on a filter hit
//            (the table itself sits in the kernel-argument segment, read through
//            the scalar cache because the entry index is wave-uniform)
//   phase 3  voucher = fixed-order fp32 sum over the L preceding positions,
//            sponsor flag = any anchor among them; 4 positions per lane so that
//            flags leave as 4-byte and vouchers as 16-byte stores
#pragma once
#include "ta_internal.h"

namespace ta {

constexpr int MATCH_THREADS = 256;
constexpr int MATCH_TILE = 1024;                 // positions per workgroup (4 per lane)
constexpr int MATCH_HALO_MAX = TA_MAX_SPAN + 4;  // roundup4(L + 3) <= 68
constexpr int FILTER_BITS = 32768;

struct MatchArgs {
    const int32_t* tok;
    const int32_t* seq_len;
    const float* anchor_B;
    uint8_t* anchor;
    uint8_t* spons;
    float* vouch;
    int32_t n;
    int32_t vec_ok;
    int32_t tiles;                               // tiles per sequence
    int32_t batch;
};

// LDS a tile needs; the caller provides it (16-byte aligned).
struct MatchLds {
    uint32_t filter[FILTER_BITS / 32];
    int32_t tok[MATCH_TILE + MATCH_HALO_MAX];
    uint8_t anc[MATCH_TILE + TA_MAX_SPAN];
};

MatchArgs make_match_args(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                          const float* anchor_B, uint8_t* anchor, uint8_t* spons, float* vouch);

__device__ __forceinline__ uint32_t filter_slot(int32_t t) { return (uint32_t)t & (FILTER_BITS - 1); }

// Called by exactly MATCH_THREADS threads (tid = 0 .. MATCH_THREADS-1) of a workgroup whose
// other wavefronts, if any, have already returned.
__device__ __forceinline__ void match_expand_tile(const MatchArgs& a, const MatchTable& tab, int32_t tile,
                                                  int32_t b, int tid, MatchLds& lds)
{
    uint32_t* s_filter = lds.filter;
    int32_t* s_tok = lds.tok;
    uint8_t* s_anc = lds.anc;
    const int32_t n = a.n;
    int32_t nb = a.seq_len ? a.seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);
    const int32_t tile0 = tile * MATCH_TILE;
    const int32_t L = tab.L;
    const int32_t halo = (L + 3 + 3) & ~3;
    const size_t row = (size_t)b * (size_t)n;

    // phase 0: last-token filter
    for (int i = tid; i < FILTER_BITS / 32; i += MATCH_THREADS) s_filter[i] = 0u;
    __syncthreads();
    if (tid < tab.E) {
        uint32_t h = filter_slot(tab.rid[tid][0]);
        atomicOr(&s_filter[h >> 5], 1u << (h & 31));
    }

    // phase 1: tokens of [tile0 - halo, tile0 + TILE); positions outside the
    // sequence hold a value no table ID can equal (IDs are validated >= 0)
    const int32_t base = tile0 - halo;
    for (int i = tid; i < MATCH_TILE + halo; i += MATCH_THREADS) {
        int32_t p = base + i;
        s_tok[i] = (p >= 0 && p < nb) ? a.tok[row + (size_t)p] : INT32_MIN;
    }
    __syncthreads();

    // phase 2: anchor flags of [tile0 - L, tile0 + TILE)
    for (int j = tid; j < MATCH_TILE + L; j += MATCH_THREADS) {
        int32_t q = tile0 - L + j;
        uint8_t hit = 0;
        if (q >= 0 && q < nb) {
            const int32_t* t = &s_tok[q - base];          // t[0] is the token at q, t[-k] at q-k
            int32_t t0 = t[0];
            uint32_t h = filter_slot(t0);
            if ((s_filter[h >> 5] >> (h & 31)) & 1u) {
                int32_t t1 = t[-1], t2 = t[-2], t3 = t[-3];   // q-3 >= base by construction
                for (int e = 0; e < tab.E; ++e) {
                    if (t0 != tab.rid[e][0]) continue;
                    int32_t len = tab.len[e];
                    bool ok = true;
                    if (len > 1) ok = ok && (t1 == tab.rid[e][1]);
                    if (len > 2) ok = ok && (t2 == tab.rid[e][2]);
                    if (len > 3) ok = ok && (t3 == tab.rid[e][3]);
                    if (ok) hit = 1;
                }
            }
        }
        s_anc[j] = hit;
    }
    __syncthreads();

    // phase 3: vouchers and sponsor flags, 4 consecutive positions per lane
    const int32_t p0 = tile0 + 4 * tid;
    if (p0 >= n) return;
    uint8_t anc4[4], sp4[4];
    float v4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        int32_t p = p0 + c;
        uint8_t an = 0, sp = 0;
        float v = 0.0f;
        if (p < nb) {
            const int j = p - tile0 + L;                   // index of p in s_anc
            an = s_anc[j];
            for (int k = 1; k <= L; ++k) {
                if (s_anc[j - k]) {
                    float Bi = a.anchor_B ? a.anchor_B[row + (size_t)(p - k)] : tab.B;
                    v = __fadd_rn(v, __fmul_rn(Bi, tab.pw[k]));
                    sp = 1;
                }
            }
        }
        anc4[c] = an;
        sp4[c] = sp;
        v4[c] = v;
    }
    if (a.vec_ok && p0 + 3 < n) {
        uchar4 au = make_uchar4(anc4[0], anc4[1], anc4[2], anc4[3]);
        uchar4 su = make_uchar4(sp4[0], sp4[1], sp4[2], sp4[3]);
        *reinterpret_cast<uchar4*>(a.anchor + row + p0) = au;
        *reinterpret_cast<uchar4*>(a.spons + row + p0) = su;
        *reinterpret_cast<float4*>(a.vouch + row + p0) = make_float4(v4[0], v4[1], v4[2], v4[3]);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (p0 + c < n) {
                a.anchor[row + p0 + c] = anc4[c];
                a.spons[row + p0 + c] = sp4[c];
                a.vouch[row + p0 + c] = v4[c];
            }
        }
    }
}

}  // namespace ta
