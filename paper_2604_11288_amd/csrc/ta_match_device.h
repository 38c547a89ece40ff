// Device side of steps 1+2 of the eviction pass (anchor n-gram match over token IDs and
// voucher / sponsor-mask expansion: Sec. 3.2; Eq. 2; Alg. 1, detection and voucher loops),
// shared by the stand-alone match kernel and by the statistics sweep of the score step, which
// can carry the match tiles as trailing workgroups of its own launch.
//
// MATCH_THREADS threads own a tile of MATCH_TILE consecutive positions of one sequence.
//   phase 0  build a 32768-bit filter of the table's last-token IDs in LDS (once per workgroup:
//            on long sequences a workgroup works through several consecutive tiles)
//   phase 1  stage the tile's tokens plus a left halo of 64 + 3 tokens in LDS
//   phase 2  anchor flag for every position of [tile - 64, tile end): one LDS
//            filter probe per position; a position that passes is compared with
//            the whole table at once, lane e holding entry e in registers; the
//            flags go to LDS as one bit per position
//   phase 3  a lane takes 4 consecutive positions: the 68 flag bits before and at
//            them are one LDS read; bit-reversed, the L bits before a position
//            list its sponsoring anchors by distance, so the voucher is a
//            fixed-order fp32 sum over the SET bits only (anchors are rare) and
//            the sponsor flag is "any bit set"; flags leave as 4-byte and
//            vouchers as 16-byte stores
#pragma once
#include "ta_internal.h"

namespace ta {

constexpr int MATCH_THREADS = 256;
constexpr int MATCH_TILE = 1024;                 // positions per workgroup (4 per lane)
constexpr int MATCH_MARGIN = 64;                 // flags are kept for this many positions before the tile (>= TA_MAX_SPAN)
constexpr int MATCH_HALO = MATCH_MARGIN + 4;     // tokens before the tile: margin + (TA_MAX_GRAM - 1), rounded up to 4
constexpr int FILTER_BITS = 32768;

struct MatchArgs {
    const int32_t* tok;
    const int32_t* seq_len;
    const float* anchor_B;
    const uint8_t* allow;                        // allowlist of positions, or null
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
    int32_t tok[MATCH_TILE + MATCH_HALO];
    uint32_t bits[(MATCH_TILE + MATCH_MARGIN) / 32 + 2];   // bit j: anchor at position tile0 - MATCH_MARGIN + j
};

static_assert(MATCH_MARGIN >= TA_MAX_SPAN && MATCH_MARGIN % 64 == 0, "flag margin");

MatchArgs make_match_args(const int32_t* tok, const int32_t* seq_len, int32_t B, int32_t n,
                          const float* anchor_B, const uint8_t* allow, uint8_t* anchor, uint8_t* spons, float* vouch);

__device__ __forceinline__ uint32_t filter_slot(int32_t t) { return (uint32_t)t & (FILTER_BITS - 1); }

constexpr int MATCH_TOK_ROUNDS = (MATCH_TILE + MATCH_HALO + MATCH_THREADS - 1) / MATCH_THREADS;

// Table entry of a lane (lane e holds entry e; the table has at most 64 entries).
struct MatchEntry {
    int32_t e0, e1, e2, e3, len;
};

// Tokens of [tile0 - HALO, tile0 + TILE) of one tile, MATCH_TOK_ROUNDS per thread, into registers;
// positions outside the sequence hold a value no table ID can equal (IDs are validated >= 0).
__device__ __forceinline__ void match_load_tokens(const MatchArgs& a, int32_t tile, int32_t b, int32_t nb, int tid,
                                                  int32_t (&tk)[MATCH_TOK_ROUNDS])
{
    const int32_t base = tile * MATCH_TILE - MATCH_HALO;
    const size_t row = (size_t)b * (size_t)a.n;
#pragma unroll
    for (int r = 0; r < MATCH_TOK_ROUNDS; ++r) {
        const int i = tid + r * MATCH_THREADS;
        const int32_t p = base + i;
        tk[r] = (i < MATCH_TILE + MATCH_HALO && p >= 0 && p < nb) ? a.tok[row + (size_t)p] : INT32_MIN;
    }
}

// Phase 0: the last-token filter of the table in LDS (the same for every tile: a workgroup that
// works on several tiles builds it once) and this lane's table entry.  Called by exactly
// MATCH_THREADS threads; the filter is complete after the next workgroup barrier.
__device__ __forceinline__ MatchEntry match_prepare(const MatchTable& tab, int tid, MatchLds& lds)
{
    for (int i = tid; i < FILTER_BITS / 32; i += MATCH_THREADS) lds.filter[i] = 0u;
    __syncthreads();
    if (tid < tab.E) {
        const uint32_t h = filter_slot(tab.rid[tid][0]);
        atomicOr(&lds.filter[h >> 5], 1u << (h & 31));
    }
    const int lane = tid & 63;
    MatchEntry e = {-1, -1, -1, -1, 0};
    if (lane < tab.E) {
        e.e0 = tab.rid[lane][0];
        e.e1 = tab.rid[lane][1];
        e.e2 = tab.rid[lane][2];
        e.e3 = tab.rid[lane][3];
        e.len = tab.len[lane];
    }
    return e;
}

// Phases 1-2 of one tile: the tokens in `tk` go to LDS, then the anchor flags of
// [tile0 - MATCH_MARGIN, tile0 + MATCH_TILE) are left as bits in lds.bits.  With `next_tile` >= 0
// the tokens of that tile are requested into `tk` as soon as the current ones are in LDS, so that
// their latency hides behind this tile's work.  Starts and ends with a workgroup barrier (the first
// also orders the previous tile's reads of lds.bits before this tile's writes).
__device__ __forceinline__ void match_flags_tile(const MatchArgs& a, const MatchEntry& e, int32_t tile, int32_t b, int32_t nb,
                                                 int tid, MatchLds& lds, int32_t (&tk)[MATCH_TOK_ROUNDS], int32_t next_tile)
{
    uint32_t* s_filter = lds.filter;
    int32_t* s_tok = lds.tok;
    uint32_t* s_bits = lds.bits;
    const int lane = tid & 63, wave = tid >> 6;
    const int32_t tile0 = tile * MATCH_TILE;
    const int32_t base = tile0 - MATCH_HALO;
    const size_t row = (size_t)b * (size_t)a.n;
#pragma unroll
    for (int r = 0; r < MATCH_TOK_ROUNDS; ++r) {
        const int i = tid + r * MATCH_THREADS;
        if (i < MATCH_TILE + MATCH_HALO) s_tok[i] = tk[r];
    }
    if (next_tile >= 0) match_load_tokens(a, next_tile, b, nb, tid, tk);
    __syncthreads();

    // phase 2: 64 positions per wavefront and round.  A position that passes the filter is compared
    // with all table entries at once, one entry per lane.
    for (int j0 = 64 * wave; j0 < MATCH_TILE + MATCH_MARGIN; j0 += MATCH_THREADS) {
        const int32_t q = tile0 - MATCH_MARGIN + j0 + lane;
        bool cand = false;
        if (q >= 0 && q < nb) {
            const uint32_t h = filter_slot(s_tok[q - base]);
            cand = ((s_filter[h >> 5] >> (h & 31)) & 1u) != 0u;
            if (cand && a.allow) cand = a.allow[row + (size_t)q] != 0;     // a match counts on allowed positions only
        }
        unsigned long long todo = __ballot(cand), m = 0ull;
        while (todo) {
            const int i = __ffsll((long long)todo) - 1;
            todo &= todo - 1ull;
            const int32_t* t = &s_tok[tile0 - MATCH_MARGIN + j0 + i - base];   // same address in every lane; t[-3] >= s_tok
            const int32_t a0 = t[0], a1 = t[-1], a2 = t[-2], a3 = t[-3];
            const bool ok = e.len >= 1 && a0 == e.e0 && (e.len < 2 || a1 == e.e1) && (e.len < 3 || a2 == e.e2) &&
                            (e.len < 4 || a3 == e.e3);
            if (__ballot(ok) != 0ull) m |= 1ull << i;
        }
        if (lane == 0) {
            s_bits[j0 / 32] = (uint32_t)m;
            s_bits[j0 / 32 + 1] = (uint32_t)(m >> 32);
        }
    }
    __syncthreads();
}

// Phase 3: vouchers and sponsor flags of the tile from the flag bits in `s_bits` (bit j: anchor
// at position tile0 - MATCH_MARGIN + j; bits of positions outside [0, seq_len) must be clear).
// The anchor flags themselves are stored too when `store_anchor` is set.
__device__ __forceinline__ void expand_tile(const MatchArgs& a, const MatchTable& tab, int32_t tile, int32_t b,
                                            int tid, const uint32_t* s_bits, bool store_anchor)
{
    const int32_t n = a.n;
    int32_t nb = a.seq_len ? a.seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);
    const int32_t tile0 = tile * MATCH_TILE;
    const int32_t L = tab.L;
    const size_t row = (size_t)b * (size_t)n;

    // phase 3: vouchers and sponsor flags, 4 consecutive positions per lane
    const int32_t p0 = tile0 + 4 * tid;
    if (p0 >= n) return;
    // flag bits of positions p0 - 64 .. p0 + 3: bit i of (f_hi:f_lo) is position p0 - 64 + i
    const int w0 = (4 * tid) >> 5, sh = (4 * tid) & 31;
    const uint32_t x0 = s_bits[w0], x1 = s_bits[w0 + 1], x2 = s_bits[w0 + 2];
    const unsigned long long lo64 = ((unsigned long long)x1 << 32) | x0;
    const unsigned long long f_lo = sh ? ((lo64 >> sh) | ((unsigned long long)x2 << (64 - sh))) : lo64;
    const uint32_t f_hi = (x2 >> sh) & 0xFu;               // positions p0 .. p0 + 3
    const unsigned long long span_mask = L >= 64 ? ~0ull : ((1ull << L) - 1ull);
    uint8_t anc4[4], sp4[4];
    float v4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        int32_t p = p0 + c;
        uint8_t an = 0, sp = 0;
        float v = 0.0f;
        if (p < nb) {
            an = (uint8_t)((f_hi >> c) & 1u);
            // bits c .. c+63 are positions p - 64 .. p - 1; reversed, bit k-1 is position p - k
            const unsigned long long win = c ? ((f_lo >> c) | ((unsigned long long)f_hi << (64 - c))) : f_lo;
            unsigned long long near = __brevll(win) & span_mask;
            sp = near != 0ull ? 1 : 0;
            while (near) {                                  // increasing distance k, as in the fixed-order sum
                const int k = __ffsll((long long)near);
                near &= near - 1ull;
                float Bi = a.anchor_B ? a.anchor_B[row + (size_t)(p - k)] : tab.B;
                v = __fadd_rn(v, __fmul_rn(Bi, tab.pw[k]));
            }
        }
        anc4[c] = an;
        sp4[c] = sp;
        v4[c] = v;
    }
    if (a.vec_ok && p0 + 3 < n) {
        uchar4 au = make_uchar4(anc4[0], anc4[1], anc4[2], anc4[3]);
        uchar4 su = make_uchar4(sp4[0], sp4[1], sp4[2], sp4[3]);
        if (store_anchor) *reinterpret_cast<uchar4*>(a.anchor + row + p0) = au;
        *reinterpret_cast<uchar4*>(a.spons + row + p0) = su;
        *reinterpret_cast<float4*>(a.vouch + row + p0) = make_float4(v4[0], v4[1], v4[2], v4[3]);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (p0 + c < n) {
                if (store_anchor) a.anchor[row + p0 + c] = anc4[c];
                a.spons[row + p0 + c] = sp4[c];
                a.vouch[row + p0 + c] = v4[c];
            }
        }
    }
}

// Steps 1+2 for `count` consecutive tiles of one sequence, starting at `tile`: flags by n-gram
// match, then the expansion.  The filter is built once; a tile's tokens are requested while the
// tile before it is worked on.
__device__ __forceinline__ void match_expand_tiles(const MatchArgs& a, const MatchTable& tab, int32_t tile, int32_t count,
                                                   int32_t b, int tid, MatchLds& lds)
{
    int32_t nb = a.seq_len ? a.seq_len[b] : a.n;
    nb = nb < 0 ? 0 : (nb > a.n ? a.n : nb);
    int32_t tk[MATCH_TOK_ROUNDS];
    match_load_tokens(a, tile, b, nb, tid, tk);            // requested before the filter is built: the latencies overlap
    const MatchEntry e = match_prepare(tab, tid, lds);
    for (int32_t t = tile; t < tile + count; ++t) {
        match_flags_tile(a, e, t, b, nb, tid, lds, tk, t + 1 < tile + count ? t + 1 : -1);
        expand_tile(a, tab, t, b, tid, lds.bits, true);
    }
}

// One tile (the form the score sweep's trailing workgroups use).
__device__ __forceinline__ void match_expand_tile(const MatchArgs& a, const MatchTable& tab, int32_t tile,
                                                  int32_t b, int tid, MatchLds& lds)
{
    match_expand_tiles(a, tab, tile, 1, b, tid, lds);
}

}  // namespace ta
