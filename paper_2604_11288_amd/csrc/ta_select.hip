// Step 4 of the eviction pass: utility (Eq. 1 / Eq. 3) and protected top-K
// (Alg. 1, utility and top-K steps; Sec. 3.3; Thm. 2-4).
//
// One workgroup per unit.  The total order is (class desc, u desc, position
// desc) and the class sizes are known before any ranking: class 2 (sinks and
// recent window) is a pair of position ranges, class 1 (sponsored) is counted
// from the sponsor mask.  Hence exactly one class straddles the budget - the
// "boundary class" - and only inside it a rank threshold is needed:
//   c2 + c1 <= K : classes 2 and 1 are kept whole, R = K - c2 - c1 slots go to class 0
//   otherwise    : class 2 is kept whole, R = K - c2 slots go to class 1 (pool overflow)
// The R-th largest (u, position) key of the boundary class is found with an
// MSD radix select (8-bit digits) over order-preserving 32-bit images of u kept
// in LDS, followed - only if several positions tie with the threshold u - by a
// radix select over their positions.  The retained positions are then written
// in ascending order with a ballot/popcount stream compaction.
//
// Options around the same selection (baselines and Sec. 3.3 as settings):
//   pool_r       the scores are max-pooled over 2 pool_r + 1 positions before the utility
//                (the clustering step of SnapKV)
//   layer_K      per-layer budgets (PyramidKV); idx rows keep the common capacity K
//   k_protected  fixed partition K = K_main + K_protected (template CAPPED): the protected pool
//                takes the k_protected best sponsored tokens, everything else that is not
//                mandatory competes for the main pool by (u, position) alone - two threshold
//                searches instead of one
#include "ta_internal.h"

namespace ta {

namespace {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int HIST_COPIES = 16;               // privatised histograms, one per lane % 16
constexpr int HIST_STRIDE = 257;              // odd stride: the same bin of different copies sits in different LDS banks
constexpr int SEL_CACHE_MAX_N = 32768;        // keys cached in LDS up to this length
constexpr int SEL_MAX_ROUNDS = SEL_CACHE_MAX_N / 4 / SEL_THREADS;   // rounds of SEL_THREADS quads in the longest cached row

struct SelectArgs {
    const float* A;
    const uint8_t* anchor;
    const uint8_t* spons;
    const float* vouch;
    const int32_t* seq_len;
    const int32_t* layer_K;
    int32_t* idx;
    int32_t* cnt;
    float* margin;                  // [units][2] or null: smallest retained / largest evicted u of the class the cut falls in
    int32_t batch, hkv, n, K;
    int32_t pool_r, k_protected;
    int32_t units, units_per_xcd;
    int32_t vec_ok;
    int32_t n_sink, n_recent;
    float alpha, beta, gamma;
};

// Order-preserving map fp32 -> uint32 (larger float <=> larger integer).
__device__ __forceinline__ uint32_t ordered_bits(float u)
{
    uint32_t b = __float_as_uint(u);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

// The inverse map; the ends of the key range stand for "no such position".
__device__ __forceinline__ float margin_value(uint32_t k)
{
    if (k == 0xFFFFFFFFu) return INFINITY;                  // no retained member
    if (k == 0u) return -INFINITY;                          // no evicted member
    return __uint_as_float((k >> 31) ? (k ^ 0x80000000u) : ~k);
}

__device__ __forceinline__ int block_sum(int v, int* s_red)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    int t = 0;
    for (int w = 0; w < SEL_WAVES; ++w) t += s_red[w];
    return t;
}

struct RadixState {
    uint32_t digit;      // chosen digit
    uint32_t need;       // keys still needed inside the chosen bin
    uint32_t bin_count;  // population of the chosen bin
    uint32_t all_of_bin; // 1: the chosen bin and everything above it is exactly what is needed
};

// After a histogram pass: s_hist[copy][bin] hold the counts.  Finds the largest
// digit d with sum_{d' >= d} h[d'] >= need.  All threads get the result.
__device__ __forceinline__ RadixState radix_pick(uint32_t (*s_hist)[HIST_STRIDE], uint32_t* s_h,
                                                 RadixState* s_state, uint32_t need)
{
    const int tid = threadIdx.x;
    if (tid < 256) {
        uint32_t t = 0;
#pragma unroll
        for (int c = 0; c < HIST_COPIES; ++c) {
            t += s_hist[c][tid];
            s_hist[c][tid] = 0;
        }
        s_h[tid] = t;
    }
    __syncthreads();
    if (tid < 64) {
        // lane l owns bins 255-4l .. 252-4l (descending), scan over lanes
        uint32_t h0 = s_h[255 - 4 * tid], h1 = s_h[254 - 4 * tid];
        uint32_t h2 = s_h[253 - 4 * tid], h3 = s_h[252 - 4 * tid];
        uint32_t mine = h0 + h1 + h2 + h3;
        uint32_t incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            uint32_t up = __shfl_up(incl, o);
            if (tid >= o) incl += up;
        }
        unsigned long long m = __ballot(incl >= need);
        int first = __ffsll((long long)m) - 1;           // first lane reaching `need`
        if (tid == first) {
            uint32_t above = incl - mine;                  // keys in strictly higher bins
            uint32_t hs[4] = {h0, h1, h2, h3};
            RadixState r;
            r.digit = 0; r.need = 0; r.bin_count = 0; r.all_of_bin = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (above + hs[j] >= need) {
                    r.digit = (uint32_t)(255 - 4 * tid - j);
                    r.need = need - above;
                    r.bin_count = hs[j];
                    r.all_of_bin = (above + hs[j] == need) ? 1u : 0u;
                    break;
                }
                above += hs[j];
            }
            *s_state = r;
        }
    }
    __syncthreads();
    return *s_state;
}

// Four consecutive positions ("a quad") are one thread's unit of work: their operands arrive
// as one 16-byte load each for A and the vouchers and one 4-byte load each for the two flag
// arrays, their keys sit in one 16-byte LDS slot, and their retained members leave in order.
struct Quad {
    float A[4];
    float v[4];
    uint8_t sp[4];
    uint8_t an[4];
};

// SEL_ROUNDS: 1 - cached rows of at most 4 * SEL_THREADS positions, a thread has one quad; SEL_MAX_ROUNDS - the longer
// cached rows; 0 - rows that are not cached (any length)
template <bool CACHED, bool CAPPED, int SEL_ROUNDS>
__global__ void __launch_bounds__(SEL_THREADS)
select_kernel(SelectArgs a)
{
    static_assert(CACHED ? (SEL_ROUNDS == 1 || SEL_ROUNDS == SEL_MAX_ROUNDS) : SEL_ROUNDS == 0, "instances");
    constexpr int SEL_BATCH = SEL_ROUNDS == SEL_MAX_ROUNDS ? 2 : 1;   // quads of a thread whose loads are in flight together
    // long cached rows, one threshold search over every cached key: the histogram of the first digit is taken while
    // the keys are built, which saves a sweep over the cache (the histograms are cleared before the class count,
    // whose reduction has a barrier)
    constexpr bool FIRST_DIGIT_EARLY = CACHED && !CAPPED && SEL_ROUNDS > 1;
    extern __shared__ uint32_t s_key[];                     // [roundup4(n)] when CACHED
    __shared__ uint32_t s_hist[HIST_COPIES][HIST_STRIDE];
    __shared__ uint32_t s_h[256];
    __shared__ int s_red[SEL_WAVES];
    __shared__ RadixState s_state;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // Same block -> unit numbering as the score step (block b runs on XCD b mod 8, which
    // scored the units [x * units_per_xcd, (x+1) * units_per_xcd)): A is then read from the
    // L2 that holds it.
    const int32_t unit = (int32_t)(blockIdx.x & 7u) * a.units_per_xcd + (int32_t)(blockIdx.x >> 3);
    if (unit >= a.units) return;
    const int32_t b = (unit / a.hkv) % a.batch;
    const int32_t n = a.n;
    int32_t K = a.K;                                         // capacity of an idx row; the budget unless a layer has its own
    if (a.layer_K) {
        int32_t lo = a.n_sink + a.n_recent;                  // the mandatory tokens must fit (validated: <= a.K)
        lo = lo < 1 ? 1 : lo;
        const int32_t kl = a.layer_K[unit / (a.batch * a.hkv)];
        K = kl < lo ? lo : (kl > K ? K : kl);
    }
    int32_t nb = a.seq_len ? a.seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);
    int32_t* idx = a.idx + (size_t)unit * (size_t)a.K;

    if (nb <= K) {                                           // nothing to evict
        for (int32_t p = tid; p < nb; p += SEL_THREADS) idx[p] = p;
        if (tid == 0) {
            a.cnt[unit] = nb;
            if (a.margin) {
                a.margin[2 * (size_t)unit] = INFINITY;
                a.margin[2 * (size_t)unit + 1] = -INFINITY;
            }
        }
        return;
    }

    const float* A = a.A ? a.A + (size_t)unit * (size_t)n : nullptr;
    const size_t row = (size_t)b * (size_t)n;
    const uint8_t* anchor = a.anchor + row;
    const uint8_t* spons = a.spons + row;
    const float* vouch = a.vouch + row;

    const int32_t ns = a.n_sink < nb ? a.n_sink : nb;
    int32_t rs = nb - a.n_recent;                            // recent window = [rs, nb)
    rs = rs < ns ? ns : rs;
    const int32_t c2 = ns + (nb - rs);
    const int32_t nquads = (nb + 3) >> 2;
    const bool use_A = (a.alpha != 0.0f);
    const bool vec = a.vec_ok != 0;                          // n % 4 == 0 and aligned rows

    for (int i = tid; i < HIST_COPIES * HIST_STRIDE; i += SEL_THREADS) (&s_hist[0][0])[i] = 0;

    auto load_flags = [&](const uint8_t* src, int32_t q, uint8_t (&out)[4]) {
        if (vec) {
            const uchar4 f = *reinterpret_cast<const uchar4*>(src + 4 * q);   // 4q + 3 < n: inside the row
            out[0] = f.x; out[1] = f.y; out[2] = f.z; out[3] = f.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) out[c] = (4 * q + c < nb) ? src[4 * q + c] : (uint8_t)0;
        }
    };
    auto load_floats = [&](const float* src, int32_t q, float (&out)[4]) {
        if (vec) {
            const float4 f = *reinterpret_cast<const float4*>(src + 4 * q);
            out[0] = f.x; out[1] = f.y; out[2] = f.z; out[3] = f.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) out[c] = (4 * q + c < nb) ? src[4 * q + c] : 0.0f;
        }
    };
    // scores of a quad, max-pooled over [p - r, p + r] clipped to the sequence (r <= 4: the quad and its neighbours)
    auto load_pooled = [&](int32_t q, float (&out)[4]) {
        float w[12];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const int32_t qq = q - 1 + j;
            if (vec && qq >= 0 && 4 * qq + 3 < n) {
                const float4 f = *reinterpret_cast<const float4*>(A + 4 * qq);
                w[4 * j + 0] = f.x; w[4 * j + 1] = f.y; w[4 * j + 2] = f.z; w[4 * j + 3] = f.w;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (4 * qq + c >= nb) w[4 * j + c] = -INFINITY;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int32_t p = 4 * qq + c;
                    w[4 * j + c] = (p >= 0 && p < nb) ? A[p] : -INFINITY;
                }
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float m = w[4 + c];
#pragma unroll
            for (int d = 1; d <= 4; ++d)
                if (d <= a.pool_r) m = fmaxf(m, fmaxf(w[4 + c - d], w[4 + c + d]));
            out[c] = (4 * q + c < nb) ? m : 0.0f;
        }
    };
    auto load_rest = [&](int32_t q, Quad& x) {               // everything but the sponsor flags
        load_flags(anchor, q, x.an);
        load_floats(vouch, q, x.v);
        if (use_A && a.pool_r > 0) load_pooled(q, x.A);
        else if (use_A) load_floats(A, q, x.A);
        else {
#pragma unroll
            for (int c = 0; c < 4; ++c) x.A[c] = 0.0f;
        }
    };

    // ---- class-1 population.  A thread's quads are taken SEL_BATCH at a time, all their loads issued
    // before the first is used (a quad index past the end is clamped and its data ignored): with few units a
    // workgroup has a compute unit to itself and nothing else hides a round trip.  The first batch's other
    // operands are requested before the reduction so that their latency hides behind it.
    Quad first[SEL_BATCH];
    int local = 0;
    for (int32_t q0 = tid; q0 < nquads; q0 += SEL_BATCH * SEL_THREADS) {
        uint8_t sp[SEL_BATCH][4];
#pragma unroll
        for (int u = 0; u < SEL_BATCH; ++u) {
            const int32_t q = q0 + u * SEL_THREADS;
            load_flags(spons, q < nquads ? q : nquads - 1, sp[u]);
        }
#pragma unroll
        for (int u = 0; u < SEL_BATCH; ++u) {
            const int32_t q = q0 + u * SEL_THREADS;
            if (q0 == tid) {
#pragma unroll
                for (int c = 0; c < 4; ++c) first[u].sp[c] = sp[u][c];
            }
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int32_t p = 4 * q + c;
                local += (q < nquads && p >= ns && p < rs && sp[u][c]) ? 1 : 0;
            }
        }
    }
    if (CACHED && tid < nquads) {
#pragma unroll
        for (int u = 0; u < SEL_BATCH; ++u) {
            const int32_t q = tid + u * SEL_THREADS;
            load_rest(q < nquads ? q : nquads - 1, first[u]);
        }
    }
    const int32_t c1 = block_sum(local, s_red);

    const int bclass = (c2 + c1 <= K) ? 0 : 1;
    const int32_t R = bclass == 0 ? K - c2 - c1 : K - c2;    // slots for the boundary class
    const float nf = (float)nb;
    // fixed partition: P sponsored tokens are protected, M more slots go to the best of everything else
    int32_t P = 0;
    if (CAPPED) {
        P = a.k_protected < c1 ? a.k_protected : c1;
        P = P < K - c2 ? P : K - c2;
    }
    const int32_t M = K - c2 - P;

    // order-preserving key of position p if it belongs to the boundary class (fixed partition:
    // if it is not mandatory), else 0
    auto key_of = [&](int32_t p, float Ap, uint8_t an, uint8_t sp, float v) -> uint32_t {
        if (p < ns || p >= rs) return 0u;
        if (!CAPPED && (sp != 0) != (bclass == 1)) return 0u;
        float r = __fdiv_rn((float)(p + 1), nf);
        float t = use_A ? __fmul_rn(a.alpha, Ap) : 0.0f;
        t = __fadd_rn(t, __fmul_rn(a.beta, r));
        t = __fadd_rn(t, __fmul_rn(a.gamma, (float)an));
        t = __fadd_rn(t, v);
        uint32_t k = ordered_bits(t);
        return k == 0u ? 1u : k;
    };
    auto quad_keys = [&](int32_t q, const Quad& x, uint32_t (&k)[4]) {
#pragma unroll
        for (int c = 0; c < 4; ++c) k[c] = key_of(4 * q + c, x.A[c], x.an[c], x.sp[c], x.v[c]);
    };
    auto keys_at = [&](int32_t q, uint32_t (&k)[4]) {
        if (CACHED) {
            const uint4 kk = *reinterpret_cast<const uint4*>(&s_key[4 * q]);
            k[0] = kk.x; k[1] = kk.y; k[2] = kk.z; k[3] = kk.w;
        } else {
            Quad x;
            load_flags(spons, q, x.sp);
            load_rest(q, x);
            quad_keys(q, x, k);
        }
    };

    if (CACHED) {
        for (int32_t q0 = tid; q0 < nquads; q0 += SEL_BATCH * SEL_THREADS) {
            Quad x[SEL_BATCH];
#pragma unroll
            for (int u = 0; u < SEL_BATCH; ++u) {
                const int32_t q = q0 + u * SEL_THREADS;
                if (q0 == tid) x[u] = first[u];
                else {
                    load_flags(spons, q < nquads ? q : nquads - 1, x[u].sp);
                    load_rest(q < nquads ? q : nquads - 1, x[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < SEL_BATCH; ++u) {
                const int32_t q = q0 + u * SEL_THREADS;
                if (q < nquads) {
                    uint32_t k[4];
                    quad_keys(q, x[u], k);
                    *reinterpret_cast<uint4*>(&s_key[4 * q]) = make_uint4(k[0], k[1], k[2], k[3]);
                    if constexpr (FIRST_DIGIT_EARLY) {       // the first pass's histogram, while the keys are at hand
                        int prev = -1;
                        uint32_t run = 0;
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const int bin = k[c] != 0u ? (int)(k[c] >> 24) : -1;
                            if (bin != prev) {
                                if (prev >= 0) atomicAdd(&s_hist[lane & (HIST_COPIES - 1)][prev], run);
                                prev = bin;
                                run = 0;
                            }
                            ++run;
                        }
                        if (prev >= 0) atomicAdd(&s_hist[lane & (HIST_COPIES - 1)][prev], run);
                    }
                }
            }
        }
    }
    __syncthreads();

    // ---- threshold search ------------------------------------------------
    // Among the positions `member` admits (it gets a quad, its keys, and clears the keys of the
    // others), finds the `want`-th largest (key, position): a member is in the top `want` iff
    // key > T, or key == T and position >= Pt.
    auto find_threshold = [&](auto&& member, uint32_t want, uint32_t& T, int32_t& Pt) {
        uint32_t prefix = 0, need = want;
        bool done = false;
        for (int pass = 0; pass < 4 && !done; ++pass) {
            const int shift = 24 - 8 * pass;
            for (int32_t q = tid; q < nquads && !(FIRST_DIGIT_EARLY && pass == 0); q += SEL_THREADS) {
                uint32_t k4[4];
                keys_at(q, k4);
                member(q, k4);
                if constexpr (SEL_ROUNDS > 1) {
                    // long rows: neighbouring positions mostly share a digit (the recency term moves slowly), and
                    // equal digits in a row go into the histogram as one add
                    int prev = -1;
                    uint32_t run = 0;
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const uint32_t k = k4[c];
                        const bool in = k != 0u && (pass == 0 || (k >> (shift + 8)) == (prefix >> (shift + 8)));
                        const int bin = in ? (int)((k >> shift) & 255u) : -1;
                        if (bin != prev) {
                            if (prev >= 0) atomicAdd(&s_hist[lane & (HIST_COPIES - 1)][prev], run);
                            prev = bin;
                            run = 0;
                        }
                        ++run;
                    }
                    if (prev >= 0) atomicAdd(&s_hist[lane & (HIST_COPIES - 1)][prev], run);
                } else {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const uint32_t k = k4[c];
                        bool in = k != 0u && (pass == 0 || (k >> (shift + 8)) == (prefix >> (shift + 8)));
                        if (in) atomicAdd(&s_hist[lane & (HIST_COPIES - 1)][(k >> shift) & 255u], 1u);
                    }
                }
            }
            __syncthreads();
            RadixState r = radix_pick(s_hist, s_h, &s_state, need);
            prefix |= r.digit << shift;
            need = r.need;
            if (r.all_of_bin) {                              // keep every key >= prefix
                T = prefix - 1u;
                Pt = 0x7FFFFFFF;
                done = true;
            } else if (pass == 3) {
                T = prefix;                                  // several positions share u == T
                // the `need` highest positions among them are kept
                int bits = 32 - __clz(nb - 1);
                int ppasses = (bits + 7) / 8;
                uint32_t pprefix = 0, pneed = need;
                for (int pp = 0; pp < ppasses; ++pp) {
                    const int ps = 8 * (ppasses - 1 - pp);
                    for (int32_t q = tid; q < nquads; q += SEL_THREADS) {
                        uint32_t k4[4];
                        keys_at(q, k4);
                        member(q, k4);
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const uint32_t p = (uint32_t)(4 * q + c);
                            bool in = k4[c] == T && (pp == 0 || (p >> (ps + 8)) == (pprefix >> (ps + 8)));
                            if (in) atomicAdd(&s_hist[lane & (HIST_COPIES - 1)][(p >> ps) & 255u], 1u);
                        }
                    }
                    __syncthreads();
                    RadixState qs = radix_pick(s_hist, s_h, &s_state, pneed);
                    pprefix |= qs.digit << ps;
                    pneed = qs.need;
                }
                Pt = (int32_t)pprefix;                       // positions are unique: pneed == 1 here
                done = true;
            }
        }
    };

    uint32_t T = 0xFFFFFFFFu;     // boundary-class position p is kept iff key > T, or key == T and p >= Pt
    int32_t Pt = 0x7FFFFFFF;
    uint32_t T1 = 0xFFFFFFFFu;    // fixed partition: a sponsored position is protected iff key > T1, or key == T1 and p >= Pt1
    int32_t Pt1 = 0x7FFFFFFF;
    if (!CAPPED) {
        if (R > 0) find_threshold([](int32_t, uint32_t (&)[4]) {}, (uint32_t)R, T, Pt);
    } else {
        if (P == c1) {                                       // every sponsored token is protected
            T1 = 0u;
            Pt1 = 0;
        } else if (P > 0) {
            find_threshold([&](int32_t q, uint32_t (&k4)[4]) {
                uint8_t sp[4];
                load_flags(spons, q, sp);
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (!sp[c]) k4[c] = 0u;
            }, (uint32_t)P, T1, Pt1);
        }
        if (M > 0) {                                         // more candidates than M remain: nb > K
            find_threshold([&](int32_t q, uint32_t (&k4)[4]) {
                uint8_t sp[4];
                load_flags(spons, q, sp);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int32_t p = 4 * q + c;
                    if (sp[c] && (k4[c] > T1 || (k4[c] == T1 && p >= Pt1))) k4[c] = 0u;   // protected: not a candidate
                }
            }, (uint32_t)M, T, Pt);
        }
    }

    // ---- which positions of a quad are retained (bit c: position 4q + c) --------------------------
    uint32_t kept_min = 0xFFFFFFFFu, gone_max = 0u;          // keys at the cut, over this thread's candidates
    const auto keep_of = [&](int32_t q) -> uint32_t {
        uint32_t keep = 0;
        uint8_t sp[4] = {0, 0, 0, 0};
        uint32_t k4[4] = {0u, 0u, 0u, 0u};
        if (CACHED && !CAPPED) {
            // no load: a key of 0 between the mandatory ranges is a position of the other class, which is
            // sponsored exactly when the cut falls among the plain ones
            keys_at(q, k4);
#pragma unroll
            for (int c = 0; c < 4; ++c) sp[c] = (uint8_t)((k4[c] == 0u) == (bclass == 0) ? 1 : 0);
        } else {
            load_flags(spons, q, sp);
            bool need_keys = false;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int32_t p = 4 * q + c;
                need_keys = need_keys || (p >= ns && p < rs && (CAPPED || (sp[c] != 0) == (bclass == 1)));
            }
            if (need_keys) keys_at(q, k4);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int32_t p = 4 * q + c;
            bool kp = false;
            bool ranked = false;                             // competes for the slots the cut divides
            if (p < nb) {
                if (p < ns || p >= rs) kp = true;
                else if (CAPPED) {
                    const bool prot = sp[c] && (k4[c] > T1 || (k4[c] == T1 && p >= Pt1));   // protected pool
                    kp = prot || (k4[c] > T) || (k4[c] == T && p >= Pt);                  // main pool
                    ranked = !prot;
                } else if ((sp[c] != 0) != (bclass == 1)) kp = sp[c] != 0;   // class 1 above the boundary class, class 0 below it
                else {
                    kp = (k4[c] > T) || (k4[c] == T && p >= Pt);
                    ranked = true;
                }
            }
            if (ranked && kp) kept_min = k4[c] < kept_min ? k4[c] : kept_min;
            if (ranked && !kp) gone_max = k4[c] > gone_max ? k4[c] : gone_max;
            keep |= kp ? (1u << c) : 0u;
        }
        return keep;
    };

    // ---- ascending write-out -------------------------------------------------------------------
    int32_t base = 0;
    if constexpr (CACHED && SEL_ROUNDS > 1) {
        // Every round of SEL_THREADS quads at once (at most SEL_ROUNDS of them fit the key cache): a thread keeps
        // the masks of its quads in one register, the rounds' counts are scanned two to a register, and ONE
        // scan over the (round, wavefront) totals gives every wavefront its offsets - three barriers instead of
        // two per round.
        uint32_t masks = 0;
#pragma unroll
        for (int r = 0; r < SEL_ROUNDS; ++r) {
            const int32_t q = r * SEL_THREADS + tid;
            if (q < nquads) masks |= keep_of(q) << (4 * r);
        }
        uint32_t incl2[SEL_ROUNDS / 2];                      // inclusive counts within the wavefront, rounds 2j and 2j + 1
#pragma unroll
        for (int j = 0; j < SEL_ROUNDS / 2; ++j) {
            uint32_t v = (uint32_t)__popc((masks >> (8 * j)) & 15u) | ((uint32_t)__popc((masks >> (8 * j + 4)) & 15u) << 16);
            if (2 * j * SEL_THREADS < nquads) {              // uniform: rounds past the row's end hold nothing
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t up = __shfl_up(v, o);
                    if (lane >= o) v += up;                  // at most 256 per field: no carry between the halves
                }
            }
            incl2[j] = v;
        }
        __syncthreads();                                     // s_h is free (the threshold search is over)
        if (lane == 63) {
#pragma unroll
            for (int r = 0; r < SEL_ROUNDS; ++r) s_h[r * SEL_WAVES + wave] = (incl2[r >> 1] >> (16 * (r & 1))) & 0xFFFFu;
        }
        __syncthreads();
        if (tid < 64) {                                      // exclusive scan of the SEL_ROUNDS * SEL_WAVES totals, two per lane
            static_assert(SEL_ROUNDS * SEL_WAVES == 128, "two entries per lane of one wavefront");
            const uint32_t t0 = s_h[2 * tid], t1 = s_h[2 * tid + 1];
            uint32_t v = t0 + t1;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t up = __shfl_up(v, o);
                if (tid >= o) v += up;
            }
            s_h[2 * tid] = v - t0 - t1;
            s_h[2 * tid + 1] = v - t1;
            if (tid == 63) s_h[SEL_ROUNDS * SEL_WAVES] = v;  // everything retained
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < SEL_ROUNDS; ++r) {
            const uint32_t keep = (masks >> (4 * r)) & 15u;
            const int32_t q = r * SEL_THREADS + tid;
            const uint32_t incl = (incl2[r >> 1] >> (16 * (r & 1))) & 0xFFFFu;
            int32_t slot = (int32_t)(s_h[r * SEL_WAVES + wave] + incl) - __popc(keep);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (keep & (1u << c)) {
                    if (slot < K) idx[slot] = 4 * q + c;
                    ++slot;
                }
            }
        }
        base = (int32_t)s_h[SEL_ROUNDS * SEL_WAVES];
    } else {
        // one scan over per-quad counts per round of 4096 positions
        for (int32_t q0 = 0; q0 < nquads; q0 += SEL_THREADS) {
            const int32_t q = q0 + tid;
            const uint32_t keep = q < nquads ? keep_of(q) : 0u;
            const int mine = __popc(keep);
            int incl = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                int up = __shfl_up(incl, o);
                if (lane >= o) incl += up;
            }
            __syncthreads();
            if (lane == 63) s_red[wave] = incl;
            __syncthreads();
            int woff = 0, total = 0;
            for (int w = 0; w < SEL_WAVES; ++w) {
                int c = s_red[w];
                woff += (w < wave) ? c : 0;
                total += c;
            }
            int32_t slot = base + woff + incl - mine;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (keep & (1u << c)) {
                    if (slot < K) idx[slot] = 4 * q + c;
                    ++slot;
                }
            }
            base += total;
        }
    }
    if (tid == 0) a.cnt[unit] = base < K ? base : K;
    if (a.margin) {                                          // uniform
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const uint32_t lo = __shfl_xor(kept_min, o), hi = __shfl_xor(gone_max, o);
            kept_min = lo < kept_min ? lo : kept_min;
            gone_max = hi > gone_max ? hi : gone_max;
        }
        __syncthreads();
        if (lane == 0) {
            s_h[wave] = kept_min;
            s_h[SEL_WAVES + wave] = gone_max;
        }
        __syncthreads();
        if (tid == 0) {
            for (int w = 0; w < SEL_WAVES; ++w) {
                kept_min = s_h[w] < kept_min ? s_h[w] : kept_min;
                gone_max = s_h[SEL_WAVES + w] > gone_max ? s_h[SEL_WAVES + w] : gone_max;
            }
            a.margin[2 * (size_t)unit] = margin_value(kept_min);
            a.margin[2 * (size_t)unit + 1] = margin_value(gone_max);
        }
    }
}


// ---- streaming form: every input is read once, whatever the length ----------------------------
// One workgroup of four wavefronts per unit walks the sequence from its end in segments and keeps
// the best candidates of the boundary class seen so far in LDS as (key, position) pairs.  A
// position joins the list if it beats the current threshold - the R-th largest (key, position) at
// the last shrink, nothing before the first - and the list is cut back to its R best whenever the
// next segment might not fit (an MSD radix select over the LDS list, the same search as above).
// Walking from the end meets the recent positions first, whose recency term is largest: with a
// non-negative beta the threshold is high after the first shrink and few later positions pass it.
// The order of the walk and of the list only affect the time, never the result: the retained set
// is defined by the total order, and the output is written in ascending position order from a
// bitmap of the sequence (bits of the mandatory positions, of the sponsored ones when they are
// all kept, and of the final R candidates).
constexpr int SS_THREADS = 256;
constexpr int SS_WAVES = SS_THREADS / 64;
#ifndef TA_SELECT_STREAM_QPT
#define TA_SELECT_STREAM_QPT 1
#endif
#ifndef TA_SELECT_STREAM_SLACK
#define TA_SELECT_STREAM_SLACK 256
#endif
constexpr int SS_QPT = TA_SELECT_STREAM_QPT;               // quads per thread and segment
constexpr int SS_SLACK = TA_SELECT_STREAM_SLACK;           // list entries beyond R + one segment: new entries between two cuts
constexpr int SS_SEG_QUADS = SS_THREADS * SS_QPT;
constexpr int SS_SEG = SS_SEG_QUADS * 4;                   // positions per segment
#ifndef TA_SELECT_STREAM_DEPTH
#define TA_SELECT_STREAM_DEPTH 2
#endif
constexpr int SS_DEPTH = TA_SELECT_STREAM_DEPTH;           // segments whose operands are in flight
constexpr int SS_HIST_COPIES = 4;
constexpr int SS_MAX_PER_THREAD = 24;                      // list entries a thread holds while the list is compacted
constexpr int SS_FEW_PER_THREAD = 10;                      // ... in the instance for short lists (budgets up to about 1300)
constexpr int SS_MAX_CAP = SS_THREADS * SS_MAX_PER_THREAD;
constexpr int SS_MAX_LDS = 144 * 1024;                     // dynamic LDS of a workgroup (list + bitmap)
// Which form runs: the streaming form whenever the keys of a row do not fit the LDS cache of the
// kernel above, and for shorter rows when there are enough units to fill the chip several times
// (its workgroups are small and many fit a compute unit; measured on 16 384 ragged units of up to
// 16 384 positions: 560 us against 1270).  With few units the latency of one workgroup counts, and
// the cached kernel's is half as long (13 us against 25 for 256 units of 4096 positions).
#ifndef TA_SELECT_STREAM_MIN_UNITS
#define TA_SELECT_STREAM_MIN_UNITS 2048
#endif
constexpr int64_t SS_MIN_UNITS = TA_SELECT_STREAM_MIN_UNITS;

struct StreamLds {
    uint32_t hist[SS_HIST_COPIES][HIST_STRIDE];
    uint32_t h[256];
    int red[SS_WAVES];
    RadixState state;
    uint32_t count;                                        // entries in the candidate list
};

// The same search as radix_pick, for a workgroup of SS_THREADS threads and SS_HIST_COPIES histograms.
__device__ __forceinline__ RadixState stream_pick(StreamLds& L, uint32_t need)
{
    const int tid = threadIdx.x;
    {
        uint32_t t = 0;
#pragma unroll
        for (int c = 0; c < SS_HIST_COPIES; ++c) {
            t += L.hist[c][tid];
            L.hist[c][tid] = 0;
        }
        L.h[tid] = t;
    }
    __syncthreads();
    if (tid < 64) {
        const uint32_t h0 = L.h[255 - 4 * tid], h1 = L.h[254 - 4 * tid];
        const uint32_t h2 = L.h[253 - 4 * tid], h3 = L.h[252 - 4 * tid];
        const uint32_t mine = h0 + h1 + h2 + h3;
        uint32_t incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o);
            if (tid >= o) incl += up;
        }
        const unsigned long long m = __ballot(incl >= need);
        const int first = __ffsll((long long)m) - 1;
        if (tid == first) {
            uint32_t above = incl - mine;
            const uint32_t hs[4] = {h0, h1, h2, h3};
            RadixState r;
            r.digit = 0; r.need = 0; r.bin_count = 0; r.all_of_bin = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (above + hs[j] >= need) {
                    r.digit = (uint32_t)(255 - 4 * tid - j);
                    r.need = need - above;
                    r.bin_count = hs[j];
                    r.all_of_bin = (above + hs[j] == need) ? 1u : 0u;
                    break;
                }
                above += hs[j];
            }
            L.state = r;
        }
    }
    __syncthreads();
    return L.state;
}

// MARGIN: the keys turned away are tracked for the margin output (instances of their own: the default
// ones keep their registers)
template <int PER_THREAD, bool MARGIN>                     // cap <= SS_THREADS * PER_THREAD
__device__ __forceinline__ void select_stream(const SelectArgs& a, const int32_t cap)
{
    extern __shared__ uint32_t s_dyn[];                    // [cap] keys, [cap] positions, [ceil(n / 32)] bitmap
    __shared__ StreamLds L;
    uint32_t* ckey = s_dyn;
    uint32_t* cpos = s_dyn + cap;
    uint32_t* bitmap = s_dyn + 2 * cap;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int32_t unit = (int32_t)(blockIdx.x & 7u) * a.units_per_xcd + (int32_t)(blockIdx.x >> 3);
    if (unit >= a.units) return;
    const int32_t b = (unit / a.hkv) % a.batch;
    const int32_t n = a.n;
    int32_t K = a.K;
    if (a.layer_K) {
        int32_t lo = a.n_sink + a.n_recent;
        lo = lo < 1 ? 1 : lo;
        const int32_t kl = a.layer_K[unit / (a.batch * a.hkv)];
        K = kl < lo ? lo : (kl > K ? K : kl);
    }
    int32_t nb = a.seq_len ? a.seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);
    int32_t* idx = a.idx + (size_t)unit * (size_t)a.K;
    if (nb <= K) {                                         // nothing to evict
        for (int32_t p = tid; p < nb; p += SS_THREADS) idx[p] = p;
        if (tid == 0) {
            a.cnt[unit] = nb;
            if (a.margin) {
                a.margin[2 * (size_t)unit] = INFINITY;
                a.margin[2 * (size_t)unit + 1] = -INFINITY;
            }
        }
        return;
    }

    const float* A = a.A ? a.A + (size_t)unit * (size_t)n : nullptr;
    const size_t row = (size_t)b * (size_t)n;
    const uint8_t* anchor = a.anchor + row;
    const uint8_t* spons = a.spons + row;
    const float* vouch = a.vouch + row;
    const int32_t ns = a.n_sink < nb ? a.n_sink : nb;
    int32_t rs = nb - a.n_recent;
    rs = rs < ns ? ns : rs;
    const int32_t c2 = ns + (nb - rs);
    const int32_t nquads = (nb + 3) >> 2;                  // rows are padded to whole quads (n % 4 == 0)
    const bool use_A = (a.alpha != 0.0f);
    const int32_t words = (nb + 31) >> 5;

    struct Loaded {
        float4 A, v;
        uint32_t sp, an;
    };
    // unconditional loads (the quad index is clamped into the row, the caller masks what lies outside):
    // straight-line loads let the compiler wait for exactly the segment it needs
    const float* A_src = use_A ? A : vouch;                // no attention term: any readable row, the values are not used
    const auto load_quad = [&](int32_t q, Loaded& x) {
        q = q < 0 ? 0 : (q >= nquads ? nquads - 1 : q);
        x.sp = *reinterpret_cast<const uint32_t*>(spons + 4 * q);
        x.an = *reinterpret_cast<const uint32_t*>(anchor + 4 * q);
        x.v = *reinterpret_cast<const float4*>(vouch + 4 * q);
        x.A = *reinterpret_cast<const float4*>(A_src + 4 * q);
    };

    // the first segments' operands are requested before anything else: they travel while the sponsored
    // positions are counted
    const int32_t nseg = (nquads + SS_SEG_QUADS - 1) / SS_SEG_QUADS;
    Loaded ring[SS_DEPTH][SS_QPT];
#pragma unroll
    for (int d = 0; d < SS_DEPTH; ++d)
#pragma unroll
        for (int j = 0; j < SS_QPT; ++j) load_quad((nseg - 1 - d) * SS_SEG_QUADS + j * SS_THREADS + tid, ring[d][j]);


    for (int i = tid; i < SS_HIST_COPIES * HIST_STRIDE; i += SS_THREADS) (&L.hist[0][0])[i] = 0;
    for (int32_t i = tid; i < words; i += SS_THREADS) bitmap[i] = 0u;
    if (tid == 0) L.count = 0u;

    // ---- sponsored positions outside the mandatory ranges (16 flags per load) -------------------
    int local = 0;
    {
        const int32_t n16 = ((uintptr_t)spons & 15u) == 0 ? nb >> 4 : 0;     // (a row that is not 16-byte aligned: byte by byte)
        const uint4* sp16 = reinterpret_cast<const uint4*>(spons);
        for (int32_t i = tid; i < n16; i += SS_THREADS) {
            const uint4 f = sp16[i];
            const uint32_t w4[4] = {f.x, f.y, f.z, f.w};
            const int32_t p0 = 16 * i;
            if (p0 >= ns && p0 + 15 < rs) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // a flag byte is 0 or not: count the non-zero bytes of the word
                    const uint32_t x = w4[j];
                    const uint32_t nz = ((x | (x >> 1) | (x >> 2) | (x >> 3) | (x >> 4) | (x >> 5) | (x >> 6) | (x >> 7)) & 0x01010101u);
                    local += __popc(nz);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int32_t p = p0 + j;
                    const uint32_t byte = (w4[j >> 2] >> (8 * (j & 3))) & 0xFFu;
                    local += (p >= ns && p < rs && byte) ? 1 : 0;
                }
            }
        }
        for (int32_t p = 16 * n16 + tid; p < nb; p += SS_THREADS) local += (p >= ns && p < rs && spons[p]) ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) local += __shfl_xor(local, o);
    if (lane == 0) L.red[wave] = local;
    __syncthreads();                                       // also: histograms, bitmap and count are cleared
    int32_t c1 = 0;
#pragma unroll
    for (int w = 0; w < SS_WAVES; ++w) c1 += L.red[w];

    const int bclass = (c2 + c1 <= K) ? 0 : 1;
    const int32_t R = bclass == 0 ? K - c2 - c1 : K - c2;  // slots of the boundary class (more members than that exist)
    const float nf = (float)nb;

    auto key_of = [&](int32_t p, float Ap, uint32_t an, float v) -> uint32_t {
        float r = __fdiv_rn((float)(p + 1), nf);
        float t = use_A ? __fmul_rn(a.alpha, Ap) : 0.0f;
        t = __fadd_rn(t, __fmul_rn(a.beta, r));
        t = __fadd_rn(t, __fmul_rn(a.gamma, an ? 1.0f : 0.0f));
        t = __fadd_rn(t, v);
        const uint32_t k = ordered_bits(t);
        return k == 0u ? 1u : k;
    };

    // ---- the list is cut back to its R best entries; returns their threshold -----------------------
    uint32_t T = 0u;              // a position joins the list iff key > T, or key == T and p >= Pt
    int32_t Pt = 0x7FFFFFFF;
    uint32_t gone_max = 0u;       // largest key this thread has turned away from the list or cut out of it
    const auto shrink = [&](const uint32_t m) {            // m: entries in the list (the same value in every thread)
        uint32_t prefix = 0, need = (uint32_t)R;
        uint32_t Tn = 0u;
        int32_t Pn = 0x7FFFFFFF;
        bool done = false;
        for (int pass = 0; pass < 4 && !done; ++pass) {
            const int shift = 24 - 8 * pass;
            for (uint32_t e = tid; e < m; e += SS_THREADS) {
                const uint32_t k = ckey[e];
                const bool in = pass == 0 || (k >> (shift + 8)) == (prefix >> (shift + 8));
                if (in) atomicAdd(&L.hist[lane & (SS_HIST_COPIES - 1)][(k >> shift) & 255u], 1u);
            }
            __syncthreads();
            const RadixState r = stream_pick(L, need);
            prefix |= r.digit << shift;
            need = r.need;
            if (r.all_of_bin) {
                Tn = prefix - 1u;
                Pn = 0x7FFFFFFF;
                done = true;
            } else if (pass == 3) {
                Tn = prefix;
                const int bits = 32 - __clz(nb - 1);
                const int ppasses = (bits + 7) / 8;
                uint32_t pprefix = 0, pneed = need;
                for (int pp = 0; pp < ppasses; ++pp) {
                    const int ps = 8 * (ppasses - 1 - pp);
                    for (uint32_t e = tid; e < m; e += SS_THREADS) {
                        const uint32_t p = cpos[e];
                        const bool in = ckey[e] == Tn && (pp == 0 || (p >> (ps + 8)) == (pprefix >> (ps + 8)));
                        if (in) atomicAdd(&L.hist[lane & (SS_HIST_COPIES - 1)][(p >> ps) & 255u], 1u);
                    }
                    __syncthreads();
                    const RadixState qs = stream_pick(L, pneed);
                    pprefix |= qs.digit << ps;
                    pneed = qs.need;
                }
                Pn = (int32_t)pprefix;
                done = true;
            }
        }
        // compaction in place: every thread takes its entries into registers, then the kept ones
        // are appended from slot 0 (exactly R of them; their order in the list does not matter)
        uint32_t mk[PER_THREAD], mp[PER_THREAD];
#pragma unroll
        for (int j = 0; j < PER_THREAD; ++j) {
            const uint32_t e = (uint32_t)tid + (uint32_t)j * SS_THREADS;
            mk[j] = e < m ? ckey[e] : 0u;
            mp[j] = e < m ? cpos[e] : 0u;
        }
        if (tid == 0) L.count = 0u;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < PER_THREAD; ++j) {
            if ((uint32_t)j * SS_THREADS >= m) continue;   // uniform: nothing of the list lies this far
            const bool keep = mk[j] > Tn || (mk[j] == Tn && mk[j] != 0u && (int32_t)mp[j] >= Pn);
            if (MARGIN && !keep) gone_max = mk[j] > gone_max ? mk[j] : gone_max;   // (0 beyond the list's end)
            const unsigned long long bal = __ballot(keep);
            uint32_t base = 0;
            if (lane == 0 && bal) base = atomicAdd(&L.count, (uint32_t)__popcll(bal));
            base = __shfl(base, 0);
            if (keep) {
                const uint32_t slot = base + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
                if (slot < (uint32_t)cap) {
                    ckey[slot] = mk[j];
                    cpos[slot] = mp[j];
                }
            }
        }
        __syncthreads();
        T = Tn;
        Pt = Pn;
    };

    // ---- the walk, from the last segment to the first; the operands of SS_DEPTH segments are in flight
    // (a segment is worked on in about a microsecond, a round trip under load takes several)
    for (int32_t top = nseg - 1; top >= 0; top -= SS_DEPTH) {
#pragma unroll
        for (int d = 0; d < SS_DEPTH; ++d) {
            const int32_t sg = top - d;
            uint32_t keys[SS_QPT][4];
            bool join[SS_QPT][4];
            uint32_t always[SS_QPT];                       // bits of a quad that are retained whatever the ranking says
#pragma unroll
            for (int j = 0; j < SS_QPT; ++j) {
                const Loaded& x = ring[d][j];
                const int32_t q = sg * SS_SEG_QUADS + j * SS_THREADS + tid;
                const float Aq[4] = {x.A.x, x.A.y, x.A.z, x.A.w};
                const float vq[4] = {x.v.x, x.v.y, x.v.z, x.v.w};
                always[j] = 0u;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int32_t p = 4 * q + c;
                    const uint32_t sp = (x.sp >> (8 * c)) & 0xFFu, an = (x.an >> (8 * c)) & 0xFFu;
                    keys[j][c] = 0u;
                    join[j][c] = false;
                    if (sg >= 0 && p < nb && q < nquads) {
                        if (p < ns || p >= rs) always[j] |= 1u << c;
                        else if ((sp != 0u) != (bclass == 1)) always[j] |= (sp != 0u) ? (1u << c) : 0u;   // class 1 above the boundary class, class 0 below it
                        else if (MARGIN || R > 0) {
                            keys[j][c] = key_of(p, Aq[c], an, vq[c]);
                            join[j][c] = R > 0 && (keys[j][c] > T || (keys[j][c] == T && p >= Pt));
                            if (MARGIN && !join[j][c]) gone_max = keys[j][c] > gone_max ? keys[j][c] : gone_max;
                        }
                    }
                }
            }
            // the segment SS_DEPTH further on takes over the registers (past the first segment: a clamped
            // address whose data nobody uses)
#pragma unroll
            for (int j = 0; j < SS_QPT; ++j) load_quad((sg - SS_DEPTH) * SS_SEG_QUADS + j * SS_THREADS + tid, ring[d][j]);
            if (sg >= 0) {                                 // uniform
#pragma unroll
                for (int j = 0; j < SS_QPT; ++j) {
                    const int32_t q = sg * SS_SEG_QUADS + j * SS_THREADS + tid;
                    if (always[j]) atomicOr(&bitmap[(4 * q) >> 5], always[j] << ((4 * q) & 31));
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const unsigned long long bal = __ballot(join[j][c]);
                        if (bal) {                         // uniform
                            uint32_t base = 0;
                            if (lane == 0) base = atomicAdd(&L.count, (uint32_t)__popcll(bal));
                            base = __shfl(base, 0);
                            if (join[j][c]) {
                                const uint32_t slot = base + (uint32_t)__popcll(bal & ((1ull << lane) - 1ull));
                                if (slot < (uint32_t)cap) {    // holds by construction: the list is cut back before it could overflow
                                    ckey[slot] = keys[j][c];
                                    cpos[slot] = (uint32_t)(4 * q + c);
                                }
                            }
                        }
                    }
                }
                __syncthreads();                           // the segment's entries are in the list
                const uint32_t m = L.count;
                __syncthreads();                           // every thread has read the count before anyone adds to it again
                // Cut back when the next segment might not fit, at the end (to exactly R), and once early: the
                // first cut gives the threshold that keeps most later positions out of the list.
                const bool early = T == 0u && m >= 2u * (uint32_t)R && m >= 512u;
                if (R > 0 && ((sg > 0 && (m + (uint32_t)SS_SEG > (uint32_t)cap || early)) || (sg == 0 && m > (uint32_t)R))) shrink(m);
            }
        }
    }

    // ---- the final candidates join the bitmap; ascending write-out from it --------------------------
    {
        const uint32_t m = L.count;                        // == R (or 0)
        for (uint32_t e = tid; e < m; e += SS_THREADS) {
            const uint32_t p = cpos[e];
            atomicOr(&bitmap[p >> 5], 1u << (p & 31u));
        }
    }
    __syncthreads();
    const int32_t wpt = (words + SS_THREADS - 1) / SS_THREADS;            // consecutive words per thread
    const int32_t w0 = tid * wpt;
    int mine = 0;
    for (int32_t w = w0; w < w0 + wpt && w < words; ++w) mine += __popc(bitmap[w]);
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    if (lane == 63) L.red[wave] = incl;
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int w = 0; w < SS_WAVES; ++w) {
        const int c = L.red[w];
        woff += (w < wave) ? c : 0;
        total += c;
    }
    int32_t slot = woff + incl - mine;
    for (int32_t w = w0; w < w0 + wpt && w < words; ++w) {
        uint32_t bits = bitmap[w];
        while (bits) {
            const int bit = __ffs((int)bits) - 1;
            bits &= bits - 1u;
            if (slot < K) idx[slot] = 32 * w + bit;
            ++slot;
        }
    }
    if (tid == 0) a.cnt[unit] = total < K ? total : K;
    if (MARGIN) {
        uint32_t kept_min = 0xFFFFFFFFu;
        const uint32_t m = L.count;
        for (uint32_t e = tid; e < m; e += SS_THREADS) kept_min = ckey[e] < kept_min ? ckey[e] : kept_min;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const uint32_t lo = __shfl_xor(kept_min, o), hi = __shfl_xor(gone_max, o);
            kept_min = lo < kept_min ? lo : kept_min;
            gone_max = hi > gone_max ? hi : gone_max;
        }
        __syncthreads();                                   // the scan's partial sums have been read
        if (lane == 0) {
            L.h[wave] = kept_min;
            L.h[SS_WAVES + wave] = gone_max;
        }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 0; w < SS_WAVES; ++w) {
                kept_min = L.h[w] < kept_min ? L.h[w] : kept_min;
                gone_max = L.h[SS_WAVES + w] > gone_max ? L.h[SS_WAVES + w] : gone_max;
            }
            a.margin[2 * (size_t)unit] = margin_value(kept_min);
            a.margin[2 * (size_t)unit + 1] = margin_value(gone_max);
        }
    }
}

// Short candidate lists (budgets up to about 1300): six wavefronts per SIMD, which the many short units
// of a ragged batch need to hide their round trips (two registers go to scratch for it).  Long lists keep
// the registers.
__global__ void __launch_bounds__(SS_THREADS) __attribute__((amdgpu_waves_per_eu(6)))
select_stream_few_kernel(SelectArgs a, int32_t cap)
{
    select_stream<SS_FEW_PER_THREAD, false>(a, cap);
}

__global__ void __launch_bounds__(SS_THREADS) __attribute__((amdgpu_waves_per_eu(6)))
select_stream_few_margin_kernel(SelectArgs a, int32_t cap)
{
    select_stream<SS_FEW_PER_THREAD, true>(a, cap);
}

__global__ void __launch_bounds__(SS_THREADS) __attribute__((amdgpu_waves_per_eu(4)))
select_stream_kernel(SelectArgs a, int32_t cap)
{
    select_stream<SS_MAX_PER_THREAD, false>(a, cap);
}

__global__ void __launch_bounds__(SS_THREADS) __attribute__((amdgpu_waves_per_eu(4)))
select_stream_margin_kernel(SelectArgs a, int32_t cap)
{
    select_stream<SS_MAX_PER_THREAD, true>(a, cap);
}

DeviceOnce g_setup;

}  // namespace

hipError_t select_setup()
{
    return g_setup.run([](int) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<true, false, SEL_MAX_ROUNDS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           SEL_CACHE_MAX_N * (int)sizeof(uint32_t));
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<true, true, SEL_MAX_ROUNDS>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    SEL_CACHE_MAX_N * (int)sizeof(uint32_t));
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_stream_few_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, SS_MAX_LDS);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_stream_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, SS_MAX_LDS);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_stream_few_margin_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, SS_MAX_LDS);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_stream_margin_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, SS_MAX_LDS);
        return e;
    });
}

hipError_t launch_select(const float* A, const uint8_t* anchor, const uint8_t* spons,
                         const float* vouch, const int32_t* seq_len,
                         int32_t layers, int32_t batch, int32_t hkv, int32_t n, int32_t K,
                         const ta_params& prm, int32_t* idx, int32_t* cnt, hipStream_t st)
{
    SelectArgs a;
    a.A = (prm.alpha != 0.0f) ? A : nullptr;
    a.anchor = anchor;
    a.spons = spons;
    a.vouch = vouch;
    a.seq_len = seq_len;
    a.layer_K = prm.layer_K;
    a.pool_r = (prm.alpha != 0.0f && prm.pool_k > 1) ? (prm.pool_k - 1) / 2 : 0;
    a.k_protected = prm.k_protected;
    a.idx = idx;
    a.cnt = cnt;
    a.margin = prm.margin;
    a.batch = batch;
    a.hkv = hkv;
    a.n = n;
    a.K = K;
    a.n_sink = prm.n_sink;
    a.n_recent = prm.n_recent;
    a.alpha = prm.alpha;
    a.beta = prm.beta;
    a.gamma = prm.gamma;
    const int64_t units = (int64_t)layers * batch * hkv;
    a.units = (int32_t)units;
    a.units_per_xcd = (int32_t)((units + 7) / 8);
    a.vec_ok = (n % 4 == 0) && ((uintptr_t)anchor % 4 == 0) && ((uintptr_t)spons % 4 == 0) &&
               ((uintptr_t)vouch % 16 == 0) && (a.A == nullptr || (uintptr_t)a.A % 16 == 0);
    const unsigned blocks = 8u * (unsigned)a.units_per_xcd;
    const bool capped = prm.k_protected >= 0;
    // The streaming form serves the plain (elastic, unpooled) selection on quad-aligned rows when
    // its candidate list and the bitmap of the sequence fit the LDS of a workgroup.
    if (!capped && a.pool_r == 0 && a.vec_ok && (n > SEL_CACHE_MAX_N || units >= SS_MIN_UNITS)) {
        const int64_t rmax = (int64_t)K - prm.n_sink - prm.n_recent;      // most slots the boundary class can have
        int64_t cap = rmax + SS_SEG + SS_SLACK;
        cap = (cap + SS_THREADS - 1) / SS_THREADS * SS_THREADS;
        const int64_t lds = cap * 8 + ((int64_t)n + 31) / 32 * 4;
        if (cap <= SS_MAX_CAP && lds <= SS_MAX_LDS) {
            const hipError_t attr_err = select_setup();
            if (attr_err != hipSuccess) return attr_err;
            const bool few = cap <= SS_THREADS * SS_FEW_PER_THREAD;
            auto kernel = few ? (a.margin ? select_stream_few_margin_kernel : select_stream_few_kernel)
                              : (a.margin ? select_stream_margin_kernel : select_stream_kernel);
            hipLaunchKernelGGL(kernel, dim3(blocks), dim3(SS_THREADS), (size_t)lds, st, a, (int32_t)cap);
            return hipGetLastError();
        }
    }
    if (n <= SEL_CACHE_MAX_N) {
        const hipError_t attr_err = select_setup();
        if (attr_err != hipSuccess) return attr_err;
        const size_t lds = (size_t)((n + 3) / 4 * 4) * sizeof(uint32_t);
        const bool one_round = n <= 4 * SEL_THREADS;         // 16 KB of keys: within the default dynamic LDS limit
        auto kernel = capped ? (one_round ? select_kernel<true, true, 1> : select_kernel<true, true, SEL_MAX_ROUNDS>)
                             : (one_round ? select_kernel<true, false, 1> : select_kernel<true, false, SEL_MAX_ROUNDS>);
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(SEL_THREADS), lds, st, a);
    } else {
        if (capped) hipLaunchKernelGGL((select_kernel<false, true, 0>), dim3(blocks), dim3(SEL_THREADS), 0, st, a);
        else hipLaunchKernelGGL((select_kernel<false, false, 0>), dim3(blocks), dim3(SEL_THREADS), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace ta
