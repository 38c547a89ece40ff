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
#include <mutex>

#include "ta_internal.h"

namespace ta {

namespace {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int HIST_COPIES = 8;
constexpr int SEL_CACHE_MAX_N = 32768;        // keys cached in LDS up to this length

struct SelectArgs {
    const float* A;
    const uint8_t* anchor;
    const uint8_t* spons;
    const float* vouch;
    const int32_t* seq_len;
    int32_t* idx;
    int32_t* cnt;
    int32_t batch, hkv, n, K;
    int32_t n_sink, n_recent;
    float alpha, beta, gamma;
};

// Order-preserving map fp32 -> uint32 (larger float <=> larger integer).
__device__ __forceinline__ uint32_t ordered_bits(float u)
{
    uint32_t b = __float_as_uint(u);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
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
__device__ __forceinline__ RadixState radix_pick(uint32_t (*s_hist)[256], uint32_t* s_h,
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

template <bool CACHED>
__global__ void __launch_bounds__(SEL_THREADS)
select_kernel(SelectArgs a)
{
    extern __shared__ uint32_t s_key[];                     // [n] when CACHED
    __shared__ uint32_t s_hist[HIST_COPIES][256];
    __shared__ uint32_t s_h[256];
    __shared__ int s_red[SEL_WAVES];
    __shared__ RadixState s_state;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int32_t unit = blockIdx.x;
    const int32_t b = (unit / a.hkv) % a.batch;
    const int32_t n = a.n, K = a.K;
    int32_t nb = a.seq_len ? a.seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);
    int32_t* idx = a.idx + (size_t)unit * (size_t)K;

    if (nb <= K) {                                           // nothing to evict
        for (int32_t p = tid; p < nb; p += SEL_THREADS) idx[p] = p;
        if (tid == 0) a.cnt[unit] = nb;
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

    for (int i = tid; i < HIST_COPIES * 256; i += SEL_THREADS) (&s_hist[0][0])[i] = 0;

    int local = 0;
    for (int32_t p = ns + tid; p < rs; p += SEL_THREADS) local += spons[p] ? 1 : 0;
    const int32_t c1 = block_sum(local, s_red);

    const int bclass = (c2 + c1 <= K) ? 0 : 1;
    const int32_t R = bclass == 0 ? K - c2 - c1 : K - c2;    // slots for the boundary class
    const float nf = (float)nb;
    const bool use_A = (a.alpha != 0.0f);

    // order-preserving key of position p if it belongs to the boundary class, else 0
    auto make_key = [&](int32_t p) -> uint32_t {
        if (p < ns || p >= rs) return 0u;
        if ((spons[p] != 0) != (bclass == 1)) return 0u;
        float r = __fdiv_rn((float)(p + 1), nf);
        float t = use_A ? __fmul_rn(a.alpha, A[p]) : 0.0f;
        t = __fadd_rn(t, __fmul_rn(a.beta, r));
        t = __fadd_rn(t, __fmul_rn(a.gamma, (float)anchor[p]));
        t = __fadd_rn(t, vouch[p]);
        uint32_t k = ordered_bits(t);
        return k == 0u ? 1u : k;
    };
    auto key_at = [&](int32_t p) -> uint32_t { return CACHED ? s_key[p] : make_key(p); };

    if (CACHED) {
        for (int32_t p = tid; p < nb; p += SEL_THREADS) s_key[p] = make_key(p);
    }
    __syncthreads();

    // ---- threshold search ------------------------------------------------
    uint32_t T = 0xFFFFFFFFu;     // boundary-class position p is kept iff key > T, or key == T and p >= Pt
    int32_t Pt = 0x7FFFFFFF;
    if (R > 0) {
        uint32_t prefix = 0, need = (uint32_t)R;
        bool done = false;
        for (int pass = 0; pass < 4 && !done; ++pass) {
            const int shift = 24 - 8 * pass;
            for (int32_t p = tid; p < nb; p += SEL_THREADS) {
                uint32_t k = key_at(p);
                bool in = k != 0u && (pass == 0 || (k >> (shift + 8)) == (prefix >> (shift + 8)));
                if (in) atomicAdd(&s_hist[lane & (HIST_COPIES - 1)][(k >> shift) & 255u], 1u);
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
                    for (int32_t p = tid; p < nb; p += SEL_THREADS) {
                        bool in = key_at(p) == T &&
                                  (pp == 0 || ((uint32_t)p >> (ps + 8)) == (pprefix >> (ps + 8)));
                        if (in) atomicAdd(&s_hist[lane & (HIST_COPIES - 1)][((uint32_t)p >> ps) & 255u], 1u);
                    }
                    __syncthreads();
                    RadixState q = radix_pick(s_hist, s_h, &s_state, pneed);
                    pprefix |= q.digit << ps;
                    pneed = q.need;
                }
                Pt = (int32_t)pprefix;                       // positions are unique: pneed == 1 here
                done = true;
            }
        }
    }

    // ---- ascending write-out ----------------------------------------------
    int32_t base = 0;
    for (int32_t p0 = 0; p0 < nb; p0 += SEL_THREADS) {
        const int32_t p = p0 + tid;
        bool keep = false;
        if (p < nb) {
            if (p < ns || p >= rs) {
                keep = true;
            } else {
                const bool sp = spons[p] != 0;
                if (sp != (bclass == 1)) {
                    keep = sp;                               // class 1 above the boundary class, class 0 below it
                } else {
                    uint32_t k = key_at(p);
                    keep = (k > T) || (k == T && p >= Pt);
                }
            }
        }
        unsigned long long m = __ballot(keep);
        int before = __popcll(m & ((1ull << lane) - 1ull));
        __syncthreads();
        if (lane == 0) s_red[wave] = __popcll(m);
        __syncthreads();
        int woff = 0, total = 0;
        for (int w = 0; w < SEL_WAVES; ++w) {
            int c = s_red[w];
            woff += (w < wave) ? c : 0;
            total += c;
        }
        const int32_t slot = base + woff + before;
        if (keep && slot < K) idx[slot] = p;
        base += total;
    }
    if (tid == 0) a.cnt[unit] = base < K ? base : K;
}

std::once_flag g_attr_once;

}  // namespace

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
    a.idx = idx;
    a.cnt = cnt;
    a.batch = batch;
    a.hkv = hkv;
    a.n = n;
    a.K = K;
    a.n_sink = prm.n_sink;
    a.n_recent = prm.n_recent;
    a.alpha = prm.alpha;
    a.beta = prm.beta;
    a.gamma = prm.gamma;
    const unsigned units = (unsigned)((int64_t)layers * batch * hkv);
    if (n <= SEL_CACHE_MAX_N) {
        hipError_t attr_err = hipSuccess;
        std::call_once(g_attr_once, [&]() {
            attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           SEL_CACHE_MAX_N * (int)sizeof(uint32_t));
        });
        if (attr_err != hipSuccess) return attr_err;
        hipLaunchKernelGGL(select_kernel<true>, dim3(units), dim3(SEL_THREADS),
                           (size_t)n * sizeof(uint32_t), st, a);
    } else {
        hipLaunchKernelGGL(select_kernel<false>, dim3(units), dim3(SEL_THREADS), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace ta
