// Learned anchor detection (Sec. 5.1 "Learned Anchor Detection"): per position the confidence
//   f(h) = sigmoid(W2 . GELU(W1 . h))
// of a small two-layer perceptron on the hidden state, the anchor flag f(h) > thr and the
// per-anchor sponsor budget of TA-Learned (fixed B) or TA-LearnRank (scale * f(h)).
//
// The first layer is a [positions x d_model] x [d_model x m] contraction: bf16 MFMA
// (v_mfma_f32_32x32x16_bf16), fp32 accumulation.  It is computed as W1 . h^T so that a lane
// owns ONE position (a column of the accumulator tile) and 16 hidden units of each tile: GELU,
// the product with W2 and the sum over the hidden units are then register arithmetic, followed
// by one half-wave exchange.  A workgroup owns 256 consecutive positions and all m hidden
// units; a wavefront owns 64 positions x (32 * HT) hidden units.  h and W1 stream through LDS
// in slices of 32 input features (64 bytes per row), a ring of three buffers filled by direct
// global->LDS loads two slices ahead, 16-byte chunks XOR-swizzled by row for conflict-free
// fragment reads.  W1 is re-read by every workgroup (from the L2: it is at most 16 MB, 1 MB for the usual
// d_model = 4096, m = 128); per workgroup that is m / positions of the bytes of h.
//
// The same kernel, in its second mode, is the embedding-based detector (Sec. 3.2 "Anchor detection",
// third instantiation; TA-Fast-Embedding): W1 holds the anchor-concept embeddings, the contraction
// gives every dot product x . c_e, the squared norms of both operands are summed from the very
// fragments the MFMA consumes (v_dot2_f32_bf16), and the epilogue takes the largest cosine and
// compares it with the threshold.
#include <math.h>


#include "ta_internal.h"
#include "ta_score_common.h"

namespace ta {

namespace {

constexpr int DT_KS = 32;                        // input features per slice

struct DetectArgs {
    const uint4* h;
    const uint4* W1;
    const uint16_t* W2;
    const int32_t* seq_len;
    float* conf;
    uint8_t* anchor;
    float* anchor_B;
    int64_t total;                               // batch * n positions
    int32_t n, dm, m;
    int32_t wrows;                               // rows W1 really has (<= m; the tile repeats the last one)
    int32_t h_row_bytes;                         // bytes between consecutive positions
    float thr, B, scale;
    int32_t rank;
};

__device__ __forceinline__ void dma16(const void* base, uint32_t off, uint32_t lds_base)
{
    // direct global->LDS load, 16 bytes per lane, lane i lands at lds_base + 16 i (inline assembly
    // so that the compiler does not wait for all of them before every LDS read)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(off), "s"(base)
                 : "memory", "m0");
}

constexpr int vm_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// erf(x) by the rational-exponential formula 7.1.26 of Abramowitz and Stegun,
//   erf(x) = sign(x) (1 - (a1 t + a2 t^2 + a3 t^3 + a4 t^4 + a5 t^5) exp(-x^2)),  t = 1 / (1 + p |x|),
// whose absolute error stays below 1.5e-7: the size of an fp32 rounding of the 1 + erf it feeds, at a
// third of the instructions of the library routine and without branches (the epilogue evaluates it
// 128 times per lane while the workgroup streams nothing).
__device__ __forceinline__ float erf_poly(float x)
{
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    poly *= t;
    const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * ax * ax);
    return copysignf(fmaf(-poly, e, 1.0f), x);
}

// acc + sum of the squares of the eight bf16 values of a fragment (fp32)
__device__ __forceinline__ float add_squares(uint4 v, float acc)
{
    union { uint32_t u; bf16x2 b; } c;
    c.u = v.x; acc = __builtin_amdgcn_fdot2_f32_bf16(c.b, c.b, acc, false);
    c.u = v.y; acc = __builtin_amdgcn_fdot2_f32_bf16(c.b, c.b, acc, false);
    c.u = v.z; acc = __builtin_amdgcn_fdot2_f32_bf16(c.b, c.b, acc, false);
    c.u = v.w; acc = __builtin_amdgcn_fdot2_f32_bf16(c.b, c.b, acc, false);
    return acc;
}

enum { MODE_MLP = 0, MODE_COSINE = 1 };
// Slice buffers of a workgroup.  Three (loads two slices ahead), except where two leave room for a third
// resident workgroup per compute unit (24 KB buffers of the 128-unit detector: 881 us against 903), which
// the long streams of the learned detector gain more from than from the deeper ring (the 256-unit
// detector, one large workgroup per compute unit either way, loses 8 % with two).
constexpr int detect_ring(int M, int MODE) { return (MODE == MODE_MLP && M == 128) ? 2 : 3; }

// TW: wavefront rows over the positions (64 TW positions per workgroup); HT: 32-unit hidden tiles
// per wavefront; MH: wavefront columns over the hidden units (m = 32 HT MH); MODE: which epilogue
template <int TW, int HT, int MH, int MODE>
__global__ void __launch_bounds__(64 * TW * MH, 2)
detect_kernel(DetectArgs a)
{
    constexpr int DT_TOKENS = 64 * TW;
    constexpr int THREADS = 64 * TW * MH;
    constexpr int M = 32 * HT * MH;
    constexpr int WAVES = TW * MH;
    constexpr int NI_H = DT_TOKENS / 16;                   // 1 KB loads per slice: h (16 rows each)
    constexpr int NI_W = M / 16;                           //                      W1
    constexpr int LH = NI_H / WAVES;                       // per wavefront
    constexpr int LW = (NI_W + WAVES - 1) / WAVES;         // (wraps: a few duplicate loads when M is small)
    constexpr int LPS = LH + LW;
    constexpr int H_BYTES = DT_TOKENS * 64;                // bytes of the h part of a buffer
    constexpr int BUF_BYTES = H_BYTES + M * 64;
    constexpr int DT_RING = detect_ring(M, MODE);

    extern __shared__ uint4 s_buf[];                       // DT_RING buffers, then W2 as floats
    float* s_w2 = reinterpret_cast<float*>(reinterpret_cast<char*>(s_buf) + DT_RING * BUF_BYTES);
    float* s_part = s_w2 + M;                              // [MH][DT_TOKENS] partial sums over hidden units
    float* s_xx = s_part + MH * DT_TOKENS;                 // [DT_TOKENS] squared norms of the positions' rows

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c32 = lane & 31, hf = lane >> 5;
    const int tw = wave % TW, mh = wave / TW;              // position block of 64, hidden column
    const int64_t tile0 = (int64_t)blockIdx.x * DT_TOKENS;
    const int nstages = a.dm / DT_KS;

    if constexpr (MODE == MODE_MLP)
        for (int j = tid; j < M; j += THREADS) s_w2[j] = bf16_bits_to_float(a.W2[j]);

    // per-lane byte offsets of this wavefront's loads inside a slice (loop invariant)
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4*)s_buf;
    uint32_t off_h[LH], off_w[LW];
    int ins_h[LH], ins_w[LW];
#pragma unroll
    for (int j = 0; j < LH; ++j) {
        const int ins = wave + WAVES * j;
        const int row = ins * 16 + (lane >> 2);
        int64_t t = tile0 + row;
        t = t < a.total ? t : a.total - 1;                 // stay inside the tensor; never stored
        const int chunk = (lane & 3) ^ ((row >> 2) & 3);
        off_h[j] = (uint32_t)((t - tile0) * a.h_row_bytes + chunk * 16);
        ins_h[j] = ins;
    }
#pragma unroll
    for (int j = 0; j < LW; ++j) {
        const int ins = (wave + WAVES * j) % NI_W;
        const int row = ins * 16 + (lane >> 2);
        const int chunk = (lane & 3) ^ ((row >> 2) & 3);
        const int src_row = row < a.wrows ? row : a.wrows - 1;   // missing rows repeat the last one
        off_w[j] = (uint32_t)(src_row * a.dm * 2 + chunk * 16);
        ins_w[j] = ins;
    }
    const char* hbase = reinterpret_cast<const char*>(a.h) + tile0 * a.h_row_bytes;
    const char* wbase = reinterpret_cast<const char*>(a.W1);
    const auto issue = [&](int s) {
        const uint32_t dst = lds0 + (uint32_t)(s % DT_RING) * BUF_BYTES;
        const char* hs = hbase + (size_t)s * (DT_KS * 2);
        const char* ws = wbase + (size_t)s * (DT_KS * 2);
#pragma unroll
        for (int j = 0; j < LH; ++j) dma16(hs, off_h[j], __builtin_amdgcn_readfirstlane(dst + ins_h[j] * 1024));
#pragma unroll
        for (int j = 0; j < LW; ++j)
            dma16(ws, off_w[j], __builtin_amdgcn_readfirstlane(dst + H_BYTES + ins_w[j] * 1024));
    };
    const auto wait_but = [](int k) {                      // at most k later slices outstanding
        switch (k) {
            case 0: __builtin_amdgcn_s_waitcnt(vm_imm(0)); break;
            case 1: __builtin_amdgcn_s_waitcnt(vm_imm(LPS)); break;
            default: __builtin_amdgcn_s_waitcnt(vm_imm(2 * LPS)); break;
        }
    };
    static_assert(2 * LPS <= 63, "vmcnt range");

#pragma unroll
    for (int s = 0; s < DT_RING - 1; ++s)
        if (s < nstages) issue(s);

    // fragment slots of this lane inside a buffer (16-byte units), for the two MFMA steps of a slice
    int slot_h[2][2], slot_w[HT][2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int row = 64 * tw + 32 * tt + c32;
            slot_h[tt][ks] = row * 4 + ((2 * ks + hf) ^ ((row >> 2) & 3));
        }
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            const int row = 32 * (mh * HT + ht) + c32;
            slot_w[ht][ks] = H_BYTES / 16 + row * 4 + ((2 * ks + hf) ^ ((row >> 2) & 3));
        }
    }

    f32x16 acc[2][HT];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tt][ht][i] = 0.0f;
    float xx[2] = {0.0f, 0.0f}, cc[HT];                    // cosine mode: squared norms, this lane's half of each row
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) cc[ht] = 0.0f;

    for (int s = 0; s < nstages; ++s) {
        const int later = nstages - 1 - s;
        wait_but(later < DT_RING - 2 ? later : DT_RING - 2);
        __syncthreads();                                   // slice s landed everywhere, slice s-1 consumed
        if (s + DT_RING - 1 < nstages) issue(s + DT_RING - 1);
        const uint4* buf = s_buf + (size_t)(s % DT_RING) * (BUF_BYTES / 16);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            uint4 hraw[2], wraw[HT];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) hraw[tt] = buf[slot_h[tt][ks]];
#pragma unroll
            for (int ht = 0; ht < HT; ++ht) wraw[ht] = buf[slot_w[ht][ks]];
            if constexpr (MODE == MODE_COSINE) {
#pragma unroll
                for (int tt = 0; tt < 2; ++tt) xx[tt] = add_squares(hraw[tt], xx[tt]);
#pragma unroll
                for (int ht = 0; ht < HT; ++ht) cc[ht] = add_squares(wraw[ht], cc[ht]);
            }
            bf16x8 hfrag[2], wfrag[HT];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) hfrag[tt] = as_frag(hraw[tt]);
#pragma unroll
            for (int ht = 0; ht < HT; ++ht) wfrag[ht] = as_frag(wraw[ht]);
#pragma unroll
            for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                for (int tt = 0; tt < 2; ++tt)   // rows: hidden units of the tile, columns: positions
                    acc[tt][ht] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfrag[ht], hfrag[tt], acc[tt][ht], 0, 0, 0);
        }
    }

    if constexpr (MODE == MODE_MLP) {
        // ---- epilogue: GELU, weights of the output unit, sum over the hidden units -----------
        // acc[tt][ht][i] is hidden unit 32 (mh HT + ht) + 8 (i / 4) + 4 hf + i % 4 of position 64 tw + 32 tt + c32
        float part[2];
    #pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            float sum = 0.0f;
    #pragma unroll
            for (int ht = 0; ht < HT; ++ht) {
    #pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    asm volatile("" ::: "memory");             // the weights are read where they are used, not all up front
                    const float4 w = *reinterpret_cast<const float4*>(&s_w2[32 * (mh * HT + ht) + 8 * i4 + 4 * hf]);
                    const float wv[4] = {w.x, w.y, w.z, w.w};
    #pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float z = acc[tt][ht][4 * i4 + c];
                        const float gelu = 0.5f * z * (1.0f + erf_poly(z * 0.70710678118654752f));
                        sum = fmaf(wv[c], gelu, sum);
                        asm volatile("" : "+v"(sum));          // consume each value now: no pile-up of live erf results
                    }
                }
            }
            sum += __shfl_xor(sum, 32);                        // the two half-waves hold disjoint hidden units
            part[tt] = sum;
        }
        if (hf == 0) {
    #pragma unroll
            for (int tt = 0; tt < 2; ++tt) s_part[mh * DT_TOKENS + 64 * tw + 32 * tt + c32] = part[tt];
        }
        __syncthreads();
        if (tid < DT_TOKENS) {                                 // THREADS >= DT_TOKENS
            const int64_t t = tile0 + tid;
            if (t < a.total) {
                float out = s_part[tid];
    #pragma unroll
                for (int c = 1; c < MH; ++c) out += s_part[c * DT_TOKENS + tid];
                float conf = 1.0f / (1.0f + expf(-out));
                if (a.seq_len) {
                    const int64_t b = t / a.n;
                    if ((int32_t)(t - b * a.n) >= a.seq_len[b]) conf = 0.0f;   // past the end of its sequence
                }
                const bool is_anchor = conf > a.thr;
                a.conf[t] = conf;
                a.anchor[t] = is_anchor ? 1 : 0;
                a.anchor_B[t] = is_anchor ? (a.rank ? a.scale * conf : a.B) : 0.0f;
            }
        }
    } else {
        // ---- epilogue: largest cosine --------------------------------------------------------
        // reciprocal norms of this wavefront column's concept rows, through LDS (s_w2 is free in this mode)
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            const float c2 = cc[ht] + __shfl_xor(cc[ht], 32);
            if (hf == 0 && tw == 0) s_w2[32 * (mh * HT + ht) + c32] = c2 > 0.0f ? 1.0f / sqrtf(c2) : 0.0f;
        }
        __syncthreads();
        float best[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            float b = -INFINITY;
#pragma unroll
            for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const float4 w = *reinterpret_cast<const float4*>(&s_w2[32 * (mh * HT + ht) + 8 * i4 + 4 * hf]);
                    b = fmaxf(b, acc[tt][ht][4 * i4 + 0] * w.x);
                    b = fmaxf(b, acc[tt][ht][4 * i4 + 1] * w.y);
                    b = fmaxf(b, acc[tt][ht][4 * i4 + 2] * w.z);
                    b = fmaxf(b, acc[tt][ht][4 * i4 + 3] * w.w);
                }
            best[tt] = fmaxf(b, __shfl_xor(b, 32));
            xx[tt] += __shfl_xor(xx[tt], 32);
        }
        if (hf == 0) {
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                s_part[mh * DT_TOKENS + 64 * tw + 32 * tt + c32] = best[tt];
                if (mh == 0) s_xx[64 * tw + 32 * tt + c32] = xx[tt];
            }
        }
        __syncthreads();
        if (tid < DT_TOKENS) {
            const int64_t t = tile0 + tid;
            if (t < a.total) {
                float b = s_part[tid];
#pragma unroll
                for (int c = 1; c < MH; ++c) b = fmaxf(b, s_part[c * DT_TOKENS + tid]);
                const float x2 = s_xx[tid];
                float sim = x2 > 0.0f ? b / sqrtf(x2) : 0.0f;
                if (a.seq_len) {
                    const int64_t sq = t / a.n;
                    if ((int32_t)(t - sq * a.n) >= a.seq_len[sq]) sim = 0.0f;
                }
                a.conf[t] = sim;
                a.anchor[t] = sim > a.thr ? 1 : 0;
            }
        }
    }
}

template <int TW, int HT, int MH, int MODE>
hipError_t launch_one(const DetectArgs& a, hipStream_t st)
{
    constexpr int M = 32 * HT * MH;
    constexpr int DT_TOKENS = 64 * TW;
    const size_t lds = (size_t)detect_ring(M, MODE) * (DT_TOKENS * 64 + M * 64) + (size_t)M * 4 + (size_t)(MH + 1) * DT_TOKENS * 4;
    static DeviceOnce setup;                               // dynamic LDS above 64 KB needs the attribute (per instantiation)
    const hipError_t attr_err = setup.run([&](int) {
        return hipFuncSetAttribute(reinterpret_cast<const void*>(&detect_kernel<TW, HT, MH, MODE>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    const unsigned blocks = (unsigned)((a.total + DT_TOKENS - 1) / DT_TOKENS);
    hipLaunchKernelGGL((detect_kernel<TW, HT, MH, MODE>), dim3(blocks), dim3(64 * TW * MH), lds, st, a);
    return hipGetLastError();
}

template <int MODE>
hipError_t launch_width(const DetectArgs& a, hipStream_t st)
{
    switch (a.m) {
        case 32: return launch_one<4, 1, 1, MODE>(a, st);
        case 64: return launch_one<4, 2, 1, MODE>(a, st);
        case 128: return launch_one<4, 4, 1, MODE>(a, st);
        default: return launch_one<4, 2, 4, MODE>(a, st);  // 256: sixteen wavefronts of 64 x 64
    }
}

}  // namespace

hipError_t launch_detect(const void* h, int64_t h_row_stride, const void* W1, const void* W2,
                         const int32_t* seq_len, int32_t batch, int32_t n, int32_t dm, int32_t m,
                         float thr, int32_t rank, float B, float scale,
                         float* conf, uint8_t* anchor, float* anchor_B, hipStream_t st)
{
    DetectArgs a;
    a.h = (const uint4*)h;
    a.W1 = (const uint4*)W1;
    a.W2 = (const uint16_t*)W2;
    a.seq_len = seq_len;
    a.conf = conf;
    a.anchor = anchor;
    a.anchor_B = anchor_B;
    a.total = (int64_t)batch * n;
    a.n = n;
    a.dm = dm;
    a.m = m;
    a.h_row_bytes = (int32_t)(h_row_stride * 2);
    a.thr = thr;
    a.B = B;
    a.scale = scale;
    a.rank = rank;
    a.wrows = m;
    return launch_width<MODE_MLP>(a, st);
}

hipError_t launch_cosine(const void* x, int64_t x_row_stride, const void* C, int32_t E, int64_t rows, int32_t dm,
                         const int32_t* seq_len, int32_t n, float tau, float* sim, uint8_t* anchor, hipStream_t st)
{
    DetectArgs a;
    a.h = (const uint4*)x;
    a.W1 = (const uint4*)C;
    a.W2 = nullptr;
    a.seq_len = seq_len;
    a.conf = sim;
    a.anchor = anchor;
    a.anchor_B = nullptr;
    a.total = rows;
    a.n = n;
    a.dm = dm;
    a.m = E <= 32 ? 32 : (E <= 64 ? 64 : (E <= 128 ? 128 : 256));
    a.wrows = E;
    a.h_row_bytes = (int32_t)(x_row_stride * 2);
    a.thr = tau;
    a.B = 0.0f;
    a.scale = 0.0f;
    a.rank = 0;
    return launch_width<MODE_COSINE>(a, st);
}

}  // namespace ta
