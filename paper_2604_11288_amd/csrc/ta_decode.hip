// Incremental form of the eviction pass: one generation step for every
// sequence and unit (Sec. 3.1 "after each generation step"; Alg. 1 with its
// budget-decay step; Sec. 3.2 "Token selection").
//
// Kernels per step:
//   decode_seq_kernel    one workgroup per sequence: append the token, test the
//                        anchor table at the new position only, set its budget
//   decode_vouch_kernel  voucher and sponsor flag of every position from the current budgets
//   decode_unit_kernel   one wavefront per unit: write the new k/v row into the
//                        free slot, add the decode queries' softmax weights over
//                        the cached rows to A (H2O-style cumulative attention,
//                        Eq. 1), free the slot that ranks last under the
//                        (class, u, position) order
//   decode_decay_kernel  B_i <- decay * B_i for every position
// The unit kernel is the hot one: it reads the unit's K slots once (HBM bound,
// (K+1) * 256 B per unit per step).  The logits of the group's query heads over the
// slots are a thin contraction that runs on the matrix cores (16-row key tiles x 16
// head columns), fed with whole key rows that are turned into operand fragments
// through a small LDS tile.
#include <math.h>

#include "ta_internal.h"

namespace ta {

namespace {

constexpr int DU_THREADS = 256;
constexpr int DU_WAVES = DU_THREADS / 64;
constexpr int MAX_GROUP = 16;                              // query heads per KV head (the columns of an MFMA tile)

struct DecodeTable {
    int32_t rid[TA_MAX_TABLE][TA_MAX_GRAM];                // n-grams reversed: rid[e][0] = last token
    int32_t len[TA_MAX_TABLE];
    int32_t E;
    float B;
};

// K/V slots kept in a paged pool (ta_decode_state::pages): strides in 16-byte units.
struct SlotPages {
    const int32_t* table;                                  // [batch][max_pages]
    int64_t s_layer, s_page, s_slot, s_head;
    int32_t page_size, max_pages, num_pages;
    int32_t page_shift;                                    // log2(page_size) when it is a power of two, else -1
};

__device__ __forceinline__ int32_t page_index(const SlotPages& pg, int32_t slot)
{
    return pg.page_shift >= 0 ? slot >> pg.page_shift : slot / pg.page_size;
}

__device__ __forceinline__ int32_t clamp_page(const SlotPages& pg, int32_t page)
{
    return page < 0 ? 0 : (page >= pg.num_pages ? pg.num_pages - 1 : page);
}

// ---- state initialisation -----------------------------------------------------
__global__ void decode_init_seq_kernel(ta_decode_state st, const int32_t* tok, const int32_t* seq_len, int32_t n,
                                       const uint8_t* anchor, const float* anchor_B, float B)
{
    const int b = blockIdx.y;
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    int32_t nb = seq_len ? seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);
    if (p == 0) st.len[b] = nb;
    if (p >= st.cap) return;
    const size_t o = (size_t)b * st.cap + p;
    if (p < nb) {
        const size_t i = (size_t)b * n + p;
        const uint8_t a = anchor[i];
        st.tok[o] = tok[i];
        st.anchor[o] = a;
        st.budget[o] = a ? (anchor_B ? anchor_B[i] : B) : 0.0f;
    } else {
        st.tok[o] = 0;
        st.anchor[o] = 0;
        st.budget[o] = 0.0f;
    }
}

template <bool PAGED>
__global__ void __launch_bounds__(DU_THREADS)
decode_init_unit_kernel(ta_decode_state st, int32_t n, const float* A, const int32_t* idx, const int32_t* cnt,
                        const uint4* Kout, const uint4* Vout, SlotPages pg)
{
    const int unit = blockIdx.x;
    const int slots = st.K + 1;
    int32_t c = cnt[unit];
    c = c < 0 ? 0 : (c > st.K ? st.K : c);
    for (int s = threadIdx.x; s < slots; s += DU_THREADS) {
        int32_t p = -1;
        float a = 0.0f;
        if (s < c) {
            p = idx[(size_t)unit * st.K + s];
            p = p < 0 ? 0 : (p >= n ? n - 1 : p);
            if (A) a = A[(size_t)unit * n + p];
        }
        st.pos[(size_t)unit * slots + s] = p;
        st.A[(size_t)unit * slots + s] = a;
    }
    if (!Kout) return;                                     // paged state whose rows are in place already
    const uint4 zero = make_uint4(0, 0, 0, 0);
    if (PAGED) {
        const int g = unit % st.hkv;
        const int b = (unit / st.hkv) % st.batch;
        const int l = unit / (st.hkv * st.batch);
        uint4* Kc = reinterpret_cast<uint4*>(st.Kc) + l * pg.s_layer + g * pg.s_head;
        uint4* Vc = reinterpret_cast<uint4*>(st.Vc) + l * pg.s_layer + g * pg.s_head;
        for (int i = threadIdx.x; i < slots * 16; i += DU_THREADS) {
            const int s = i >> 4;
            const int32_t j = page_index(pg, s);
            const int32_t page = clamp_page(pg, pg.table[(size_t)b * pg.max_pages + j]);
            const int64_t at = (int64_t)page * pg.s_page + (int64_t)(s - j * pg.page_size) * pg.s_slot + (i & 15);
            Kc[at] = s < c ? Kout[(size_t)unit * st.K * 16 + i] : zero;
            Vc[at] = s < c ? Vout[(size_t)unit * st.K * 16 + i] : zero;
        }
        return;
    }
    uint4* Kc = reinterpret_cast<uint4*>(st.Kc) + (size_t)unit * slots * 16;
    uint4* Vc = reinterpret_cast<uint4*>(st.Vc) + (size_t)unit * slots * 16;
    for (int i = threadIdx.x; i < slots * 16; i += DU_THREADS) {
        const int s = i >> 4;
        Kc[i] = s < c ? Kout[(size_t)unit * st.K * 16 + i] : zero;
        Vc[i] = s < c ? Vout[(size_t)unit * st.K * 16 + i] : zero;
    }
}

// ---- step, sequence part ---------------------------------------------------------
__global__ void __launch_bounds__(64)
decode_seq_kernel(ta_decode_state st, const int32_t* new_tok, DecodeTable tab)
{
    const int b = blockIdx.x;
    const int32_t p = st.len[b];
    if (p < 0 || p >= st.cap) {                            // at capacity: the step leaves this sequence and its units alone
        if (threadIdx.x == 0) st.stepped[b] = 0;
        return;
    }
    int32_t* tok = st.tok + (size_t)b * st.cap;
    const int32_t t0 = new_tok[b];
    const int e = threadIdx.x;
    bool hit = false;
    if (e < tab.E && t0 == tab.rid[e][0]) {
        const int32_t len = tab.len[e];
        hit = p - len + 1 >= 0;
        for (int k = 1; k < len && hit; ++k) hit = tok[p - k] == tab.rid[e][k];
    }
    const bool any = __ballot(hit) != 0ull;
    if (threadIdx.x == 0) {
        tok[p] = t0;
        st.anchor[(size_t)b * st.cap + p] = any ? 1 : 0;
        st.budget[(size_t)b * st.cap + p] = any ? tab.B : 0.0f;
        st.len[b] = p + 1;
        st.stepped[b] = 1;
    }
}

__global__ void decode_decay_kernel(ta_decode_state st, float decay)
{
    const int b = blockIdx.y;
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < st.len[b] && p < st.cap && st.stepped[b]) {
        float* B = st.budget + (size_t)b * st.cap + p;
        *B = __fmul_rn(decay, *B);
    }
}

// Voucher and sponsor flag of every position from the current budgets (Eq. 2): the same for all
// units of a sequence, so it is computed once per sequence and step, not once per cached row.
struct VouchArgs {
    int32_t L;
    float pw[TA_MAX_SPAN + 1];
};

__global__ void decode_vouch_kernel(ta_decode_state st, VouchArgs a)
{
    const int b = blockIdx.y;
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= st.len[b] || p >= st.cap) return;
    const size_t row = (size_t)b * st.cap;
    const uint8_t* anchor = st.anchor + row;
    const float* budget = st.budget + row;
    float v = 0.0f;
    uint8_t sp = 0;
    for (int k = 1; k <= a.L; ++k) {
        const int32_t i = p - k;
        if (i >= 0 && anchor[i]) {
            v = __fadd_rn(v, __fmul_rn(budget[i], a.pw[k]));
            sp = 1;
        }
    }
    st.vouch[row + p] = v;
    st.spons[row + p] = sp;
}

// ---- step, unit part ----------------------------------------------------------------
struct UnitArgs {
    const uint4* q_new;
    const uint4* k_new;
    const uint4* v_new;
    int32_t* evicted;
    int32_t n_sink, n_recent;
    float alpha, beta, gamma;
    float scale_log2;
    int32_t last_query;                                    // 1: A holds this step's attention, not the running sum
    int32_t pg_off;                                        // paged slots: offset (in floats) of the page list in the wavefront's LDS
};

__device__ __forceinline__ uint32_t ordered_bits(float u)
{
    uint32_t b = __float_as_uint(u);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

template <typename T, typename Op>
__device__ __forceinline__ T block_reduce(T v, T* s_red, Op op)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = op(v, __shfl_xor(v, o));
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) s_red[wave] = v;
    __syncthreads();
    T r = s_red[0];
#pragma unroll
    for (int w = 1; w < DU_WAVES; ++w) r = op(r, s_red[w]);
    return r;
}

constexpr int DT_RING = 4;                                 // 16-row key tiles held per wavefront: one multiplied, the others in flight

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// the two 8-byte halves of a 16-byte load as MFMA operand fragments (four bf16 each)
__device__ __forceinline__ s16x4 lo_half(const uint4& v)
{
    union { uint2 u; s16x4 s; } c;
    c.u = make_uint2(v.x, v.y);
    return c.s;
}
__device__ __forceinline__ s16x4 hi_half(const uint4& v)
{
    union { uint2 u; s16x4 s; } c;
    c.u = make_uint2(v.z, v.w);
    return c.s;
}

// One wavefront per unit, no workgroup barriers: the step of a unit is a chain of short
// phases, and what hides their latency is the number of units in flight per compute unit.
// LDS (private to the wavefront): slot table, accumulated attention, [G][slots] logits.
template <int GH, bool PAGED>                             // query heads per KV head the loops are unrolled for; K/V slots in pages
__global__ void __launch_bounds__(64)
decode_unit_kernel(ta_decode_state st, UnitArgs a, SlotPages pg)
{
    extern __shared__ float s_dyn[];

    const int lane = threadIdx.x;
    const int sub = lane & 15, grp = lane >> 4;            // 16 lanes per key row, 4 rows per instruction
    const int unit = blockIdx.x;
    const int slots = st.K + 1;
    const int G = st.hq / st.hkv;
    const int g = unit % st.hkv;
    const int b = (unit / st.hkv) % st.batch;
    const int l = unit / (st.hkv * st.batch);
    const int32_t len_new = st.len[b];                     // the sequence part of the step has run
    const int32_t p_new = len_new - 1;
    int32_t* pos = st.pos + (size_t)unit * slots;
    float* A = st.A + (size_t)unit * slots;
    uint4* Kc = reinterpret_cast<uint4*>(st.Kc) + (PAGED ? l * pg.s_layer + g * pg.s_head : (int64_t)unit * slots * 16);
    uint4* Vc = reinterpret_cast<uint4*>(st.Vc) + (PAGED ? l * pg.s_layer + g * pg.s_head : (int64_t)unit * slots * 16);
    const bool scored = a.alpha != 0.0f;
    // Paged slots: the pages of this unit's slots go to LDS first (one dependent round trip through
    // the L2 per unit), so that a row's address afterwards costs an LDS read and no memory access.
    int32_t* s_pg = reinterpret_cast<int32_t*>(s_dyn + a.pg_off);
    if (PAGED) {
        const int npg = page_index(pg, slots - 1) + 1;
        for (int j = lane; j < npg; j += 64) s_pg[j] = clamp_page(pg, pg.table[(size_t)b * pg.max_pages + j]);
        __builtin_amdgcn_wave_barrier();
    }
    const auto row_at = [&](int row) -> int64_t {           // 16-byte index of a slot's first chunk
        if (!PAGED) return (int64_t)row * 16;
        const int32_t j = page_index(pg, row);
        return (int64_t)s_pg[j] * pg.s_page + (int64_t)(row - j * pg.page_size) * pg.s_slot;
    };
    int32_t* s_pos = reinterpret_cast<int32_t*>(s_dyn);
    float* s_A = s_dyn + slots;
    const int wstride = (slots + 3) & ~3;                  // logits of a head: padded to whole 16-byte groups
    uint4* s_t = reinterpret_cast<uint4*>(s_dyn + ((2 * slots + 3) & ~3));   // one 16-row key tile, 4 KB (scored only)
    float* s_w = reinterpret_cast<float*>(s_t + 256);

    // The logits of the group's decode queries over the cached rows are a [slots x d] x [d x G]
    // contraction: v_mfma_f32_16x16x16_bf16 with 16 key rows as the rows of a tile and the heads
    // as its columns (G <= 16 of them are used; the matrix pipe is idle otherwise).
    // Key rows are loaded the way memory likes them - a wavefront instruction takes four whole
    // consecutive rows, 16 lanes x 16 bytes each - and turned into operand fragments through a
    // 4 KB tile in LDS: lane (i16, kq) of the matrix layout needs 16 bytes of row i16 at chunk
    // kq + 4 t, t = 0..3, and uses their two halves as two k-steps.  (Loading the fragments
    // straight from global memory - 16 rows x 64 bytes per instruction - streams at 4.6 TB/s,
    // whole rows at 5.8.)  The query fragments are loaded with the fragment addressing, so both
    // operands see the features in the same (permuted) order, which a contraction does not
    // care about.  The first tiles and the queries are requested before anything else.
    const int i16 = sub, kq = grp;
    const int ntiles = (slots + 15) >> 4;
    uint4 qf[4], tiles[DT_RING][4];                        // DT_RING - 1 tiles in flight while one is multiplied
    const auto load_tile = [&](int tile, uint4 (&dst)[4]) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            int row = tile * 16 + 4 * t + grp;
            row = row < slots ? row : slots - 1;           // past the last slot: a valid row, masked at the store
            dst[t] = Kc[row_at(row) + sub];
        }
    };
    if (scored) {
        const uint4* qrow = a.q_new + ((size_t)(l * st.batch + b) * st.hq + g * G + (i16 < G ? i16 : 0)) * 16;
#pragma unroll
        for (int t = 0; t < 4; ++t) qf[t] = i16 < G ? qrow[kq + 4 * t] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < DT_RING - 1; ++j)
            if (j < ntiles) load_tile(j, tiles[j]);
    }
    int first_free = 0x7FFFFFFF;                           // lowest-numbered free slot
    for (int s0 = lane; s0 < slots; s0 += 4 * 64) {        // four slots per lane and round trip
        int32_t p4[4];
        float a4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s = s0 + 64 * j;
            p4[j] = s < slots ? pos[s] : 0;
            a4[j] = s < slots ? A[s] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s = s0 + 64 * j;
            if (s < slots) {
                s_pos[s] = p4[j];
                s_A[s] = a4[j];
                if (p4[j] < 0) first_free = first_free < s ? first_free : s;
            }
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const int other = __shfl_xor(first_free, o);
        first_free = other < first_free ? other : first_free;
    }
    const int f = first_free;
    if (f >= slots || p_new < 0 || !st.stepped[b]) {       // no room, empty sequence, or a sequence at capacity: nothing to do
        if (lane == 0 && a.evicted) a.evicted[unit] = -1;
        return;
    }
    const uint4* kn = a.k_new + ((size_t)(l * st.batch + b) * st.hkv + g) * 16;
    const uint4* vn = a.v_new + ((size_t)(l * st.batch + b) * st.hkv + g) * 16;
    if (lane < 16) Kc[row_at(f) + lane] = kn[lane];
    else if (lane < 32) Vc[row_at(f) + lane - 16] = vn[lane - 16];
    __builtin_amdgcn_wave_barrier();                       // the slot table is in LDS for every lane

    // ---- attention of the group's decode queries over the occupied slots ----------
    if (scored) {
        const auto frag_logits = [&](const uint4 (&frag)[4]) -> f32x4 {
            f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(lo_half(frag[t]), lo_half(qf[t]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(hi_half(frag[t]), hi_half(qf[t]), acc, 0, 0, 0);
            }
            return acc;                                    // rows 4 kq .. 4 kq + 3 of the tile, head i16
        };
        // whole rows -> fragments through the LDS tile: row r chunk c sits at r * 16 + (c ^ r), which
        // keeps both the row-wise writes and the column-wise reads free of bank conflicts.  LDS
        // operations of a wavefront execute in order, so the tile needs no barrier (a wave-barrier
        // builtin here would also keep the staging registers in scratch memory).
        const auto tile_logits = [&](const uint4 (&rows)[4]) -> f32x4 {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int r = 4 * t + grp;
                s_t[r * 16 + (sub ^ r)] = make_uint4(rows[t].x, rows[t].y, rows[t].z, rows[t].w);   // by components: a struct copy keeps `rows` in scratch memory
            }
            uint4 frag[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint4 v = s_t[i16 * 16 + ((kq + 4 * t) ^ i16)];
                frag[t] = make_uint4(v.x, v.y, v.z, v.w);
            }
            return frag_logits(frag);
        };
        const auto store_tile = [&](int tile, const f32x4& acc) {
            const int s = tile * 16 + 4 * kq;
            if (i16 < G && s < wstride) {
                const int4 p4 = *reinterpret_cast<const int4*>(&s_pos[s]);   // past `slots`: other LDS of this wavefront, masked
                float4 o;
                o.x = (s + 0 < slots && p4.x >= 0) ? acc[0] * a.scale_log2 : -INFINITY;
                o.y = (s + 1 < slots && p4.y >= 0) ? acc[1] * a.scale_log2 : -INFINITY;
                o.z = (s + 2 < slots && p4.z >= 0) ? acc[2] * a.scale_log2 : -INFINITY;
                o.w = (s + 3 < slots && p4.w >= 0) ? acc[3] * a.scale_log2 : -INFINITY;
                *reinterpret_cast<float4*>(&s_w[i16 * wstride + s]) = o;
            }
        };
        // the tiles rotate through the registers (constant indices once unrolled)
        for (int tb = 0; tb < ntiles; tb += DT_RING) {
#pragma unroll
            for (int j = 0; j < DT_RING; ++j) {
                if (tb + j < ntiles) {
                    if (tb + j + DT_RING - 1 < ntiles) load_tile(tb + j + DT_RING - 1, tiles[(j + DT_RING - 1) % DT_RING]);
                    store_tile(tb + j, tile_logits(tiles[j]));
                }
            }
        }
        // the row that has just been written is not read back: its logits come from the new key
        // itself (whatever the loop stored for that slot is replaced here)
        {
            uint4 knf[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) knf[t] = kn[kq + 4 * t];          // every row of this tile is the new key
            const f32x4 acc = frag_logits(knf);
            __builtin_amdgcn_wave_barrier();
            if (i16 < G && kq == 0) s_w[i16 * wstride + f] = acc[0] * a.scale_log2;
            __builtin_amdgcn_wave_barrier();
        }
        // softmax statistics of every head, then the weights are added per slot in head order
        // (H2O-style cumulative attention)
        float m_h[GH], inv_h[GH];
#pragma unroll
        for (int h = 0; h < GH; ++h) {
            m_h[h] = 0.0f;
            inv_h[h] = 0.0f;
            if (h < G) {
                const float* sh = s_w + h * wstride;
                float m = -INFINITY;
                for (int s = lane; s < slots; s += 64) m = fmaxf(m, sh[s]);
                m = wave_max(m);
                float z = 0.0f;
                for (int s = lane; s < slots; s += 64) z += __builtin_amdgcn_exp2f(sh[s] - m);
                z = wave_sum(z);
                m_h[h] = m;
                inv_h[h] = 1.0f / z;
            }
        }
        for (int s = lane; s < slots; s += 64) {
            if (s == f || s_pos[s] >= 0) {
                float add = 0.0f;
#pragma unroll
                for (int h = 0; h < GH; ++h)
                    if (h < G) add += __builtin_amdgcn_exp2f(s_w[h * wstride + s] - m_h[h]) * inv_h[h];
                // cumulative mass over the steps, or (TOVA's step-wise rule) this step's mass alone
                const float v = a.last_query ? add : (s == f ? 0.0f : s_A[s]) + add;
                s_A[s] = v;
                A[s] = v;
            }
        }
    } else {
        if (lane == 0) {
            s_A[f] = 0.0f;
            A[f] = 0.0f;
        }
    }

    // ---- rank the occupied slots; evict the last one if the cache is over budget -----
    // (every lane ranks the slots it wrote s_A for)
    const size_t srow = (size_t)b * st.cap;
    const uint8_t* anchor = st.anchor + srow;
    const uint8_t* spons = st.spons + srow;
    const float* vouch = st.vouch + srow;
    const float lenf = (float)len_new;
    unsigned long long worst = ~0ull;
    int nfree = 0;
    for (int s0 = lane; s0 < slots; s0 += 4 * 64) {        // four slots per lane and round trip
        int32_t p4[4];
        float v4[4];
        uint8_t sp4[4], an4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s = s0 + 64 * j;
            p4[j] = s < slots ? ((s == f) ? p_new : s_pos[s]) : -2;
            const int32_t pc = p4[j] < 0 ? 0 : p4[j];
            v4[j] = vouch[pc];
            sp4[j] = spons[pc];
            an4[j] = anchor[pc];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int s = s0 + 64 * j;
            const int32_t p = p4[j];
            if (p == -2) continue;                         // past the last slot
            if (p < 0) { ++nfree; continue; }
            const float r = __fdiv_rn((float)(p + 1), lenf);
            float t = scored ? __fmul_rn(a.alpha, s_A[s]) : 0.0f;
            t = __fadd_rn(t, __fmul_rn(a.beta, r));
            t = __fadd_rn(t, __fmul_rn(a.gamma, (float)an4[j]));
            t = __fadd_rn(t, v4[j]);
            const unsigned cls = (p < a.n_sink || p >= len_new - a.n_recent) ? 2u : (sp4[j] ? 1u : 0u);
            // (class, u, position) packed so that the smallest integer ranks last
            const unsigned long long key = ((unsigned long long)cls << 62) |
                                           ((unsigned long long)ordered_bits(t) << 30) | (unsigned long long)(uint32_t)p;
            worst = key < worst ? key : worst;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        nfree += __shfl_xor(nfree, o);
        const unsigned long long other = __shfl_xor(worst, o);
        worst = other < worst ? other : worst;
    }
    const int32_t evict_pos = nfree > 0 ? -1 : (int32_t)(worst & 0x3FFFFFFFull);
    for (int s = lane; s < slots; s += 64) {
        const int32_t p = (s == f) ? p_new : s_pos[s];
        if (s == f || (p >= 0 && p == evict_pos)) pos[s] = (p == evict_pos) ? -1 : p;
    }
    if (lane == 0 && a.evicted) a.evicted[unit] = evict_pos;
}

DeviceOnce g_setup;

SlotPages slot_pages(const ta_decode_state& st)
{
    SlotPages pg = {};
    pg.page_size = 1;
    pg.page_shift = -1;
    if (st.pages) {
        const ta_paged_kv& p = *st.pages;
        pg.table = p.block_table;
        pg.s_layer = p.stride[0] / 8;
        pg.s_page = p.stride[1] / 8;
        pg.s_slot = p.stride[2] / 8;
        pg.s_head = p.stride[3] / 8;
        pg.page_size = p.page_size;
        pg.max_pages = p.max_pages;
        pg.num_pages = p.num_pages;
        if ((p.page_size & (p.page_size - 1)) == 0) {
            pg.page_shift = 0;
            while ((1 << pg.page_shift) < p.page_size) ++pg.page_shift;
        }
    }
    return pg;
}

template <int GH>
hipError_t unit_attributes()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_unit_kernel<GH, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_unit_kernel<GH, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return e;
}

template <int GH>
void launch_unit(const ta_decode_state& st, const UnitArgs& a, const SlotPages& pg, unsigned units, size_t lds, hipStream_t s)
{
    if (st.pages) hipLaunchKernelGGL((decode_unit_kernel<GH, true>), dim3(units), dim3(64), lds, s, st, a, pg);
    else hipLaunchKernelGGL((decode_unit_kernel<GH, false>), dim3(units), dim3(64), lds, s, st, a, pg);
}

}  // namespace

hipError_t decode_setup()
{
    return g_setup.run([](int) {
        hipError_t e = unit_attributes<4>();
        if (e == hipSuccess) e = unit_attributes<8>();
        if (e == hipSuccess) e = unit_attributes<MAX_GROUP>();
        return e;
    });
}

hipError_t launch_decode_init(const ta_decode_state& st, const int32_t* tok, const int32_t* seq_len, int32_t n,
                              const uint8_t* anchor, const float* anchor_B, const float* A,
                              const int32_t* idx, const int32_t* cnt, const void* Kout, const void* Vout,
                              float B, hipStream_t s)
{
    dim3 g1((unsigned)((st.cap + 255) / 256), (unsigned)st.batch);
    hipLaunchKernelGGL(decode_init_seq_kernel, g1, dim3(256), 0, s, st, tok, seq_len, n, anchor, anchor_B, B);
    const unsigned units = (unsigned)(st.layers * st.batch * st.hkv);
    const SlotPages pg = slot_pages(st);
    if (st.pages)
        hipLaunchKernelGGL(decode_init_unit_kernel<true>, dim3(units), dim3(DU_THREADS), 0, s, st, n, A, idx, cnt,
                           (const uint4*)Kout, (const uint4*)Vout, pg);
    else
        hipLaunchKernelGGL(decode_init_unit_kernel<false>, dim3(units), dim3(DU_THREADS), 0, s, st, n, A, idx, cnt,
                           (const uint4*)Kout, (const uint4*)Vout, pg);
    return hipGetLastError();
}

hipError_t launch_decode_step(const ta_decode_state& st, const int32_t* new_tok, const void* q_new,
                              const void* k_new, const void* v_new, const MatchTable& tab,
                              const ta_params& prm, int32_t* evicted, hipStream_t s)
{
    DecodeTable dt;
    for (int e = 0; e < TA_MAX_TABLE; ++e) {
        for (int k = 0; k < TA_MAX_GRAM; ++k) dt.rid[e][k] = tab.rid[e][k];
        dt.len[e] = tab.len[e];
    }
    dt.E = tab.E;
    dt.B = tab.B;
    hipLaunchKernelGGL(decode_seq_kernel, dim3((unsigned)st.batch), dim3(64), 0, s, st, new_tok, dt);

    VouchArgs va;
    va.L = prm.span_L;
    for (int k = 0; k <= TA_MAX_SPAN; ++k) va.pw[k] = tab.pw[k];
    dim3 gv((unsigned)((st.cap + 255) / 256), (unsigned)st.batch);
    hipLaunchKernelGGL(decode_vouch_kernel, gv, dim3(256), 0, s, st, va);

    UnitArgs a;
    a.q_new = (const uint4*)q_new;
    a.k_new = (const uint4*)k_new;
    a.v_new = (const uint4*)v_new;
    a.evicted = evicted;
    a.n_sink = prm.n_sink;
    a.n_recent = prm.n_recent;
    a.alpha = prm.alpha;
    a.beta = prm.beta;
    a.gamma = prm.gamma;
    a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)st.d));
    a.last_query = prm.last_query;
    const unsigned units = (unsigned)(st.layers * st.batch * st.hkv);
    const int G = st.hq / st.hkv;
    const int slots = st.K + 1;
    // slot table and accumulated attention; with an attention term also one key tile and the logits
    size_t lds_floats = prm.alpha != 0.0f ? (size_t)((2 * slots + 3) & ~3) + 1024 + (size_t)G * ((slots + 3) & ~3) : (size_t)2 * slots;
    const SlotPages pg = slot_pages(st);
    a.pg_off = (int32_t)lds_floats;
    if (st.pages) lds_floats += (size_t)((slots - 1) / pg.page_size + 1);      // the pages of the unit's slots
    const size_t lds = lds_floats * sizeof(float);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    const hipError_t attr_err = decode_setup();            // dynamic LDS above 64 KB (large budgets) needs the attribute
    if (attr_err != hipSuccess) return attr_err;
    if (G <= 4) launch_unit<4>(st, a, pg, units, lds, s);
    else if (G <= 8) launch_unit<8>(st, a, pg, units, lds, s);
    else launch_unit<MAX_GROUP>(st, a, pg, units, lds, s);

    dim3 g3((unsigned)((st.cap + 255) / 256), (unsigned)st.batch);
    hipLaunchKernelGGL(decode_decay_kernel, g3, dim3(256), 0, s, st, prm.budget_decay);
    return hipGetLastError();
}

}  // namespace ta
