// Incremental form of the eviction pass: one generation step for every
// sequence and unit (Sec. 3.1 "after each generation step"; Alg. 1 with its
// budget-decay step; Sec. 3.2 "Token selection").
//
// Two launches per step:
//   decode_seq_vouch_kernel  per sequence: append the token, test the anchor table at the new
//                            position only, set its budget; voucher and sponsor flag of every
//                            position from the current budgets
//   decode_unit_kernel       one wavefront per unit: write the new k/v row into the
//                            free slot, add the decode queries' softmax weights over
//                            the cached rows to A (H2O-style cumulative attention,
//                            Eq. 1), free the slot that ranks last under the
//                            (class, u, position) order; trailing workgroups of the same
//                            launch do B_i <- decay * B_i for every position
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
            uint4 kv = zero, vv = zero;                        // (a conditional expression on the structs goes through scratch memory)
            if (s < c) {
                kv = Kout[(size_t)unit * st.K * 16 + i];
                vv = Vout[(size_t)unit * st.K * 16 + i];
            }
            Kc[at] = kv;
            Vc[at] = vv;
        }
        return;
    }
    uint4* Kc = reinterpret_cast<uint4*>(st.Kc) + (size_t)unit * slots * 16;
    uint4* Vc = reinterpret_cast<uint4*>(st.Vc) + (size_t)unit * slots * 16;
    for (int i = threadIdx.x; i < slots * 16; i += DU_THREADS) {
        const int s = i >> 4;
        uint4 kv = zero, vv = zero;
        if (s < c) {
            kv = Kout[(size_t)unit * st.K * 16 + i];
            vv = Vout[(size_t)unit * st.K * 16 + i];
        }
        Kc[i] = kv;
        Vc[i] = vv;
    }
}

// ---- step, sequence part ---------------------------------------------------------
// Voucher and sponsor flag of every position from the current budgets (Eq. 2): the same for all
// units of a sequence, so it is computed once per sequence and step, not once per cached row.
struct VouchArgs {
    int32_t L;
    float pw[TA_MAX_SPAN + 1];
};

// Sequence part of a step, one launch: every workgroup reads the old length (nobody writes it here),
// the first wavefront of a sequence's first workgroup appends the token, tests the table at the new
// position and publishes the new length in `stepped` (0: the sequence is at capacity and is left
// alone); all workgroups compute the vouchers of their positions, which depend on earlier positions
// only and so not on anything the append writes.
__global__ void __launch_bounds__(256)
decode_seq_vouch_kernel(ta_decode_state st, const int32_t* new_tok, DecodeTable tab, VouchArgs a)
{
    const int b = blockIdx.y;
    const int32_t len_old = st.len[b];
    if (len_old < 0 || len_old >= st.cap) {
        if (blockIdx.x == 0 && threadIdx.x == 0) st.stepped[b] = 0;
        return;
    }
    const size_t row = (size_t)b * st.cap;
    if (blockIdx.x == 0 && threadIdx.x < 64) {
        const int32_t p = len_old;
        int32_t* tok = st.tok + row;
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
            st.anchor[row + p] = any ? 1 : 0;
            st.budget[row + p] = any ? tab.B : 0.0f;
            st.stepped[b] = (p + 1) | (any ? (1 << 30) : 0);   // new length; bit 30: the new token is an anchor
        }
    }
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p > len_old) return;                               // positions 0 .. len_old exist after the append
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
    // bit 0: sponsored; bit 1: the position is an anchor itself (the new position's flag travels in
    // `stepped`: it is being written by another workgroup of this launch)
    st.spons[row + p] = sp | (p < len_old && anchor[p] ? 2 : 0);
}

// Trailing workgroups of the unit launch: budget decay of 256 positions each, and the new length.
// Units read neither array (they take the length from `stepped`), so the two kinds of workgroup
// touch disjoint memory.
__device__ __forceinline__ void decay_rider(const ta_decode_state& st, int r, float decay)
{
    const int tiles = (st.cap + 255) >> 8;
    const int b = r / tiles, tile = r - b * tiles;
    const int32_t len_new = st.stepped[b] & 0x3FFFFFFF;
    if (len_new == 0) return;
    float* B = st.budget + (size_t)b * st.cap;
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int p = tile * 256 + j * 64 + (int)threadIdx.x;
        v[j] = B[p < len_new ? p : 0];                      // len_new >= 1
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int p = tile * 256 + j * 64 + (int)threadIdx.x;
        if (p < len_new) B[p] = __fmul_rn(decay, v[j]);
    }
    if (tile == 0 && threadIdx.x == 0) st.len[b] = len_new;
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
    int32_t units;                                         // workgroups beyond this many decay the budgets
    float decay;
};

__device__ __forceinline__ uint32_t ordered_bits(float u)
{
    uint32_t b = __float_as_uint(u);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

constexpr int SLOTS_PER_LANE = 5;                          // budgets up to 5 * 64 - 1 keep a lane's slots in registers

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

// ---- cross-lane reductions on the data-parallel-primitive path (no LDS round trips) ----------
// Steps: neighbours within quads, quads within a row of 16 by rotation, then the last lane of a row
// broadcast to the next row(s); lane 63 ends up with the reduction over the wavefront.
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}
#define TA_DPP_STEPS(STEP) STEP(0xb1) STEP(0x4e) STEP(0x124) STEP(0x128) STEP(0x142) STEP(0x143)

__device__ __forceinline__ float wave_max_dpp(float v)
{
#define STEP(C) v = fmaxf(v, __int_as_float(dpp_move<C>(__float_as_int(v))));
    TA_DPP_STEPS(STEP)
#undef STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_sum_dpp(float v)
{
#define STEP(C) v += __int_as_float(dpp_move<C>(__float_as_int(v)));
    TA_DPP_STEPS(STEP)
#undef STEP
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ int wave_sum_dpp(int v)
{
#define STEP(C) v += dpp_move<C>(v);
    TA_DPP_STEPS(STEP)
#undef STEP
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ int wave_min_dpp(int v)
{
#define STEP(C) { const int o = dpp_move<C>(v); v = o < v ? o : v; }
    TA_DPP_STEPS(STEP)
#undef STEP
    return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ unsigned long long wave_min_dpp(unsigned long long v)
{
#define STEP(C) { const unsigned lo = (unsigned)dpp_move<C>((int)(unsigned)v), hi = (unsigned)dpp_move<C>((int)(unsigned)(v >> 32)); \
                  const unsigned long long o = ((unsigned long long)hi << 32) | lo; v = o < v ? o : v; }
    TA_DPP_STEPS(STEP)
#undef STEP
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, 63);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), 63);
    return ((unsigned long long)hi << 32) | lo;
}

// One wavefront per unit, no workgroup barriers.  SMALL: at most SLOTS_PER_LANE * 64 slots, so a
// lane's slots (position, voucher, flags, accumulated attention) stay in its registers from the
// first round trip to the ranking and nothing loops over slots.
// DT_RING: 16-row key tiles in flight per wavefront.
// WAVES > 1 (few units with many slots: one wavefront per unit would leave most of the chip idle, stream its
// keys one tile after the other and loop over its slots): WAVES wavefronts share a unit.  Each keeps its
// SLOTS_PER_LANE * 64 slots in registers like the SMALL form and streams every WAVES-th key tile; the slot
// table, the logits and three small exchanges go through LDS (three workgroup barriers).  Every logit, every
// softmax statistic (each wavefront reduces all of them, in the single wavefront's order) and every slot's
// key is computed by the same instructions as in the single-wavefront form: the two give the same bits.
template <int GH, bool PAGED, bool SCORED, bool SMALL, int DT_RING, int WAVES>
__device__ __forceinline__ void decode_unit(const ta_decode_state& st, const UnitArgs& a, const SlotPages& pg)
{
    extern __shared__ float s_dyn[];
    static_assert(WAVES == 1 || (SCORED && SMALL), "several wavefronts: an attention term, slots in registers");

    const int lane = threadIdx.x & 63;
    const int wave = WAVES > 1 ? (int)(threadIdx.x >> 6) : 0;
    const int sub = lane & 15, grp = lane >> 4;            // 16 lanes per key row, 4 rows per instruction
    if ((int)blockIdx.x >= a.units) {                      // trailing workgroups: budget decay
        if (wave == 0) decay_rider(st, (int)blockIdx.x - a.units, a.decay);
        return;
    }
    const int unit = blockIdx.x;
    const int slots = st.K + 1;
    const int G = st.hq / st.hkv;
    const int g = unit % st.hkv;
    const int b = (unit / st.hkv) % st.batch;
    const int l = unit / (st.hkv * st.batch);
    int32_t* pos = st.pos + (size_t)unit * slots;
    float* A = st.A + (size_t)unit * slots;
    uint4* Kc = reinterpret_cast<uint4*>(st.Kc) + (PAGED ? l * pg.s_layer + g * pg.s_head : (int64_t)unit * slots * 16);
    uint4* Vc = reinterpret_cast<uint4*>(st.Vc) + (PAGED ? l * pg.s_layer + g * pg.s_head : (int64_t)unit * slots * 16);
    constexpr int SPL = SLOTS_PER_LANE;                            // slots per lane that one round trip covers
    const int sbase = wave * (SPL * 64);                           // first slot of this wavefront's share

    // Everything that does not depend on loaded data is requested first, in the order it is needed
    // (loads of a wavefront return in order), and unconditionally (clamped addresses, results masked
    // afterwards): straight-line loads let the compiler wait for exactly the load it needs.
    const int32_t stepped = st.stepped[b];                 // the sequence part of the step has run
    int32_t p0[SPL];
#pragma unroll
    for (int j = 0; j < SPL; ++j) {
        const int s = sbase + lane + 64 * j;
        p0[j] = SMALL ? pos[s < slots ? s : slots - 1] : 0;
    }
    const uint4* nsrc = ((lane & 16) ? a.v_new : a.k_new) + ((size_t)(l * st.batch + b) * st.hkv + g) * 16;
    const uint4 nrow = nsrc[lane & 15];                    // lanes 0-15: the new key row, 16-31: the new value row

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
    const int wstride = (slots + 3) & ~3;                  // logits of a head: padded to whole 16-byte groups
    // scored only: per wavefront one 16-row key tile (4 KB) and a copy of the new key row; with several
    // wavefronts 64 words for what they exchange; the logits
    uint4* s_t = reinterpret_cast<uint4*>(s_dyn + wstride) + 256 * wave;
    uint4* s_kn = reinterpret_cast<uint4*>(s_dyn + wstride) + 256 * WAVES + 16 * wave;
    int32_t* s_x = reinterpret_cast<int32_t*>(reinterpret_cast<uint4*>(s_dyn + wstride) + (256 + 16) * WAVES);
    float* s_w = reinterpret_cast<float*>(s_x) + (WAVES > 1 ? 64 : 0);

    const int i16 = sub, kq = grp;
    // this wavefront's tiles are wave, wave + WAVES, ...; `tile` below counts them, tile_of gives the unit's tile
    const int ntiles = (((slots + 15) >> 4) - wave + WAVES - 1) / WAVES;
    const auto tile_of = [&](int tile) { return wave + WAVES * tile; };
    uint4 qf[4], tiles[DT_RING][4];                        // DT_RING tiles in flight
    // Key rows are read once per step: the non-temporal hint keeps them from displacing the slot tables,
    // the accumulated attention and the per-sequence arrays in the caches (231 -> 210 us on 16 384 units).
    const auto load_tile = [&](int tile, uint4 (&dst)[4]) {
        if (!PAGED) {                                      // dense unit: one uniform base, a 32-bit byte offset per lane
            const char* base = reinterpret_cast<const char*>(Kc);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                int row = tile_of(tile) * 16 + 4 * t + grp;
                row = row < slots ? row : slots - 1;       // past the last slot: a valid row, masked at the store
                {
                    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
                    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + (uint32_t)(row * 256 + sub * 16)));
                    dst[t] = make_uint4(v.x, v.y, v.z, v.w);
                }
            }
            return;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            int row = tile_of(tile) * 16 + 4 * t + grp;
            row = row < slots ? row : slots - 1;
            typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(&Kc[row_at(row) + sub]));
            dst[t] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    if (SCORED) {
        const uint4* qrow = a.q_new + ((size_t)(l * st.batch + b) * st.hq + g * G + (i16 < G ? i16 : 0)) * 16;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint4 v = qrow[kq + 4 * t];
            qf[t] = i16 < G ? v : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < DT_RING; ++j) load_tile(j, tiles[j]);     // past the last tile: the last row again, never used
    }

    // ---- the slot table goes to LDS; lowest-numbered free slot ---------------------------------
    int first_free = 0x7FFFFFFF;
    if (SMALL) {
#pragma unroll
        for (int j = 0; j < SPL; ++j) {
            const int s = sbase + lane + 64 * j;
            if (s < slots) {
                s_pos[s] = p0[j];
                if (p0[j] < 0) first_free = first_free < s ? first_free : s;
            }
        }
    }
    for (int s0 = lane; !SMALL && s0 < slots; s0 += SPL * 64) {    // more slots than a lane's registers hold
        int32_t p4[SPL];
#pragma unroll
        for (int j = 0; j < SPL; ++j) {
            const int s = s0 + 64 * j;
            p4[j] = pos[s < slots ? s : slots - 1];
        }
#pragma unroll
        for (int j = 0; j < SPL; ++j) {
            const int s = s0 + 64 * j;
            if (s < slots) {
                s_pos[s] = p4[j];
                if (p4[j] < 0) first_free = first_free < s ? first_free : s;
            }
        }
    }
    int f = wave_min_dpp(first_free);
    if (WAVES > 1) {
        if (lane == 0) s_x[wave] = f;
        __syncthreads();                                   // every share of the slot table is in LDS
        f = s_x[0];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) f = s_x[w] < f ? s_x[w] : f;
    }
    const int32_t len_new = stepped & 0x3FFFFFFF;
    const uint8_t an_new = (uint8_t)((stepped >> 30) & 1);
    if (len_new == 0 || f >= slots) {                      // a sequence at capacity, or no room: nothing to do
        if (wave == 0 && lane == 0 && a.evicted) a.evicted[unit] = -1;
        return;                                            // (every wavefront of the unit: the same test)
    }
    const int32_t p_new = len_new - 1;

    // the per-position inputs of the utility and the accumulated attention of the first SPL * 64 slots
    // are requested now and used after the key stream: they travel while the keys do
    const size_t srow = (size_t)b * st.cap;
    const uint8_t* spons = st.spons + srow;               // bit 0: sponsored, bit 1: anchor
    const float* vouch = st.vouch + srow;
    float v0[SPL], a0[SPL];
    uint8_t fl0[SPL];
#pragma unroll
    for (int j = 0; SMALL && j < SPL; ++j) {
        const int s = sbase + lane + 64 * j;
        if (s == f) p0[j] = p_new;
        if (s >= slots) p0[j] = -2;
        const int32_t pc = p0[j] < 0 ? 0 : p0[j];
        v0[j] = vouch[pc];
        fl0[j] = spons[pc];
        if (SCORED) {
            const float av = A[s < slots ? s : slots - 1];
            a0[j] = (!a.last_query && p0[j] >= 0 && s != f) ? av : 0.0f;
        } else {
            a0[j] = 0.0f;
        }
    }
    if (lane < 16) {
        if (wave == 0) Kc[row_at(f) + lane] = nrow;
        if (SCORED) s_kn[lane] = nrow;
    } else if (lane < 32 && wave == 0) Vc[row_at(f) + lane - 16] = nrow;
    __builtin_amdgcn_wave_barrier();                       // the slot table is in LDS for every lane

    float m_h[GH], inv_h[GH];
    if (SCORED) {
        const auto frag_logits = [&](const uint4 (&frag)[4]) -> f32x4 {
            f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(lo_half(frag[t]), lo_half(qf[t]), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(hi_half(frag[t]), hi_half(qf[t]), acc, 0, 0, 0);
            }
            return acc;                                    // rows 4 kq .. 4 kq + 3 of the tile, head i16
        };
        // several wavefronts: the new key's logit goes into the free slot with the tile that holds it (every
        // row of this pseudo-tile is the new key, so every lane of a head gets that head's logit)
        float new_logit = 0.0f;
        if (WAVES > 1) {
            uint4 knf[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint4 v = s_kn[kq + 4 * t];
                knf[t] = make_uint4(v.x, v.y, v.z, v.w);
            }
            new_logit = frag_logits(knf)[0] * a.scale_log2;
        }
        const auto store_tile = [&](int tile, const f32x4& acc) {
            const int s = tile_of(tile) * 16 + 4 * kq;
            if (i16 < G && s < wstride) {
                const int4 p4 = *reinterpret_cast<const int4*>(&s_pos[s]);   // padded to whole groups of four
                float4 o;
                o.x = (s + 0 < slots && p4.x >= 0) ? acc[0] * a.scale_log2 : -INFINITY;
                o.y = (s + 1 < slots && p4.y >= 0) ? acc[1] * a.scale_log2 : -INFINITY;
                o.z = (s + 2 < slots && p4.z >= 0) ? acc[2] * a.scale_log2 : -INFINITY;
                o.w = (s + 3 < slots && p4.w >= 0) ? acc[3] * a.scale_log2 : -INFINITY;
                if (WAVES > 1) {
                    o.x = s + 0 == f ? new_logit : o.x;
                    o.y = s + 1 == f ? new_logit : o.y;
                    o.z = s + 2 == f ? new_logit : o.z;
                    o.w = s + 3 == f ? new_logit : o.w;
                }
                *reinterpret_cast<float4*>(&s_w[i16 * wstride + s]) = o;
            }
        };
        // One tile: its rows go to LDS as soon as they are there, which frees its registers for the
        // tile DT_RING further on; the fragments come back out of LDS in the matrix layout.
        const auto one_tile = [&](int tile, uint4 (&regs)[4], bool reload) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int r = 4 * t + grp;
                s_t[r * 16 + (sub ^ r)] = make_uint4(regs[t].x, regs[t].y, regs[t].z, regs[t].w);
            }
            if (reload) load_tile(tile + DT_RING, regs);
            uint4 frag[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint4 v = s_t[i16 * 16 + ((kq + 4 * t) ^ i16)];
                frag[t] = make_uint4(v.x, v.y, v.z, v.w);
            }
            store_tile(tile, frag_logits(frag));
        };
        // Passes of DT_RING tiles.  While every tile of a pass has a successor DT_RING further on, the
        // pass is straight-line code (first pass apart from the loop: other loads are still in flight
        // around it); the last one or two passes test every tile.
        int tb = 0;
        if (2 * DT_RING <= ntiles) {
#pragma unroll
            for (int j = 0; j < DT_RING; ++j) one_tile(j, tiles[j], true);
            for (tb = DT_RING; tb + 2 * DT_RING <= ntiles; tb += DT_RING) {
#pragma unroll
                for (int j = 0; j < DT_RING; ++j) one_tile(tb + j, tiles[j], true);
            }
        }
        for (; tb < ntiles; tb += DT_RING) {
#pragma unroll
            for (int j = 0; j < DT_RING; ++j)
                if (tb + j < ntiles) one_tile(tb + j, tiles[j], tb + j + DT_RING < ntiles);
        }
        if (WAVES > 1) {
            __syncthreads();                               // the logits of every wavefront's tiles are in LDS
        } else {
            uint4 knf[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {                                  // every row of this tile is the new key
                const uint4 v = s_kn[kq + 4 * t];
                knf[t] = make_uint4(v.x, v.y, v.z, v.w);
            }
            const f32x4 acc = frag_logits(knf);
            __builtin_amdgcn_wave_barrier();
            if (i16 < G && kq == 0) s_w[i16 * wstride + f] = acc[0] * a.scale_log2;
            __builtin_amdgcn_wave_barrier();
        }
        // softmax statistics of all heads at once: one pass for the maxima, one for the sums.  Several
        // wavefronts: each takes every WAVES-th head (a head's reduction runs in one wavefront, in the
        // single wavefront's order) and the results are exchanged through LDS.
        const auto mine = [&](int h) { return h < G && (WAVES == 1 || h % WAVES == wave); };
#pragma unroll
        for (int h = 0; h < GH; ++h) m_h[h] = -INFINITY;
        for (int s = lane; s < slots; s += 64) {
#pragma unroll
            for (int h = 0; h < GH; ++h)
                if (mine(h)) m_h[h] = fmaxf(m_h[h], s_w[h * wstride + s]);
        }
#pragma unroll
        for (int h = 0; h < GH; ++h)
            if (mine(h)) m_h[h] = wave_max_dpp(m_h[h]);
        float z_h[GH];
#pragma unroll
        for (int h = 0; h < GH; ++h) z_h[h] = 0.0f;
        for (int s = lane; s < slots; s += 64) {
#pragma unroll
            for (int h = 0; h < GH; ++h)
                if (mine(h)) z_h[h] += __builtin_amdgcn_exp2f(s_w[h * wstride + s] - m_h[h]);
        }
#pragma unroll
        for (int h = 0; h < GH; ++h) inv_h[h] = mine(h) ? __builtin_amdgcn_rcpf(wave_sum_dpp(z_h[h])) : 0.0f;
        if (WAVES > 1) {
            static_assert(WAVES == 1 || GH <= 16, "the exchange area holds 16 heads");
            float* s_stat = reinterpret_cast<float*>(s_x) + 32;            // [0..16): maxima, [16..32): reciprocal sums
            if (lane == 0) {
#pragma unroll
                for (int h = 0; h < GH; ++h) {
                    if (mine(h)) {
                        s_stat[h] = m_h[h];
                        s_stat[16 + h] = inv_h[h];
                    }
                }
            }
            __syncthreads();                               // every head's statistics
#pragma unroll
            for (int h = 0; h < GH; ++h) {
                m_h[h] = h < G ? s_stat[h] : -INFINITY;
                inv_h[h] = h < G ? s_stat[16 + h] : 0.0f;
            }
        }
    }

    // ---- new attention mass per slot, then the rank of the slot, in one pass (a lane handles the
    // same slots in both, so the mass stays in a register)
    const float lenf = (float)len_new;
    unsigned long long worst = ~0ull;
    int nfree = 0;
    const auto rank_slot = [&](int s, int32_t p, float v, uint8_t fl, float a_old) {
        const uint8_t sp = fl & 1, an = (s == f) ? an_new : (uint8_t)((fl >> 1) & 1);
        if (p == -2) return;                               // past the last slot
        if (p < 0) { ++nfree; return; }
        float mass = 0.0f;
        if (SCORED) {
            float add = 0.0f;
#pragma unroll
            for (int h = 0; h < GH; ++h)
                if (h < G) add += __builtin_amdgcn_exp2f(s_w[h * wstride + s] - m_h[h]) * inv_h[h];
            // cumulative mass over the steps, or (TOVA's step-wise rule) this step's mass alone
            mass = a_old + add;
            A[s] = mass;
        } else if (s == f) {
            A[s] = 0.0f;
        }
        const float r = __fdiv_rn((float)(p + 1), lenf);
        float t = SCORED ? __fmul_rn(a.alpha, mass) : 0.0f;
        t = __fadd_rn(t, __fmul_rn(a.beta, r));
        t = __fadd_rn(t, __fmul_rn(a.gamma, (float)an));
        t = __fadd_rn(t, v);
        const unsigned cls = (p < a.n_sink || p >= len_new - a.n_recent) ? 2u : (sp ? 1u : 0u);
        // (class, u, position) packed so that the smallest integer ranks last
        const unsigned long long key = ((unsigned long long)cls << 62) |
                                       ((unsigned long long)ordered_bits(t) << 30) | (unsigned long long)(uint32_t)p;
        worst = key < worst ? key : worst;
    };
#pragma unroll
    for (int j = 0; SMALL && j < SPL; ++j) rank_slot(sbase + lane + 64 * j, p0[j], v0[j], fl0[j], a0[j]);
    for (int s0 = lane; !SMALL && s0 < slots; s0 += SPL * 64) {    // more slots than a lane's registers hold
        int32_t p4[SPL];
        float v4[SPL], a4[SPL];
        uint8_t fl4[SPL];
#pragma unroll
        for (int j = 0; j < SPL; ++j) {
            const int s = s0 + 64 * j;
            p4[j] = s < slots ? ((s == f) ? p_new : s_pos[s]) : -2;
            const int32_t pc = p4[j] < 0 ? 0 : p4[j];
            v4[j] = vouch[pc];
            fl4[j] = spons[pc];
            if (SCORED) {
                const float av = A[s < slots ? s : slots - 1];
                a4[j] = (!a.last_query && p4[j] >= 0 && s != f) ? av : 0.0f;
            } else {
                a4[j] = 0.0f;
            }
        }
#pragma unroll
        for (int j = 0; j < SPL; ++j) rank_slot(s0 + 64 * j, p4[j], v4[j], fl4[j], a4[j]);
    }
    nfree = wave_sum_dpp(nfree);
    worst = wave_min_dpp(worst);
    if (WAVES > 1) {
        if (lane == 0) {
            s_x[8 + wave] = nfree;
            s_x[16 + 2 * wave] = (int32_t)(uint32_t)worst;
            s_x[17 + 2 * wave] = (int32_t)(uint32_t)(worst >> 32);
        }
        __syncthreads();                                   // every wavefront's free count and worst key
        nfree = 0;
        worst = ~0ull;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            nfree += s_x[8 + w];
            const unsigned long long k = ((unsigned long long)(uint32_t)s_x[17 + 2 * w] << 32) | (uint32_t)s_x[16 + 2 * w];
            worst = k < worst ? k : worst;
        }
    }
    const int32_t evict_pos = nfree > 0 ? -1 : (int32_t)(worst & 0x3FFFFFFFull);
    const int s_end = (WAVES > 1 && sbase + SPL * 64 < slots) ? sbase + SPL * 64 : slots;   // a wavefront updates its own share
    for (int s = sbase + lane; s < s_end; s += 64) {
        const int32_t p = (s == f) ? p_new : s_pos[s];
        if (s == f || (p >= 0 && p == evict_pos)) pos[s] = (p == evict_pos) ? -1 : p;
    }
    if (wave == 0 && lane == 0 && a.evicted) a.evicted[unit] = evict_pos;
}

// Dense slots: three tiles in flight at four wavefronts per SIMD (124 registers).  Paged slots need
// more registers for their addresses: four tiles in flight at three wavefronts per SIMD instead of
// spilling.  The same number of key bytes is in flight per SIMD either way.
template <int GH, bool SCORED, bool SMALL>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(4)))
decode_unit_kernel(ta_decode_state st, UnitArgs a, SlotPages pg)
{
    decode_unit<GH, false, SCORED, SMALL, 3, 1>(st, a, pg);
}

template <int GH, bool SCORED, bool SMALL>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(3)))
decode_unit_paged_kernel(ta_decode_state st, UnitArgs a, SlotPages pg)
{
    decode_unit<GH, true, SCORED, SMALL, 4, 1>(st, a, pg);
}

// More slots than one wavefront's registers hold: four wavefronts per unit (up to 1280 slots) or eight (up to 2560),
// each with SLOTS_PER_LANE * 64 of the slots.  Six key tiles in flight per wavefront (seven with paged slots) in two
// wavefronts' worth of registers per SIMD.
constexpr int DU_WIDE = 4;
constexpr int DU_WIDER = 8;
constexpr int DU_WIDE_RING = 6;
// When: measured against one wavefront per unit on 32 x batch x 8 units.  From about 700 slots on the shared form is
// ahead at every unit count (1025 slots: 24 against 44 us per step at 256 units, 198 against 220 us at 4096, 386
// against 412 us at 8192 - the single wavefront has to loop over its slots there); below that it is ahead up to
// about 640 units (513 slots: 18 against 27 us at 256 units, level at 768, behind from 1024 on).
#ifndef TA_DECODE_WIDE_MAX_UNITS
#define TA_DECODE_WIDE_MAX_UNITS 640
#endif
constexpr int DU_WIDE_MAX_UNITS = TA_DECODE_WIDE_MAX_UNITS;   // (0: never)
constexpr int DU_WIDE_ALWAYS_SLOTS = 704;
// Eight wavefronts (1281 to 2560 slots): 2048 slots: 37 against 74 us at 256 units, 140 against 173 us at 1024, 509
// against 538 us at 4096; 1501 slots: 32 against 57 us at 256 units, but 207 against 183 us at 2048.
constexpr int DU_WIDER_MAX_UNITS = 1024;
constexpr int DU_WIDER_ALWAYS_SLOTS = 1792;

template <int GH, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(2)))
decode_unit_wide_kernel(ta_decode_state st, UnitArgs a, SlotPages pg)
{
    decode_unit<GH, false, true, true, DU_WIDE_RING, WAVES>(st, a, pg);
}

template <int GH, int WAVES>
__global__ void __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(2)))
decode_unit_paged_wide_kernel(ta_decode_state st, UnitArgs a, SlotPages pg)
{
    decode_unit<GH, true, true, true, DU_WIDE_RING + 1, WAVES>(st, a, pg);
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
    // dynamic LDS above 64 KB (large budgets with an attention term) needs the attribute
    const void* fns[] = {reinterpret_cast<const void*>(&decode_unit_kernel<GH, true, true>),
                         reinterpret_cast<const void*>(&decode_unit_kernel<GH, true, false>),
                         reinterpret_cast<const void*>(&decode_unit_paged_kernel<GH, true, true>),
                         reinterpret_cast<const void*>(&decode_unit_paged_kernel<GH, true, false>),
                         reinterpret_cast<const void*>(&decode_unit_wide_kernel<GH, DU_WIDE>),
                         reinterpret_cast<const void*>(&decode_unit_paged_wide_kernel<GH, DU_WIDE>),
                         reinterpret_cast<const void*>(&decode_unit_wide_kernel<GH, DU_WIDER>),
                         reinterpret_cast<const void*>(&decode_unit_paged_wide_kernel<GH, DU_WIDER>)};
    hipError_t e = hipSuccess;
    for (const void* fn : fns)
        if (e == hipSuccess) e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return e;
}

template <int GH>
void launch_unit(const ta_decode_state& st, const UnitArgs& a, const SlotPages& pg, unsigned grid, size_t lds, int waves,
                 hipStream_t s)
{
    const bool scored = a.alpha != 0.0f, small = st.K + 1 <= SLOTS_PER_LANE * 64;
    if (waves > 1) {                                       // several wavefronts per unit
        auto kernel = st.pages ? (waves == DU_WIDE ? decode_unit_paged_wide_kernel<GH, DU_WIDE> : decode_unit_paged_wide_kernel<GH, DU_WIDER>)
                               : (waves == DU_WIDE ? decode_unit_wide_kernel<GH, DU_WIDE> : decode_unit_wide_kernel<GH, DU_WIDER>);
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(64 * waves), lds, s, st, a, pg);
        return;
    }
#define TA_LAUNCH_UNIT(KERNEL, S, M) \
    hipLaunchKernelGGL((KERNEL<GH, S, M>), dim3(grid), dim3(64), lds, s, st, a, pg)
    if (st.pages) {
        if (scored) { if (small) TA_LAUNCH_UNIT(decode_unit_paged_kernel, true, true); else TA_LAUNCH_UNIT(decode_unit_paged_kernel, true, false); }
        else { if (small) TA_LAUNCH_UNIT(decode_unit_paged_kernel, false, true); else TA_LAUNCH_UNIT(decode_unit_paged_kernel, false, false); }
    } else {
        if (scored) { if (small) TA_LAUNCH_UNIT(decode_unit_kernel, true, true); else TA_LAUNCH_UNIT(decode_unit_kernel, true, false); }
        else { if (small) TA_LAUNCH_UNIT(decode_unit_kernel, false, true); else TA_LAUNCH_UNIT(decode_unit_kernel, false, false); }
    }
#undef TA_LAUNCH_UNIT
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
    VouchArgs va;
    va.L = prm.span_L;
    for (int k = 0; k <= TA_MAX_SPAN; ++k) va.pw[k] = tab.pw[k];
    const unsigned tiles = (unsigned)((st.cap + 255) / 256);            // 256 positions per workgroup
    hipLaunchKernelGGL(decode_seq_vouch_kernel, dim3(tiles, (unsigned)st.batch), dim3(256), 0, s, st, new_tok, dt, va);

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
    // slot table; with an attention term also one key tile, the new key row and the logits
    const size_t wstride = (size_t)((slots + 3) & ~3);
    const SlotPages pg = slot_pages(st);
    const size_t page_list = st.pages ? (size_t)((slots - 1) / pg.page_size + 1) : 0;      // the pages of the unit's slots
    // per wavefront a key tile and the new key row; several wavefronts: 64 words more
    const auto scored_floats = [&](int waves) { return wstride + (1024 + 64) * (size_t)waves + (waves > 1 ? 64 : 0) + (size_t)G * wstride; };
    // several wavefronts per unit when the slots do not fit one wavefront's registers (but do fit those of four or
    // eight) and either are many or the units are few
    int waves = 1;
    if (prm.alpha != 0.0f && slots > SLOTS_PER_LANE * 64 && DU_WIDE_MAX_UNITS > 0) {
        if (slots <= DU_WIDE * SLOTS_PER_LANE * 64) {
            if (units <= (unsigned)DU_WIDE_MAX_UNITS || slots > DU_WIDE_ALWAYS_SLOTS) waves = DU_WIDE;
        } else if (slots <= DU_WIDER * SLOTS_PER_LANE * 64) {
            if (units <= (unsigned)DU_WIDER_MAX_UNITS || slots > DU_WIDER_ALWAYS_SLOTS) waves = DU_WIDER;
        }
    }
    if (waves > 1 && (scored_floats(waves) + page_list) * sizeof(float) > 160 * 1024) waves = 1;
    size_t lds_floats = prm.alpha != 0.0f ? scored_floats(waves) : wstride;
    a.pg_off = (int32_t)lds_floats;
    a.units = (int32_t)units;
    a.decay = prm.budget_decay;
    lds_floats += page_list;
    const size_t lds = lds_floats * sizeof(float);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    const hipError_t attr_err = decode_setup();
    if (attr_err != hipSuccess) return attr_err;
    // the units, then one workgroup per 256 positions for the budget decay
    const uint64_t grid = (uint64_t)units + (uint64_t)tiles * (uint64_t)st.batch;
    if (grid > 0x7FFFFFFFull) return hipErrorInvalidValue;
    if (G <= 4) launch_unit<4>(st, a, pg, (unsigned)grid, lds, waves, s);
    else if (G <= 8) launch_unit<8>(st, a, pg, (unsigned)grid, lds, waves, s);
    else launch_unit<MAX_GROUP>(st, a, pg, (unsigned)grid, lds, waves, s);
    return hipGetLastError();
}

}  // namespace ta
