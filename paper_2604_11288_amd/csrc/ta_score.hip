// Step 3 of the eviction pass: the attention term A_i of Eq. 1 as column sums
// of the observation window's softmax (cumulative attention over heads and
// steps, App. A dormant-token definition; SnapKV/H2O-style scoring, Sec. 2).
//
// Per unit (layer, sequence, KV head): S = Q K^T with M = G*W query rows
// (G query heads of the group x W window rows), d = 128, n keys; row softmax
// over the visible keys; A[i] = sum over rows of the softmax column i.
//
// Column sums need every row's (max, normaliser) over ALL keys before any row
// can be added into a column, so the keys are swept twice:
//   sweep 1 (stats)  : per row, online (m, Z) over a chunk of keys -> workspace
//   sweep 2 (colsum) : merge the chunk statistics of a row into one constant
//                      c_r = m_r + log2 Z_r, recompute S, p = 2^(s - c_r),
//                      sum p over the rows -> A
// Both sweeps are one kernel template.  A workgroup owns one chunk of keys of
// one unit and streams it through LDS in 64-key stages: a ring of four 16 KB
// buffers filled by direct global->LDS loads issued three stages ahead (no
// staging registers), 16-byte chunks XOR-swizzled by row so that the
// ds_read_b128 fragment loads are conflict free.  Blocks are numbered so that
// all chunks of a unit run on one XCD (block b lands on XCD b mod 8): the
// unit's Q rows and chunk statistics are then fetched into one L2 only.  The M rows are split
// into RG groups of 64; the workgroup has 2*RG wavefronts, wavefront (rg, kt)
// owns row group rg (its Q fragments stay in 64 registers for the whole chunk)
// and the kt-th 32-key tile of every stage, so one K fragment read from LDS
// feeds two MFMA row tiles.
// The contraction runs on v_mfma_f32_32x32x16_bf16:
//   sweep 1 computes K Q^T (keys x rows): a lane then holds 16 keys of ONE
//           query row, so (m, Z) are two registers per row tile and need no
//           cross-lane traffic until the end of the chunk;
//   sweep 2 computes Q K^T (rows x keys): a lane holds 16 rows of ONE key, so
//           the column sum is a register accumulation plus one half-wave swap.
#include <math.h>

#include <atomic>
#include <type_traits>

#include "ta_match_device.h"
#include "ta_score_common.h"

namespace ta {

namespace {

constexpr int STAGE_KEYS = 64;
constexpr int STAGE_UNITS = STAGE_KEYS * 16;     // 16-byte units per stage (256 B per key)
// Stage buffers per workgroup; loads run that many minus one stages ahead.  (Eight buffers for
// the wider workgroups, which have a compute unit to themselves, were measured: no gain.)
constexpr int ring_of(int) { return 4; }
// the widest workgroup: 64 * MAX_RG rows at a time (more row groups leave too few registers per lane)
constexpr int MAX_RG = 4;

// Direct global->LDS load of 16 bytes per lane: lane i reads 16 bytes at base + off (base
// wave-uniform, off per lane) and its data lands at lds_base + 16*i (lds_base wave-uniform,
// passed in M0).  Written as inline assembly on purpose: the compiler would otherwise make
// every later LDS read wait for ALL outstanding direct loads, which would serialise the stage
// pipeline; the waits for these loads are explicit below.  Extra outstanding loads only make
// the compiler's own vmcnt waits more conservative.
__device__ __forceinline__ void load_to_lds_16(const void* base, uint32_t off, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(off), "s"(base)
                 : "memory", "m0");
}

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding)
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

// A sweep that also carries the match tiles: workgroups past the score grid each run one tile
// of the anchor match (they start as the first score workgroups retire).  The statistics sweep
// carries them in the two-sweep step, the column-sum sweep when the normalisers are given.
struct RiderArgs {
    MatchArgs m;
    MatchTable tab;
    uint32_t score_blocks;
};

// RG row groups of RT 32-row MFMA tiles each per workgroup; 2 * RG wavefronts.
// row_base: first of the 64 * RG rows this call works on (units with more rows take several calls)
template <int RG, int RT, bool COLSUM, bool PAGED>
__device__ __forceinline__ void score_body(const ScoreArgs& a, uint4 (*s_k)[STAGE_UNITS], int32_t row_base);

// one tile per wavefront: four wavefronts per SIMD (at most 128 registers each)
template <int RG, int RT, bool COLSUM, bool PAGED>
__global__ void __launch_bounds__(128 * RG, RT == 1 ? 4 : 2)
score_kernel(ScoreArgs a)
{
    __shared__ uint4 s_k[ring_of(RG)][STAGE_UNITS];        // 16 KB per stage
    // a workgroup holds 64 * RG rows at a time; a unit with more rows is done in passes over its chunk
    // (the keys of the later passes come from the L2; their column sums are added to the first pass's)
    if constexpr (RG < MAX_RG) {
        score_body<RG, RT, COLSUM, PAGED>(a, s_k, 0);      // these kernels only get units that fit one pass
    } else {
        for (int32_t row_base = 0; row_base < a.rows_pad; row_base += 64 * RG) {
            if (row_base > 0) __syncthreads();             // the previous pass is done with the LDS
            score_body<RG, RT, COLSUM, PAGED>(a, s_k, row_base);
        }
    }
}

template <int RG, int RT, bool COLSUM>
__global__ void __launch_bounds__(128 * RG, RT == 1 ? 4 : 2)
score_match_kernel(ScoreArgs a, RiderArgs r)
{
    __shared__ uint4 s_k[ring_of(RG)][STAGE_UNITS];
    static_assert(sizeof(MatchLds) <= sizeof(uint4) * ring_of(RG) * STAGE_UNITS, "match tile must fit the stage ring");
    if (blockIdx.x >= r.score_blocks) {
        if (threadIdx.x >= MATCH_THREADS) return;          // a tile is the work of four wavefronts
        const uint32_t t = blockIdx.x - r.score_blocks;
        match_expand_tile(r.m, r.tab, (int32_t)(t % (uint32_t)r.m.tiles), (int32_t)(t / (uint32_t)r.m.tiles),
                          (int)threadIdx.x, *reinterpret_cast<MatchLds*>(&s_k[0][0]));
        return;
    }
    if constexpr (RG < MAX_RG) {
        score_body<RG, RT, COLSUM, false>(a, s_k, 0);
    } else {
        for (int32_t row_base = 0; row_base < a.rows_pad; row_base += 64 * RG) {
            if (row_base > 0) __syncthreads();
            score_body<RG, RT, COLSUM, false>(a, s_k, row_base);
        }
    }
}

template <int RG, int RT, bool COLSUM, bool PAGED>
__device__ __forceinline__ void score_body(const ScoreArgs& a, uint4 (*s_k)[STAGE_UNITS], const int32_t row_base)
{
    constexpr int ROW_TILES = RT;
    constexpr int GROUP_ROWS = 32 * RT;                    // rows of one wavefront
    constexpr int THREADS = 128 * RG;
    constexpr int WAVES = 2 * RG;
    constexpr int LPS = 16 / WAVES;                        // 1 KB direct loads per wavefront per stage
    static_assert(LPS >= 1, "unsupported row-group count");
    constexpr int RING = ring_of(RG);
    // waits until the loads of at most k later stages are outstanding (loads complete in issue order)
    const auto wait_but = [](int k) {
        static_assert(RING - 2 <= 6, "cases below");
        switch (k) {
            case 0: __builtin_amdgcn_s_waitcnt(vmcnt_imm(0)); break;
            case 1: __builtin_amdgcn_s_waitcnt(vmcnt_imm(LPS)); break;
            case 2: __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * LPS)); break;
            case 3: __builtin_amdgcn_s_waitcnt(vmcnt_imm(3 * LPS)); break;
            case 4: __builtin_amdgcn_s_waitcnt(vmcnt_imm(4 * LPS)); break;
            case 5: __builtin_amdgcn_s_waitcnt(vmcnt_imm(5 * LPS)); break;
            default: __builtin_amdgcn_s_waitcnt(vmcnt_imm(6 * LPS)); break;
        }
    };

    __shared__ float s_c[COLSUM ? GROUP_ROWS * RG : 1];            // per-row constant m + log2 Z
    __shared__ int32_t s_lim[COLSUM ? GROUP_ROWS * RG : 1];        // per-row last visible key
    __shared__ float s_part[COLSUM ? 2 : 1][RG][STAGE_KEYS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c32 = lane & 31, hf = lane >> 5;
    const int rg = wave % RG, kt = wave / RG;              // row group, key tile of the stage

    // XCD x = block % 8 runs the units [x * units_per_xcd, (x+1) * units_per_xcd)
    const int32_t seq_in_xcd = (int32_t)(blockIdx.x >> 3);
    const int32_t unit_in_xcd = seq_in_xcd / a.nchunks;
    const int32_t chunk = seq_in_xcd - unit_in_xcd * a.nchunks;
    const int32_t unit = (int32_t)(blockIdx.x & 7u) * a.units_per_xcd + unit_in_xcd;
    if (unit >= a.units) return;
    const int32_t g = unit % a.hkv;
    const int32_t b = (unit / a.hkv) % a.batch;
    const int32_t l = unit / (a.hkv * a.batch);
    const int32_t n = a.n, W = a.W;
    int32_t nb = a.seq_len ? a.seq_len[b] : n;
    nb = nb < 0 ? 0 : (nb > n ? n : nb);

    const int32_t key_lo = chunk * a.chunk_keys;
    int32_t key_hi = key_lo + a.chunk_keys;
    key_hi = key_hi > n ? n : key_hi;
    // keys at or past the end of a ragged sequence are visible to no row: their stages are not
    // streamed at all (their column sums are written as zeros at the end)
    const int32_t key_end = key_hi < nb ? key_hi : nb;
    const int nstages = key_end > key_lo ? (key_end - key_lo + STAGE_KEYS - 1) / STAGE_KEYS : 0;
    // keys <= min_lim are visible to every live row of a full window
    const int32_t min_lim = a.causal ? nb - W : nb - 1;

    if (key_lo >= nb) {
        // the whole chunk lies past the end of this sequence: nothing is visible
        if constexpr (!COLSUM) {
            float* st = a.ws + (((size_t)unit * a.nchunks + chunk) * a.rows_pad) * 2;
            for (int r = tid; r < a.rows_pad; r += THREADS) {
                st[r * 2] = -INFINITY;
                st[r * 2 + 1] = 0.0f;
            }
        } else {
            for (int32_t key = key_lo + tid; key < key_hi; key += THREADS) a.A[(size_t)unit * n + key] = 0.0f;
        }
        return;
    }

    // Stages whose keys are all visible to every row, [0, nfast), are visited in rotated
    // order, starting at a stage that differs from block to block.  Chunks start at
    // multiples of a large power of two, so blocks that advance in step would otherwise
    // all read the same offset within their chunk at the same time and crowd a few
    // memory channels.
    int nfast = min_lim >= key_lo + STAGE_KEYS - 1 ? (min_lim - key_lo + 1) / STAGE_KEYS : 0;
    nfast = nfast > nstages ? nstages : nfast;
    const int rot = nfast > 1 ? (int)((seq_in_xcd + 5 * (int32_t)(blockIdx.x & 7u)) % nfast) : 0;
    // The column-sum sweep visits them in the reverse order of the statistics sweep: what
    // that sweep read last is the likeliest to still sit in the last-level cache.
    const auto stage_pos = [&](int s) {
        if (s >= nfast) return s;
        const int p = (COLSUM ? nfast - 1 - s : s) + rot;
        return p >= nfast ? p - nfast : p;
    };

    // ---- K staging: direct global->LDS loads, 1 KB (4 key rows) per wavefront instruction.
    // Lane i of a load lands at (buffer + block*1 KB + 16*i): LDS slot row*16 + c' receives the
    // 16-byte chunk c' ^ (row & 15) of key row `row`.
    // The byte offset of a lane's 16 bytes inside a stage does not depend on the stage, so a
    // stage costs one scalar base address and no vector arithmetic (except the ragged last one).
    // Paged K: the keys of a stage (64 positions, page_size is a multiple of 64) lie in one page; lane j
    // keeps the page of the j-th page slot of this chunk, so a stage costs a lane read, not a load.
    const uint4* kbase = (a.Kl ? uniform_global_ptr(a.Kl[l]) : a.K + l * a.k_sl) + (PAGED ? 0 : b * a.k_sb) + g * a.k_sh;
    const auto slot_of = [&](int32_t key) { return a.page_shift >= 0 ? key >> a.page_shift : key / a.page_size; };
    const int32_t slot_lo = PAGED ? slot_of(key_lo) : 0;
    int32_t my_page = 0;
    if constexpr (PAGED) {
        const int32_t slot = slot_lo + lane;
        if (slot < a.max_pages) my_page = a.table[(size_t)b * a.max_pages + slot];
        my_page = my_page < 0 ? 0 : (my_page >= a.num_pages ? a.num_pages - 1 : my_page);
    }
    const auto stage_base = [&](int32_t key0) -> const uint4* {
        if constexpr (!PAGED) return kbase + (int64_t)key0 * a.k_sp;
        const int32_t slot = slot_of(key0);
        const int32_t rel = __builtin_amdgcn_readfirstlane(slot - slot_lo);
        int32_t page;
        if (rel < 64) page = __builtin_amdgcn_readlane(my_page, rel);
        else {                                             // chunks longer than 64 pages: read the table
            page = a.table[(size_t)b * a.max_pages + slot];
            page = page < 0 ? 0 : (page >= a.num_pages ? a.num_pages - 1 : page);
        }
        return kbase + (int64_t)page * a.k_spage + (int64_t)(key0 - slot * a.page_size) * a.k_sp;
    };
    const uint32_t lds_ring = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint4*)&s_k[0][0];
    const uint32_t lds_wave = lds_ring + 1024u * (uint32_t)__builtin_amdgcn_readfirstlane(wave);
    uint32_t lane_off[LPS];
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int row = (wave + WAVES * j) * 4 + (lane >> 4);
        lane_off[j] = (uint32_t)(row * a.k_sp + ((lane & 15) ^ (row & 15))) * 16u;
    }
    auto stage_issue = [&](int s) {
        const int32_t key0 = key_lo + stage_pos(s) * STAGE_KEYS;
        const uint4* sbase = stage_base(key0);
        const uint32_t dst = lds_wave + (uint32_t)(s % RING) * (STAGE_UNITS * 16u);
        if (key0 + STAGE_KEYS <= n) {
#pragma unroll
            for (int j = 0; j < LPS; ++j) load_to_lds_16(sbase, lane_off[j], dst + WAVES * j * 1024u);
        } else {
#pragma unroll
            for (int j = 0; j < LPS; ++j) {
                const int row = (wave + WAVES * j) * 4 + (lane >> 4);
                const int32_t last = n - 1 - key0;         // stay inside the tensor; masked later
                const int32_t rclamp = row > last ? last : row;
                const uint32_t off = (uint32_t)(rclamp * a.k_sp + ((lane & 15) ^ (row & 15))) * 16u;
                load_to_lds_16(sbase, off, dst + WAVES * j * 1024u);
            }
        }
    };
    // ---- Q fragments of this wavefront's 64 rows (registers, whole chunk) -----------
    const uint4* qlayer = a.Ql ? uniform_global_ptr(a.Ql[l]) : a.Q + l * a.q_sl;
    bf16x8 qf[ROW_TILES][8];
    int32_t my_lim[ROW_TILES];                             // sweep 1: last visible key of this lane's row
#pragma unroll
    for (int t = 0; t < ROW_TILES; ++t) {
        const int32_t r = row_base + GROUP_ROWS * rg + 32 * t + c32;
        int32_t lim = -1;
        if (r < a.rows) {
            const int32_t h = r / W, w = r - h * W;
            const uint4* qrow = qlayer + b * a.q_sb + (int64_t)(g * a.G + h) * a.q_sh + (int64_t)w * 16;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) qf[t][ks] = as_frag(qrow[2 * ks + hf]);
            lim = a.causal ? nb - W + w : nb - 1;
        } else {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) qf[t][ks] = as_frag(make_uint4(0, 0, 0, 0));
        }
        my_lim[t] = lim;
    }
    // ---- sweep 2: merge the chunk statistics of a row into its constant (before any direct
    // load is issued: these are ordinary loads, and waiting for them later would also wait for
    // every direct load issued in between).  Chunks are added in index order, four loads in flight.
    if constexpr (COLSUM) {
        for (int lr = tid; lr < GROUP_ROWS * RG; lr += THREADS) {
            const int32_t r = row_base + lr;
            float c = INFINITY;
            int32_t lim = -1;
            if (r < a.rows && a.lse) {
                // the row's normaliser comes from the prefill attention kernel: c = lse * log2(e)
                const int32_t h = r / W, w = r - h * W;
                const float v = a.lse[(((size_t)l * a.batch + b) * ((size_t)a.hkv * a.G) + (size_t)(g * a.G + h)) * W + w];
                if (v > -INFINITY) c = v * 1.4426950408889634f;
                lim = a.causal ? nb - W + w : nb - 1;
            } else if (r < a.rows) {
                const float2* st = reinterpret_cast<const float2*>(a.ws) + ((size_t)unit * a.nchunks * a.rows_pad + r);
                const size_t step = (size_t)a.rows_pad;
                const int last_ch = a.nchunks - 1;
                float2 first[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) first[j] = st[(size_t)(j < last_ch ? j : last_ch) * step];
                float mstar = first[0].x;
#pragma unroll
                for (int j = 1; j < 4; ++j) mstar = fmaxf(mstar, first[j].x);
                for (int ch0 = 4; ch0 < a.nchunks; ch0 += 4) {
                    float2 more[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) more[j] = st[(size_t)(ch0 + j < last_ch ? ch0 + j : last_ch) * step];
#pragma unroll
                    for (int j = 0; j < 4; ++j) mstar = fmaxf(mstar, more[j].x);
                }
                float Z = 0.0f;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (j <= last_ch && first[j].y > 0.0f) Z += first[j].y * fast_exp2(first[j].x - mstar);
                for (int ch0 = 4; ch0 < a.nchunks; ch0 += 4) {
                    float2 more[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) more[j] = st[(size_t)(ch0 + j < last_ch ? ch0 + j : last_ch) * step];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (ch0 + j <= last_ch && more[j].y > 0.0f) Z += more[j].y * fast_exp2(more[j].x - mstar);
                }
                if (Z > 0.0f) c = mstar + log2f(Z);
                const int32_t h = r / W, w = r - h * W;
                lim = a.causal ? nb - W + w : nb - 1;
            }
            s_c[lr] = c;
            s_lim[lr] = lim;
        }
    }

    // The compiler waits for ordinary loads with a count that knows nothing of the direct loads
    // below: a wait placed after them would also wait for every stage in flight.  Using the
    // fragments here puts that wait before the first direct load is issued.
    if constexpr (PAGED) asm volatile("" ::"v"(my_page) : "memory");
#pragma unroll
    for (int t = 0; t < ROW_TILES; ++t)
        asm volatile("" ::"v"(qf[t][0]), "v"(qf[t][1]), "v"(qf[t][2]), "v"(qf[t][3]), "v"(qf[t][4]), "v"(qf[t][5]),
                     "v"(qf[t][6]), "v"(qf[t][7])
                     : "memory");

    // ---- first stages of K; the loop starts as soon as stage 0 is in ---------------------
#pragma unroll
    for (int s = 0; s < RING - 1; ++s)
        if (s < nstages) stage_issue(s);
    wait_but(nstages - 1 < RING - 2 ? nstages - 1 : RING - 2);          // stage 0 is in

    float cst[ROW_TILES][16];
    if constexpr (COLSUM) {
        __syncthreads();                                   // per-row constants are in LDS
#pragma unroll
        for (int t = 0; t < ROW_TILES; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                cst[t][i] = s_c[GROUP_ROWS * rg + 32 * t + 8 * (i >> 2) + 4 * hf + (i & 3)];
    }

    float m_run[ROW_TILES], z_run[ROW_TILES];
#pragma unroll
    for (int t = 0; t < ROW_TILES; ++t) { m_run[t] = -INFINITY; z_run[t] = 0.0f; }
    const float sc = a.scale_log2;

    // LDS slots of this lane's eight K fragments inside a stage buffer
    const int krow = 32 * kt + c32;
    int kslot[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kslot[ks] = krow * 16 + ((2 * ks + hf) ^ (krow & 15));

    // Every wavefront has waited for its own part of stage 0 above; the only loads in flight
    // from here on are the direct loads of later stages.
    __syncthreads();

    // ---- main loop, software pipelined over stages -------------------------------------
    // Iteration s issues the MFMAs of stage s while the vector ALUs reduce the
    // accumulators of stage s-1 (softmax statistics or column sums), so the matrix pipe
    // and the VALU of a wavefront overlap instead of alternating.
    const auto stage_sync = [&](int s) {
        if (s > 0) {
            // stage s has landed once at most the loads of the later stages issued so far
            // (up to RING - 2 of them) are outstanding
            const int later = nstages - 1 - s;
            wait_but(later < RING - 2 ? later : RING - 2);
            __syncthreads();                               // every wavefront: stage s landed, stage s-1 consumed
        }
        if (s + RING - 1 < nstages) stage_issue(s + RING - 1);   // overwrites the buffer of stage s-1
    };
    const auto mma = [&](int s, f32x16 (&acc)[ROW_TILES]) {
        const uint4* buf = &s_k[s % RING][0];
        bf16x8 kf[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kf[ks] = as_frag(buf[kslot[ks]]);
#pragma unroll
        for (int t = 0; t < ROW_TILES; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][i] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int t = 0; t < ROW_TILES; ++t) {
                if constexpr (!COLSUM)   // keys x rows: acc[t][i] = key tile + 8*(i/4) + 4*hf + i%4, this lane's row
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[t][ks], acc[t], 0, 0, 0);
                else                     // rows x keys: acc[t][i] = row 64*rg + 32*t + 8*(i/4) + 4*hf + i%4, key tile + c32
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[t][ks], kf[ks], acc[t], 0, 0, 0);
            }
    };
    // reduction of the accumulators of stage s; MASKED: some key of the stage is hidden from some row
    const auto reduce = [&](int s, f32x16 (&acc)[ROW_TILES], auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int32_t tile_key0 = key_lo + stage_pos(s) * STAGE_KEYS + 32 * kt;
        float colsum = 0.0f;
#pragma unroll
        for (int t = 0; t < ROW_TILES; ++t) {
            if constexpr (!COLSUM) {
                if constexpr (MASKED) {
                    const int32_t lim = my_lim[t];
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int32_t key = tile_key0 + 8 * (i >> 2) + 4 * hf + (i & 3);
                        acc[t][i] = key <= lim ? acc[t][i] : -INFINITY;
                    }
                }
                float tmax = acc[t][0];
#pragma unroll
                for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, acc[t][i]);
                const float mnew = fmaxf(m_run[t], tmax * sc);
                const float mref = (MASKED && mnew == -INFINITY) ? 0.0f : mnew;   // every key hidden so far
                float sum = 0.0f;
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(acc[t][i], sc, -mref));
                z_run[t] = z_run[t] * fast_exp2(m_run[t] - mref) + sum;
                m_run[t] = mnew;
            } else {
                if constexpr (!MASKED) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) colsum += fast_exp2(fmaf(acc[t][i], sc, -cst[t][i]));
                } else {
                    const int32_t key = tile_key0 + c32;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int row = GROUP_ROWS * rg + 32 * t + 8 * (i >> 2) + 4 * hf + (i & 3);
                        const float p = fast_exp2(fmaf(acc[t][i], sc, -cst[t][i]));
                        colsum += key <= s_lim[row] ? p : 0.0f;
                    }
                }
            }
        }
        if constexpr (COLSUM) {
            colsum += __shfl_xor(colsum, 32);
            if (hf == 0) s_part[s & 1][rg][32 * kt + c32] = colsum;
        }
    };
    // column sums of stage s: add the row groups' partial sums (complete after the next barrier)
    const auto flush = [&](int s) {
        if constexpr (COLSUM) {
            if (tid < STAGE_KEYS) {
                const int32_t key = key_lo + stage_pos(s) * STAGE_KEYS + tid;
                if (key < key_hi) {
                    float v = s_part[s & 1][0][tid];
#pragma unroll
                    for (int w = 1; w < RG; ++w) v += s_part[s & 1][w][tid];
                    float* dst = &a.A[(size_t)unit * n + key];
                    *dst = row_base > 0 ? *dst + v : v;    // the same thread wrote it in the pass before
                }
            }
        }
    };
    using fast_tag = std::integral_constant<bool, false>;
    using masked_tag = std::integral_constant<bool, true>;

    int flushed = 0, reduced = 0;                          // stages whose column sums are written / in LDS
    const auto flush_pending = [&]() {
        for (; flushed < reduced; ++flushed) flush(flushed);
    };
    // The same in two halves for the pipelined loop: the LDS reads of the partial sums are issued
    // right behind the barrier and their sum is stored after the stage's MFMAs and reduction.  Done
    // in one piece at the top of the stage, the wavefront that flushes waits for its reads behind
    // the fragment reads of every other wavefront (all issued at the barrier), falls behind by that
    // wait in every stage, and the whole workgroup waits for it at the next barrier.
    float fl_v[RG];
    int32_t fl_key = -1;
    const auto flush_begin = [&]() {
        fl_key = -1;
        if constexpr (COLSUM) {
            if (flushed < reduced) {
                if (tid < STAGE_KEYS) {
                    const int32_t key = key_lo + stage_pos(flushed) * STAGE_KEYS + tid;
                    if (key < key_hi) {
                        fl_key = key;
#pragma unroll
                        for (int w = 0; w < RG; ++w) fl_v[w] = s_part[flushed & 1][w][tid];
                    }
                }
                ++flushed;
            }
            flush_pending();                               // (the pipelined loop never has a second stage pending)
        }
    };
    const auto flush_end = [&]() {
        if constexpr (COLSUM) {
            if (fl_key >= 0) {
                float v = fl_v[0];
#pragma unroll
                for (int w = 1; w < RG; ++w) v += fl_v[w];
                float* dst = &a.A[(size_t)unit * n + fl_key];
                *dst = row_base > 0 ? *dst + v : v;
            }
        }
    };

    // (A) fully visible stages: MFMAs of stage s and the reduction of stage s-1 in one block.
    // Two accumulator sets alternate (loop unrolled by two) so that no registers are copied.
    if (nfast > 0) {
        f32x16 acc_even[ROW_TILES], acc_odd[ROW_TILES];
        stage_sync(0);
        mma(0, acc_even);
        int s = 1;
        for (; s + 1 < nfast; s += 2) {
            stage_sync(s);
            flush_begin();                                 // reductions before this barrier are complete
            mma(s, acc_odd);
            reduce(s - 1, acc_even, fast_tag{});
            flush_end();
            reduced = s;
            stage_sync(s + 1);
            flush_begin();
            mma(s + 1, acc_even);
            reduce(s, acc_odd, fast_tag{});
            flush_end();
            reduced = s + 1;
        }
        const bool odd_left = s < nfast;                   // one more stage, into the odd set
        if (odd_left) {
            stage_sync(s);
            flush_pending();
            mma(s, acc_odd);
            reduce(s - 1, acc_even, fast_tag{});
            reduced = s;
        }
        if constexpr (COLSUM) {
            // the drain below writes the partial-sum buffer that the last flush above read
            __syncthreads();
            flush_pending();
        }
        if (odd_left) reduce(nfast - 1, acc_odd, fast_tag{});
        else reduce(nfast - 1, acc_even, fast_tag{});
        reduced = nfast;
        if constexpr (COLSUM) {
            // both partial-sum buffers are pending here; empty them before loop (B) reuses one
            __syncthreads();
            flush_pending();
        }
    }
    // (B) the few stages near the causal diagonal or past the sequence end: masked, not pipelined
    for (int s = nfast; s < nstages; ++s) {
        stage_sync(s);
        flush_pending();
        f32x16 acc_cur[ROW_TILES];
        mma(s, acc_cur);
        reduce(s, acc_cur, masked_tag{});
        reduced = s + 1;
    }
    if constexpr (COLSUM) {
        __syncthreads();
        flush_pending();
        for (int32_t key = key_lo + nstages * STAGE_KEYS + tid; key < key_hi; key += THREADS)
            a.A[(size_t)unit * n + key] = 0.0f;
    }

    if constexpr (!COLSUM) {
        // merge the two half-waves (disjoint key subsets of the same row), then the two
        // key-tile wavefronts of the row group through LDS, then store
        __syncthreads();                                       // staging buffers are idle now
        float* s_m = reinterpret_cast<float*>(&s_k[0][0]);
        float* s_z = s_m + GROUP_ROWS * RG;
#pragma unroll
        for (int t = 0; t < ROW_TILES; ++t) {
            const float mo = __shfl_xor(m_run[t], 32), zo = __shfl_xor(z_run[t], 32);
            const float mf = fmaxf(m_run[t], mo);
            float zf = 0.0f;
            if (mf > -INFINITY) zf = z_run[t] * fast_exp2(m_run[t] - mf) + zo * fast_exp2(mo - mf);
            m_run[t] = mf;
            z_run[t] = zf;
        }
        if (kt == 1 && hf == 0) {
#pragma unroll
            for (int t = 0; t < ROW_TILES; ++t) {
                s_m[GROUP_ROWS * rg + 32 * t + c32] = m_run[t];
                s_z[GROUP_ROWS * rg + 32 * t + c32] = z_run[t];
            }
        }
        __syncthreads();
        if (kt == 0 && hf == 0) {
            float* st = a.ws + (((size_t)unit * a.nchunks + chunk) * a.rows_pad) * 2;
#pragma unroll
            for (int t = 0; t < ROW_TILES; ++t) {
                const int32_t r = GROUP_ROWS * rg + 32 * t + c32;
                const float mo = s_m[r], zo = s_z[r];
                const float mf = fmaxf(m_run[t], mo);
                float zf = 0.0f;
                if (mf > -INFINITY) zf = z_run[t] * fast_exp2(m_run[t] - mf) + zo * fast_exp2(mo - mf);
                st[(row_base + r) * 2] = mf;
                st[(row_base + r) * 2 + 1] = zf;
            }
        }
    }
}

template <int RG, int RT, bool COLSUM>
hipError_t launch_sweep(const ScoreArgs& a, unsigned blocks, const MatchRider* rider, hipStream_t st)
{
    if (rider && a.table) {
        // paged keys: the match runs as a launch of its own in front of the sweep
        const hipError_t e = launch_match(rider->tok, a.seq_len, a.batch, a.n, *rider->tab, rider->anchor_B, rider->allow,
                                          rider->anchor, rider->spons, rider->vouch, st);
        if (e != hipSuccess) return e;
        rider = nullptr;
    }
    if (rider) {
        RiderArgs r;
        r.m = make_match_args(rider->tok, a.seq_len, a.batch, a.n, rider->anchor_B, rider->allow, rider->anchor, rider->spons,
                              rider->vouch);
        r.tab = *rider->tab;
        r.score_blocks = blocks;
        const unsigned extra = (unsigned)r.m.tiles * (unsigned)r.m.batch;
        hipLaunchKernelGGL((score_match_kernel<RG, RT, COLSUM>), dim3(blocks + extra), dim3(128 * RG), 0, st, a, r);
    } else if (a.table) {
        hipLaunchKernelGGL((score_kernel<RG, RT, COLSUM, true>), dim3(blocks), dim3(128 * RG), 0, st, a);
    } else {
        hipLaunchKernelGGL((score_kernel<RG, RT, COLSUM, false>), dim3(blocks), dim3(128 * RG), 0, st, a);
    }
    return hipGetLastError();
}

template <int RG, int RT>
hipError_t launch_rg(ScoreArgs a, int64_t units, const MatchRider* rider, hipStream_t st)
{
    // One launch per sweep over all units.  (Splitting the units into cache-sized groups
    // so that sweep 2 re-reads its keys from the last-level cache was measured slower.)
    a.units = (int32_t)units;
    a.units_per_xcd = (int32_t)((units + 7) / 8);
    const unsigned blocks = (unsigned)(8ll * a.units_per_xcd * a.nchunks);
    if (a.lse)                                             // the row normalisers are given: column sums alone
        return launch_sweep<RG, RT, true>(a, blocks, rider, st);
    const hipError_t e = launch_sweep<RG, RT, false>(a, blocks, rider, st);
    if (e != hipSuccess) return e;
    return launch_sweep<RG, RT, true>(a, blocks, nullptr, st);
}

}  // namespace

namespace {

int32_t padded_rows(int32_t rows)
{
    if (rows <= 128) return 128;
    if (rows <= 256) return 256;
    return 512;
}

int compute_units()
{
    static std::atomic<int> cached{0};                     // callers on several threads may race to fill it
    int cu = cached.load(std::memory_order_relaxed);
    if (cu == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu < 1)
            cu = 256;                                      // MI355X
        cached.store(cu, std::memory_order_relaxed);
    }
    return cu;
}

struct ScorePlan {
    int32_t rows, rows_pad, chunk_keys, nchunks;
    int64_t units;
};

ScorePlan make_plan(const ta_layout& lay)
{
    ScorePlan p;
    p.rows = (lay.hq / lay.hkv) * lay.window;
    p.rows_pad = padded_rows(p.rows);
    // Chunks as long as possible (the per-workgroup prologue - Q fragments, first stages,
    // statistics merge - is amortised over the chunk) while the grid still offers about two
    // workgroups per compute unit; never more than 32 chunks per unit.
    p.units = (int64_t)lay.layers * lay.batch * lay.hkv;
    const int64_t want_blocks = 2 * (int64_t)compute_units();
    int64_t per_unit = (want_blocks + p.units - 1) / p.units;            // chunks per unit we would like
    per_unit = per_unit < 1 ? 1 : (per_unit > 32 ? 32 : per_unit);
    int64_t ck = ((lay.n + per_unit - 1) / per_unit + STAGE_KEYS - 1) / STAGE_KEYS * STAGE_KEYS;
    if (ck < 512) ck = 512;
    while (ck * 32 < lay.n) ck += STAGE_KEYS;
    p.chunk_keys = (int32_t)ck;
    p.nchunks = (lay.n + p.chunk_keys - 1) / p.chunk_keys;
    return p;
}

}  // namespace

size_t score_workspace_bytes(const ta_layout& lay)
{
    const ScorePlan p = make_plan(lay);
    // per-chunk row statistics (m, Z)
    return (size_t)p.units * p.nchunks * p.rows_pad * 2 * sizeof(float);
}

int64_t score_grid_blocks(const ta_layout& lay)
{
    const ScorePlan p = make_plan(lay);
    return 8 * ((p.units + 7) / 8) * p.nchunks;
}

hipError_t launch_score(const void* Q, const void* K, const ta_layout& lay, const int32_t* seq_len,
                        int causal, float* A, float* ws, const float* lse, const MatchRider* rider,
                        const ta_paged_kv* pg, const LayerPtrs* lp, hipStream_t st)
{
    const ScorePlan p = make_plan(lay);
    ScoreArgs a;
    a.Ql = lp ? reinterpret_cast<const uint4* const*>(&lp->Q[0]) : nullptr;
    a.Kl = lp ? reinterpret_cast<const uint4* const*>(&lp->K[0]) : nullptr;
    a.lse = lse;
    a.table = pg ? pg->block_table : nullptr;
    a.k_spage = pg ? pg->stride[1] / 8 : 0;
    a.page_size = pg ? pg->page_size : 0;
    a.max_pages = pg ? pg->max_pages : 0;
    a.num_pages = pg ? pg->num_pages : 0;
    a.page_shift = -1;
    if (pg && (pg->page_size & (pg->page_size - 1)) == 0) {
        a.page_shift = 0;
        while ((1 << a.page_shift) < pg->page_size) ++a.page_shift;
    }
    a.Q = (const uint4*)Q;
    a.K = (const uint4*)K;
    a.seq_len = seq_len;
    a.A = A;
    a.ws = ws;
    a.q_sl = lay.q_stride[0] / 8;
    a.q_sb = lay.q_stride[1] / 8;
    a.q_sh = lay.q_stride[2] / 8;
    if (pg) {
        a.k_sl = pg->stride[0] / 8;
        a.k_sb = 0;
        a.k_sp = (int32_t)(pg->stride[2] / 8);
        a.k_sh = pg->stride[3] / 8;
    } else {
        a.k_sl = lay.kv_stride[0] / 8;
        a.k_sb = lay.kv_stride[1] / 8;
        a.k_sh = lay.kv_stride[2] / 8;
        a.k_sp = (int32_t)(lay.kv_stride[3] / 8);
    }
    a.batch = lay.batch;
    a.hkv = lay.hkv;
    a.G = lay.hq / lay.hkv;
    a.W = lay.window;
    a.n = lay.n;
    a.rows = p.rows;
    a.rows_pad = p.rows_pad;
    a.chunk_keys = p.chunk_keys;
    a.nchunks = p.nchunks;
    a.causal = causal;
    a.scale_log2 = (float)(1.4426950408889634 / sqrt((double)lay.d));
    switch (a.rows_pad) {
        // two 32-row tiles per wavefront (one tile per wavefront with twice the wavefronts - four
        // per SIMD instead of two - was measured: same time at 128 rows, 5 % slower at 256)
        case 128: return launch_rg<2, 2>(a, p.units, rider, st);
        case 256: return launch_rg<4, 2>(a, p.units, rider, st);
        default: return launch_rg<4, 2>(a, p.units, rider, st);   // 512 rows: two passes of 256 (eight row groups
                                                                  // at once leave 128 registers per lane: spills, 3x slower)
    }
}

}  // namespace ta
