// Step 5 of the eviction pass: gather of the retained K/V rows (index_select
// along the sequence dimension, Sec. 3.2 "Token selection"; Alg. 1, eviction
// step).  Pure data movement, bound by HBM.
//
// A 256-byte row (d = 128 bf16) is moved by 16 lanes with one 16-byte load and
// one 16-byte store each, so a wavefront moves 4 rows per instruction.  A
// workgroup takes ROWS_PER_BLOCK consecutive output rows of one unit and issues
// all of its loads (K and V) before the first store to keep many requests in
// flight per lane.
#include "ta_internal.h"

namespace ta {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int COMPACT_THREADS = 256;
constexpr int ROWS_PER_ITER = COMPACT_THREADS / 16;     // 16 rows per pass over the block
constexpr int COMPACT_ITERS = 4;
constexpr int ROWS_PER_BLOCK = ROWS_PER_ITER * COMPACT_ITERS;

struct CompactArgs {
    const uint4* Kin;
    const uint4* Vin;
    const int32_t* idx;
    const int32_t* cnt;
    uint4* Kout;
    uint4* Vout;
    int64_t s_layer, s_batch, s_head, s_pos;   // input strides in 16-byte units
    int32_t batch, hkv, n, K;
    int32_t idx_shared;
    int32_t blocks_per_unit;
    // paged input: rows are addressed through the block table (s_batch unused, s_page per page)
    const int32_t* table;
    int64_t s_page;
    int32_t page_size, max_pages, num_pages;
    // one tensor per layer: DEVICE tables; layer l reads Kin_l[l], Vin_l[l] and writes Kout_l[l], Vout_l[l]
    const uint4* const* Kin_l;
    const uint4* const* Vin_l;
    uint4* const* Kout_l;
    uint4* const* Vout_l;
    // paged output: row r of a unit goes to slot r of its sequence's pages in the destination pools
    const int32_t* d_table;
    int64_t d_layer, d_page, d_pos, d_head;    // destination strides in 16-byte units
    int32_t d_page_size, d_max_pages, d_num_pages;
};

// marks a pointer read from a device table as a global address (else it is accessed with flat instructions)
template <typename T>
__device__ __forceinline__ T* global_ptr(T* p)
{
    typedef __attribute__((address_space(1))) T* gp;
    return (T*)(gp)(uintptr_t)p;
}

template <bool PAGED, bool LAYERED, bool DST_PAGED = false>
__global__ void __launch_bounds__(COMPACT_THREADS)
compact_kernel(CompactArgs a)
{
    const int32_t unit = (int32_t)(blockIdx.x / (uint32_t)a.blocks_per_unit);
    const int32_t blk = (int32_t)(blockIdx.x % (uint32_t)a.blocks_per_unit);
    const int32_t h = unit % a.hkv;
    const int32_t b = (unit / a.hkv) % a.batch;
    const int32_t l = unit / (a.hkv * a.batch);
    const int32_t sel = a.idx_shared ? b : unit;
    int32_t cnt = a.cnt[sel];
    cnt = cnt > a.K ? a.K : cnt;
    const int32_t* idx = a.idx + (size_t)sel * (size_t)a.K;
    const int64_t in_base = (LAYERED ? 0 : l * a.s_layer) + (PAGED ? 0 : b * a.s_batch) + h * a.s_head;
    const int64_t out_base = (int64_t)(LAYERED ? unit - l * a.hkv * a.batch : unit) * a.K * 16;

    const int lane16 = threadIdx.x & 15;
    const int rsub = threadIdx.x >> 4;
    if (blk * ROWS_PER_BLOCK >= cnt) return;              // whole block past the retained rows
    // named registers (not an indexed array) so the loads stay in VGPRs
    const int32_t row0 = blk * ROWS_PER_BLOCK + rsub;
    auto src = [&](int32_t r) -> int64_t {
        r = r < cnt ? r : cnt - 1;                          // tail lanes re-read the last row, store nothing
        int32_t p = idx[r];
        p = p < 0 ? 0 : (p >= a.n ? a.n - 1 : p);
        if (PAGED) {
            const int32_t slot = p / a.page_size;
            int32_t page = a.table[(size_t)b * a.max_pages + slot];
            page = page < 0 ? 0 : (page >= a.num_pages ? a.num_pages - 1 : page);
            return in_base + (int64_t)page * a.s_page + (int64_t)(p - slot * a.page_size) * a.s_pos + lane16;
        }
        return in_base + (int64_t)p * a.s_pos + lane16;
    };
    static_assert(COMPACT_ITERS == 4, "loads below are written out four times");
    const int64_t o0 = src(row0), o1 = src(row0 + ROWS_PER_ITER);
    const int64_t o2 = src(row0 + 2 * ROWS_PER_ITER), o3 = src(row0 + 3 * ROWS_PER_ITER);
    // The compacted rows are not read again by this pass: streaming stores keep them from
    // lingering in the caches as dirty lines that the next kernel's reads would have to evict.
    const u32x4* Kin = reinterpret_cast<const u32x4*>(LAYERED ? global_ptr(a.Kin_l[l]) : a.Kin);
    const u32x4* Vin = reinterpret_cast<const u32x4*>(LAYERED ? global_ptr(a.Vin_l[l]) : a.Vin);
    u32x4* Kout = reinterpret_cast<u32x4*>(LAYERED ? global_ptr(a.Kout_l[l]) : a.Kout);
    u32x4* Vout = reinterpret_cast<u32x4*>(LAYERED ? global_ptr(a.Vout_l[l]) : a.Vout);
    const u32x4 k0 = __builtin_nontemporal_load(&Kin[o0]), k1 = __builtin_nontemporal_load(&Kin[o1]);
    const u32x4 k2 = __builtin_nontemporal_load(&Kin[o2]), k3 = __builtin_nontemporal_load(&Kin[o3]);
    const u32x4 v0 = __builtin_nontemporal_load(&Vin[o0]), v1 = __builtin_nontemporal_load(&Vin[o1]);
    const u32x4 v2 = __builtin_nontemporal_load(&Vin[o2]), v3 = __builtin_nontemporal_load(&Vin[o3]);
    auto put = [&](int32_t r, const u32x4& kk, const u32x4& vv) {
        if (r < cnt) {
            int64_t off = out_base + (int64_t)r * 16 + lane16;
            if (DST_PAGED) {
                const int32_t slot = r / a.d_page_size;
                int32_t page = a.d_table[(size_t)b * a.d_max_pages + slot];
                page = page < 0 ? 0 : (page >= a.d_num_pages ? a.d_num_pages - 1 : page);
                off = l * a.d_layer + (int64_t)page * a.d_page + (int64_t)(r - slot * a.d_page_size) * a.d_pos + h * a.d_head + lane16;
            }
            __builtin_nontemporal_store(kk, &Kout[off]);
            __builtin_nontemporal_store(vv, &Vout[off]);
        }
    };
    put(row0, k0, v0);
    put(row0 + ROWS_PER_ITER, k1, v1);
    put(row0 + 2 * ROWS_PER_ITER, k2, v2);
    put(row0 + 3 * ROWS_PER_ITER, k3, v3);
}

// Writes a table of per-layer addresses, handed over by value, to device memory: the kernels of the
// pass then read their layer's entries from there.  (Arrays inside those kernels' own argument
// structs were measured first: a run-time choice between a table entry and the base pointer made
// the compiler copy the whole argument block to scratch memory per lane - the compaction took
// 690 us instead of 42 - and the statistics sweep reloaded arguments inside its stage loop.)
// N layers of the five tables, packed: small argument blocks stay on the fast path (the table of
// a 32-layer model is 1.3 KB).
template <int N>
struct PackedLayerPtrs {
    const void* p[5][N];
};

template <int N>
__global__ void layer_table_kernel(PackedLayerPtrs<N> t, LayerPtrs* dst, int32_t layers)
{
    const void** out[5] = {dst->Q, dst->K, dst->V, const_cast<const void**>(reinterpret_cast<void* const*>(dst->Kout)),
                           const_cast<const void**>(reinterpret_cast<void* const*>(dst->Vout))};
    for (int i = (int)threadIdx.x; i < 5 * layers; i += (int)blockDim.x) {
        const int arr = i / layers, l = i - arr * layers;
        out[arr][l] = t.p[arr][l];
    }
}

template <int N>
void launch_layer_table_n(const LayerPtrs& h, LayerPtrs* dev_table, int32_t layers, hipStream_t st)
{
    PackedLayerPtrs<N> t;
    for (int l = 0; l < N; ++l) {
        const bool on = l < layers;
        t.p[0][l] = on ? h.Q[l] : nullptr;
        t.p[1][l] = on ? h.K[l] : nullptr;
        t.p[2][l] = on ? h.V[l] : nullptr;
        t.p[3][l] = on ? h.Kout[l] : nullptr;
        t.p[4][l] = on ? h.Vout[l] : nullptr;
    }
    hipLaunchKernelGGL(layer_table_kernel<N>, dim3(1), dim3(256), 0, st, t, dev_table, layers);
}

}  // namespace

hipError_t launch_layer_table(const LayerPtrs& host_table, LayerPtrs* dev_table, int32_t layers, hipStream_t st)
{
    if (layers <= 32) launch_layer_table_n<32>(host_table, dev_table, layers, st);
    else launch_layer_table_n<TA_MAX_LAYER_PTRS>(host_table, dev_table, layers, st);
    return hipGetLastError();
}

hipError_t launch_compact(const void* Kin, const void* Vin, const int32_t* idx, const int32_t* cnt,
                          const ta_layout& lay, int32_t K, int32_t idx_shared,
                          void* Kout, void* Vout, const ta_paged_kv* pg, const LayerPtrs* lp, hipStream_t st,
                          const ta_paged_kv* dst_pg)
{
    CompactArgs a;
    a.d_table = dst_pg ? dst_pg->block_table : nullptr;
    a.d_layer = dst_pg ? dst_pg->stride[0] / 8 : 0;
    a.d_page = dst_pg ? dst_pg->stride[1] / 8 : 0;
    a.d_pos = dst_pg ? dst_pg->stride[2] / 8 : 0;
    a.d_head = dst_pg ? dst_pg->stride[3] / 8 : 0;
    a.d_page_size = dst_pg ? dst_pg->page_size : 1;
    a.d_max_pages = dst_pg ? dst_pg->max_pages : 0;
    a.d_num_pages = dst_pg ? dst_pg->num_pages : 0;
    a.Kin_l = lp ? reinterpret_cast<const uint4* const*>(&lp->K[0]) : nullptr;
    a.Vin_l = lp ? reinterpret_cast<const uint4* const*>(&lp->V[0]) : nullptr;
    a.Kout_l = lp ? reinterpret_cast<uint4* const*>(&lp->Kout[0]) : nullptr;
    a.Vout_l = lp ? reinterpret_cast<uint4* const*>(&lp->Vout[0]) : nullptr;
    a.Kin = (const uint4*)Kin;
    a.Vin = (const uint4*)Vin;
    a.idx = idx;
    a.cnt = cnt;
    a.Kout = (uint4*)Kout;
    a.Vout = (uint4*)Vout;
    if (pg) {
        a.s_layer = pg->stride[0] / 8;
        a.s_page = pg->stride[1] / 8;
        a.s_pos = pg->stride[2] / 8;
        a.s_head = pg->stride[3] / 8;
        a.s_batch = 0;
        a.table = pg->block_table;
        a.page_size = pg->page_size;
        a.max_pages = pg->max_pages;
        a.num_pages = pg->num_pages;
    } else {
        a.s_layer = lay.kv_stride[0] / 8;
        a.s_batch = lay.kv_stride[1] / 8;
        a.s_head = lay.kv_stride[2] / 8;
        a.s_pos = lay.kv_stride[3] / 8;
        a.table = nullptr;
        a.s_page = 0;
        a.page_size = a.max_pages = a.num_pages = 0;
    }
    a.batch = lay.batch;
    a.hkv = lay.hkv;
    a.n = lay.n;
    a.K = K;
    a.idx_shared = idx_shared;
    a.blocks_per_unit = (K + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK;
    int64_t units = (int64_t)lay.layers * lay.batch * lay.hkv;
    int64_t blocks = units * a.blocks_per_unit;
    const dim3 grid((unsigned)blocks), block(COMPACT_THREADS);
    if (dst_pg && pg) hipLaunchKernelGGL((compact_kernel<true, false, true>), grid, block, 0, st, a);
    else if (dst_pg) hipLaunchKernelGGL((compact_kernel<false, false, true>), grid, block, 0, st, a);
    else if (pg && lp) hipLaunchKernelGGL((compact_kernel<true, true>), grid, block, 0, st, a);
    else if (pg) hipLaunchKernelGGL((compact_kernel<true, false>), grid, block, 0, st, a);
    else if (lp) hipLaunchKernelGGL((compact_kernel<false, true>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((compact_kernel<false, false>), grid, block, 0, st, a);
    return hipGetLastError();
}

}  // namespace ta
