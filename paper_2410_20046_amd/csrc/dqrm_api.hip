// C ABI of the DQRM embedding hot path: host-side validation and kernel dispatch.
// Every entry point validates on the host first and enqueues nothing on error.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <algorithm>
#include <cstring>
#include <mutex>

#include "dqrm.h"
#include "dqrm_device.hpp"
#include "dqrm_fwd.hpp"
#include "dqrm_bwd.hpp"
#include "dqrm_update.hpp"
#include "dqrm_merge.hpp"
#include "dqrm_dense.hpp"

// Scratch of dqrm_embbag_bwd_noalloc: one copy per GPU, held until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels receive the address that call returns.
static __device__ __align__(256) unsigned char scratch[DQRM_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local char t_hip_error[256] = "";

int32_t hip_fail(hipError_t e, const char *what)
{
    std::snprintf(t_hip_error, sizeof(t_hip_error), "%s: %s", what, hipGetErrorString(e));
    return DQRM_ERR_HIP;
}

#define DQRM_HIP_CHECK(expr)                                 \
    do {                                                     \
        hipError_t e_ = (expr);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);    \
    } while (0)

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

int pow2ceil(int x)
{
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

// Checks the table descriptor; *total_rows receives R.
int32_t check_tables(const dqrm_tables_t *tb, bool need_packed, int64_t *total_rows)
{
    if (!tb) return DQRM_ERR_INVALID_ARG;
    if (tb->num_tables < 1 || tb->dim < 1) return DQRM_ERR_INVALID_ARG;
    if (!tb->row_offsets_host || !tb->row_offsets_dev || !tb->master || !tb->w_scale) return DQRM_ERR_INVALID_ARG;
    if (need_packed && !tb->packed) return DQRM_ERR_INVALID_ARG;
    if (tb->num_tables > DQRM_MAX_TABLES) return DQRM_ERR_UNSUPPORTED;
    if (tb->dim % 8 != 0 || tb->dim > DQRM_MAX_DIM) return DQRM_ERR_UNSUPPORTED;
    if (!aligned(tb->master, 16) || (tb->packed && !aligned(tb->packed, 4))) return DQRM_ERR_INVALID_ARG;
    const int64_t *ro = tb->row_offsets_host;
    if (ro[0] != 0) return DQRM_ERR_INVALID_ARG;
    for (int t = 0; t < tb->num_tables; ++t) {
        if (ro[t + 1] < ro[t]) return DQRM_ERR_INVALID_ARG;
        if (ro[t + 1] - ro[t] > DQRM_MAX_TABLE_ROWS) return DQRM_ERR_UNSUPPORTED;
    }
    *total_rows = ro[tb->num_tables];
    return DQRM_OK;
}

constexpr int64_t kMaxIndices = 2147483647LL - 2 * DQRM_MAX_TABLES - 64;
// the element-wise kernels index quarter-rows (float4) of the sparse gradient with 32-bit numbers
constexpr int64_t kMaxRowQuarters = 2147483647LL - 4LL * 2048 * 256;

int32_t check_batch(const dqrm_tables_t *tb, const int64_t *indices, const int64_t *offsets, int32_t batch,
                    int64_t num_indices)
{
    if (!offsets || batch < 1 || num_indices < 0) return DQRM_ERR_INVALID_ARG;
    if (num_indices > 0 && !indices) return DQRM_ERR_INVALID_ARG;
    if (num_indices > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    if ((int64_t)batch * tb->num_tables > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    return DQRM_OK;
}

// ---- workspace layout of dqrm_embbag_bwd -------------------------------------
struct WsLayout {
    size_t off_table_base, off_table_nuniq, off_table_nchunk, off_table_nsingle, off_totals, off_bag_of_pos, off_sorted_bag,
        off_chunk_local, off_single_local, off_chunk_desc, off_chunk_bags, off_single_desc, off_run_key, off_run_pos,
        off_merged_key, off_merged_pos, off_head_of_seg, off_seg_count, off_partial_full,
        off_partial_last, off_absmax_slots, total;
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

WsLayout ws_layout(int32_t T, int32_t D, int64_t N)
{
    WsLayout L{};
    size_t o = 0;
    const size_t n = (size_t)N, t = (size_t)T, slots = (size_t)(N / DQRM_SEG_CHUNK + 2);
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes, 256);
        return at;
    };
    L.off_table_base = take(t * sizeof(int));
    L.off_table_nuniq = take(t * sizeof(int));
    L.off_table_nchunk = take(t * sizeof(int));
    L.off_table_nsingle = take(t * sizeof(int));
    L.off_totals = take(4 * sizeof(int));
    L.off_bag_of_pos = take(n * sizeof(int));
    L.off_sorted_bag = take(n * sizeof(int));
    // (the lists have a slot even for an empty batch: the summing kernels request their first entries before they
    // know the counts)
    const size_t n1 = n ? n : 1;
    L.off_chunk_local = take(n1 * 16);
    L.off_single_local = take(n1 * 16);
    L.off_chunk_desc = take(n1 * 16);
    L.off_chunk_bags = take((n / 2 + 1) * DQRM_SEG_CHUNK * sizeof(int));
    L.off_single_desc = take(n1 * 16);
    // (the large-table path exists only for batches that can hold a large table)
    const size_t big = N > dqrm::kDdCap ? n : 0;
    L.off_run_key = take(big * sizeof(int));
    L.off_run_pos = take(big * sizeof(int));
    L.off_merged_key = take(big * sizeof(int));
    L.off_merged_pos = take(big * sizeof(int));
    L.off_head_of_seg = take(big ? (big + t + 1) * sizeof(int) : 0);
    L.off_seg_count = take(slots * sizeof(int));
    L.off_partial_full = take(slots * (size_t)D * sizeof(float));
    L.off_partial_last = take(slots * (size_t)D * sizeof(float));
    L.off_absmax_slots = take(t * dqrm::kAbsmaxSlots * dqrm::kAbsmaxStride * sizeof(float));
    L.total = o;
    return L;
}

dqrm::BwdWs ws_views(void *workspace, const WsLayout &L)
{
    char *b = static_cast<char *>(workspace);
    dqrm::BwdWs w;
    w.table_base = reinterpret_cast<int *>(b + L.off_table_base);
    w.table_nuniq = reinterpret_cast<int *>(b + L.off_table_nuniq);
    w.table_nchunk = reinterpret_cast<int *>(b + L.off_table_nchunk);
    w.table_nsingle = reinterpret_cast<int *>(b + L.off_table_nsingle);
    w.totals = reinterpret_cast<int *>(b + L.off_totals);
    w.bag_of_pos = reinterpret_cast<int *>(b + L.off_bag_of_pos);
    w.sorted_bag = reinterpret_cast<int *>(b + L.off_sorted_bag);
    w.chunk_local = reinterpret_cast<int4 *>(b + L.off_chunk_local);
    w.single_local = reinterpret_cast<int4 *>(b + L.off_single_local);
    w.chunk_desc = reinterpret_cast<int4 *>(b + L.off_chunk_desc);
    w.chunk_bags = reinterpret_cast<int *>(b + L.off_chunk_bags);
    w.single_desc = reinterpret_cast<int4 *>(b + L.off_single_desc);
    w.run_key = reinterpret_cast<unsigned *>(b + L.off_run_key);
    w.run_pos = reinterpret_cast<int *>(b + L.off_run_pos);
    w.merged_key = reinterpret_cast<unsigned *>(b + L.off_merged_key);
    w.merged_pos = reinterpret_cast<int *>(b + L.off_merged_pos);
    w.head_of_seg = reinterpret_cast<int *>(b + L.off_head_of_seg);
    w.seg_count = reinterpret_cast<int *>(b + L.off_seg_count);
    w.partial_full = reinterpret_cast<float *>(b + L.off_partial_full);
    w.partial_last = reinterpret_cast<float *>(b + L.off_partial_last);
    w.absmax_slots = reinterpret_cast<float *>(b + L.off_absmax_slots);
    return w;
}

int num_cus()
{
    static thread_local int cached_dev = -1, cached = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (dev != cached_dev) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cached = v;
        cached_dev = dev;
    }
    return cached;
}

int grid_for(int64_t work_items, int threads, int blocks_per_cu)
{
    int64_t want = (work_items + threads - 1) / threads;
    int64_t cap = (int64_t)num_cus() * blocks_per_cu;
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    return (int)want;
}

template <bool PACKED>
void launch_fwd(int G, dim3 grid, hipStream_t st, const dqrm::FwdArgs &a)
{
    using namespace dqrm;
    switch (G) {
    case 2: hipLaunchKernelGGL((embbag_fwd_kernel<2, PACKED>), grid, dim3(kFwdThreads), 0, st, a); break;
    case 4: hipLaunchKernelGGL((embbag_fwd_kernel<4, PACKED>), grid, dim3(kFwdThreads), 0, st, a); break;
    case 8: hipLaunchKernelGGL((embbag_fwd_kernel<8, PACKED>), grid, dim3(kFwdThreads), 0, st, a); break;
    case 16: hipLaunchKernelGGL((embbag_fwd_kernel<16, PACKED>), grid, dim3(kFwdThreads), 0, st, a); break;
    case 32: hipLaunchKernelGGL((embbag_fwd_kernel<32, PACKED>), grid, dim3(kFwdThreads), 0, st, a); break;
    default: hipLaunchKernelGGL((embbag_fwd_kernel<64, PACKED>), grid, dim3(kFwdThreads), 0, st, a); break;
    }
}

void launch_segsum(int G, dim3 grid, hipStream_t st, const dqrm::SegArgs &a)
{
    using namespace dqrm;
    switch (G) {
    case 2: hipLaunchKernelGGL((segment_sum_kernel<2>), grid, dim3(kSumThreads), 0, st, a); break;
    case 4: hipLaunchKernelGGL((segment_sum_kernel<4>), grid, dim3(kSumThreads), 0, st, a); break;
    case 8: hipLaunchKernelGGL((segment_sum_kernel<8>), grid, dim3(kSumThreads), 0, st, a); break;
    case 16: hipLaunchKernelGGL((segment_sum_kernel<16>), grid, dim3(kSumThreads), 0, st, a); break;
    case 32: hipLaunchKernelGGL((segment_sum_kernel<32>), grid, dim3(kSumThreads), 0, st, a); break;
    default: hipLaunchKernelGGL((segment_sum_kernel<64>), grid, dim3(kSumThreads), 0, st, a); break;
    }
}

void launch_segsum_multi(int G, dim3 grid, hipStream_t st, const dqrm::SegMulti &m)
{
    using namespace dqrm;
    switch (G) {
    case 2: hipLaunchKernelGGL((segment_sum_multi_kernel<2>), grid, dim3(kSumThreads), 0, st, m); break;
    case 4: hipLaunchKernelGGL((segment_sum_multi_kernel<4>), grid, dim3(kSumThreads), 0, st, m); break;
    case 8: hipLaunchKernelGGL((segment_sum_multi_kernel<8>), grid, dim3(kSumThreads), 0, st, m); break;
    case 16: hipLaunchKernelGGL((segment_sum_multi_kernel<16>), grid, dim3(kSumThreads), 0, st, m); break;
    case 32: hipLaunchKernelGGL((segment_sum_multi_kernel<32>), grid, dim3(kSumThreads), 0, st, m); break;
    default: hipLaunchKernelGGL((segment_sum_multi_kernel<64>), grid, dim3(kSumThreads), 0, st, m); break;
    }
}

int32_t sparse_update_impl(const dqrm_tables_t *tables, int64_t capacity, const int64_t *uniq_rows,
                           const int32_t *table_uniq_offsets, const int8_t *gq, const int32_t *sums,
                           const float *g_scale, float lr, void *stream)
{
    int64_t R = 0;
    int32_t rc = check_tables(tables, false, &R);
    if (rc != DQRM_OK) return rc;
    if (capacity < 0 || !uniq_rows || !table_uniq_offsets || !g_scale) return DQRM_ERR_INVALID_ARG;
    if (capacity > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    if (capacity * (tables->dim / 4) > kMaxRowQuarters) return DQRM_ERR_UNSUPPORTED;
    dqrm::UpdateArgs a;
    a.master = tables->master;
    a.packed = tables->packed;
    a.w_scale = tables->w_scale;
    a.row_offsets = tables->row_offsets_dev;
    a.uniq_rows = uniq_rows;
    a.tuo = table_uniq_offsets;
    a.gq = gq;
    a.sums = sums;
    a.g_scale = g_scale;
    a.capacity = capacity;
    a.lr = lr;
    a.T = tables->num_tables;
    a.D = tables->dim;
    a.by_q4 = dqrm::FastDiv::make((unsigned)(a.D / 4));
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(dqrm::sparse_update_kernel, dim3(grid_for(capacity * (a.D / 4), dqrm::kEwThreads, 8)),
                       dim3(dqrm::kEwThreads), dqrm::TableLds::bytes(a.T), st, a);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

// workspace of dqrm_sparse_merge: table offsets of the merged list, and per place the source word, the
// first-of-its-row flag and the flags before it
struct MergeLayout {
    size_t off_base, off_src, off_head, off_excl, off_table_heads, total;
};
MergeLayout merge_layout(int T, int64_t max_total)
{
    MergeLayout L{};
    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        o = align_up(o + bytes, 256);
        return at;
    };
    const size_t m = (size_t)max_total;
    L.off_base = take(((size_t)T + 1) * sizeof(int32_t));
    L.off_src = take(m * sizeof(int32_t));
    L.off_head = take(m * sizeof(int32_t));
    L.off_excl = take(m * sizeof(int32_t));
    L.off_table_heads = take((size_t)T * sizeof(int32_t));
    L.total = o;
    return L;
}

} // namespace

extern "C" {

const char *dqrm_version(void) { return "0.1"; }

const char *dqrm_last_hip_error(void) { return t_hip_error; }

int32_t dqrm_find_scale(const dqrm_tables_t *tables, void *stream)
{
    int64_t R = 0;
    int32_t rc = check_tables(tables, false, &R);
    if (rc != DQRM_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int T = tables->num_tables, D = tables->dim;
    // w_scale doubles as the absmax accumulator (bit pattern of a non-negative float)
    hipLaunchKernelGGL(dqrm::fill_u32_kernel, dim3((T + 255) / 256), dim3(256), 0, st,
                       reinterpret_cast<unsigned *>(tables->w_scale), 0u, T);
    const int64_t f4 = R * (D / 4);
    if (f4 > 0) {
        hipLaunchKernelGGL(dqrm::table_absmax_kernel, dim3(grid_for(f4, dqrm::kEwThreads * 4, 16)),
                           dim3(dqrm::kEwThreads), 0, st, tables->master, tables->row_offsets_dev, T, D, tables->w_scale);
    }
    hipLaunchKernelGGL(dqrm::finalize_scale_kernel, dim3((T + 255) / 256), dim3(256), 0, st, tables->w_scale, T);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_pack_int4(const dqrm_tables_t *tables, void *stream)
{
    int64_t R = 0;
    int32_t rc = check_tables(tables, true, &R);
    if (rc != DQRM_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int T = tables->num_tables, D = tables->dim;
    const int64_t g8 = R * (D / 8);
    if (g8 > 0) {
        hipLaunchKernelGGL(dqrm::pack_int4_kernel, dim3(grid_for(g8, dqrm::kEwThreads * dqrm::kPackPerThread, 8)), dim3(dqrm::kEwThreads),
                           0, st, tables->master, tables->row_offsets_dev, tables->w_scale, T, D, tables->packed);
    }
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_embbag_fwd(const dqrm_tables_t *tables, const int64_t *indices, const int64_t *offsets, int32_t batch,
                        int64_t num_indices, int32_t mode, float *out, int8_t *codes_dbg, void *stream)
{
    int64_t R = 0;
    if (mode != DQRM_FWD_MASTER && mode != DQRM_FWD_PACKED) return DQRM_ERR_INVALID_ARG;
    int32_t rc = check_tables(tables, mode == DQRM_FWD_PACKED, &R);
    if (rc != DQRM_OK) return rc;
    rc = check_batch(tables, indices, offsets, batch, num_indices);
    if (rc != DQRM_OK) return rc;
    if (!out || !aligned(out, 16) || (codes_dbg && !aligned(codes_dbg, 4))) return DQRM_ERR_INVALID_ARG;

    dqrm::FwdArgs a;
    a.master = tables->master;
    a.packed = tables->packed;
    a.w_scale = tables->w_scale;
    a.row_offsets = tables->row_offsets_dev;
    a.indices = indices;
    a.offsets = offsets;
    a.out = out;
    a.codes = codes_dbg;
    a.num_indices = num_indices;
    a.T = tables->num_tables;
    a.B = batch;
    a.D = tables->dim;
    a.no_rows = tables->row_offsets_host[a.T] <= 0;
    a.tile_t = a.T < dqrm::kFwdTileT ? a.T : dqrm::kFwdTileT;

    const int G = pow2ceil(a.D / 4);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)((a.B + dqrm::kFwdTileB - 1) / dqrm::kFwdTileB),
                    (unsigned)((a.T + a.tile_t - 1) / a.tile_t));
    if (mode == DQRM_FWD_PACKED)
        launch_fwd<true>(G, grid, st, a);
    else
        launch_fwd<false>(G, grid, st, a);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

size_t dqrm_embbag_bwd_workspace_bytes(int32_t num_tables, int32_t dim, int32_t batch, int64_t num_indices)
{
    if (num_tables < 1 || num_tables > DQRM_MAX_TABLES || dim < 8 || dim > DQRM_MAX_DIM || dim % 8 != 0 || batch < 1 ||
        num_indices < 0 || num_indices > kMaxIndices)
        return 0;
    return ws_layout(num_tables, dim, num_indices).total;
}

int32_t dqrm_dedupe_multi(const dqrm_tables_t *tables, int32_t batch, int32_t num_batches,
                          const dqrm_dedupe_batch_t *batches, size_t workspace_bytes, void *stream)
{
    int64_t R = 0;
    int32_t rc = check_tables(tables, false, &R);
    if (rc != DQRM_OK) return rc;
    if (!batches || num_batches < 1) return DQRM_ERR_INVALID_ARG;
    if (num_batches > DQRM_MAX_DEDUPE_BATCHES) return DQRM_ERR_UNSUPPORTED;
    const int T = tables->num_tables, D = tables->dim;
    int64_t max_n = 0;
    for (int i = 0; i < num_batches; ++i) {
        const dqrm_dedupe_batch_t &b = batches[i];
        rc = check_batch(tables, b.indices, b.offsets, batch, b.num_indices);
        if (rc != DQRM_OK) return rc;
        if (!b.sorted_pos || !b.uniq_rows || !b.seg_offsets || !b.table_uniq_offsets || !b.num_unique || !b.workspace ||
            !aligned(b.workspace, 256))
            return DQRM_ERR_INVALID_ARG;
        if (b.max_table_lookups < 0) return DQRM_ERR_INVALID_ARG;
        if (workspace_bytes < ws_layout(T, D, b.num_indices).total) return DQRM_ERR_WORKSPACE_TOO_SMALL;
        if (b.num_indices > max_n) max_n = b.num_indices;
    }
    dqrm::DedupeArgs da;
    std::memset(&da, 0, sizeof(da));
    int64_t largest = 0; // no table of any batch has more lookups than this
    for (int i = 0; i < num_batches; ++i) {
        const dqrm_dedupe_batch_t &b = batches[i];
        dqrm::DedupeBatch &o = da.b[i];
        o.indices = b.indices;
        o.offsets = b.offsets;
        o.N = b.num_indices;
        o.limit = b.max_table_lookups > 0 ? std::min<int32_t>(b.max_table_lookups, DQRM_MAX_TABLE_LOOKUPS)
                                          : DQRM_MAX_TABLE_LOOKUPS;
        largest = std::max<int64_t>(largest, std::min<int64_t>(b.num_indices, o.limit));
        o.ws = ws_views(b.workspace, ws_layout(T, D, b.num_indices));
        o.sorted_pos = b.sorted_pos;
        o.tuo = b.table_uniq_offsets;
        o.num_unique = b.num_unique;
        o.uniq_rows = b.uniq_rows;
        o.seg_offsets = b.seg_offsets;
    }
    da.row_offsets = tables->row_offsets_dev;
    da.T = T;
    da.B = batch;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // a table of more than kDdCap lookups is sorted in tiles (grid z), which dedupe_large_kernel merges
    const int tiles = (int)std::max<int64_t>(1, (largest + dqrm::kDdCap - 1) / dqrm::kDdCap);
    hipLaunchKernelGGL(dqrm::dedupe_kernel, dim3(T, num_batches, tiles), dim3(dqrm::kDdThreads), 0, st, da);
    if (tiles > 1) {
        hipLaunchKernelGGL(dqrm::dedupe_merge_kernel, dim3(T, num_batches, tiles), dim3(dqrm::kDdThreads), 0, st, da);
        hipLaunchKernelGGL(dqrm::dedupe_large_kernel, dim3(T, num_batches), dim3(dqrm::kDdThreads), 0, st, da);
    }
    hipLaunchKernelGGL(dqrm::dedupe_finish_kernel, dim3(grid_for(max_n, dqrm::kSegThreads, 2), num_batches),
                       dim3(dqrm::kSegThreads), 0, st, da);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_dedupe(const dqrm_tables_t *tables, const int64_t *indices, const int64_t *offsets, int32_t batch,
                    int64_t num_indices, int32_t *sorted_pos, int64_t *uniq_rows, int32_t *seg_offsets,
                    int32_t *table_uniq_offsets, int32_t *num_unique, void *workspace, size_t workspace_bytes,
                    void *stream)
{
    dqrm_dedupe_batch_t b;
    b.indices = indices;
    b.offsets = offsets;
    b.num_indices = num_indices;
    b.sorted_pos = sorted_pos;
    b.uniq_rows = uniq_rows;
    b.seg_offsets = seg_offsets;
    b.table_uniq_offsets = table_uniq_offsets;
    b.num_unique = num_unique;
    b.workspace = workspace;
    b.max_table_lookups = 0;
    return dqrm_dedupe_multi(tables, batch, 1, &b, workspace_bytes, stream);
}

int32_t dqrm_segment_sum(const dqrm_tables_t *tables, int32_t batch, int64_t num_indices, const float *grad_out,
                         float *values, float *g_absmax, void *workspace, size_t workspace_bytes, void *stream)
{
    int64_t R = 0;
    int32_t rc = check_tables(tables, false, &R);
    if (rc != DQRM_OK) return rc;
    if (batch < 1 || num_indices < 0) return DQRM_ERR_INVALID_ARG;
    if (num_indices > kMaxIndices || (int64_t)batch * tables->num_tables > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    if (!grad_out || !values || !workspace) return DQRM_ERR_INVALID_ARG;
    if (!aligned(grad_out, 16) || !aligned(values, 16) || !aligned(workspace, 256)) return DQRM_ERR_INVALID_ARG;
    const int T = tables->num_tables, D = tables->dim;
    const WsLayout L = ws_layout(T, D, num_indices);
    if (workspace_bytes < L.total) return DQRM_ERR_WORKSPACE_TOO_SMALL;

    hipStream_t st = static_cast<hipStream_t>(stream);
    dqrm::SegArgs sa;
    sa.grad_out = grad_out;
    sa.ws = ws_views(workspace, L);
    sa.N = num_indices;
    sa.values = values;
    sa.g_absmax = g_absmax;
    sa.T = T;
    sa.B = batch;
    sa.D = D;
    const int G = pow2ceil(D / 4);
    // at most one lane group per four lookups (a window of the chunk list per workgroup, a few singles per group)
    const int grid_sum = grid_for((num_indices + 3) / 4 * G, dqrm::kSumThreads, dqrm::kSumBlocksPerCu);
    launch_segsum(G, dim3(grid_sum), st, sa);
    if (g_absmax)
        hipLaunchKernelGGL(dqrm::absmax_finalize_kernel, dim3((T + 255) / 256), dim3(256), 0, st, sa.ws.absmax_slots,
                           T, g_absmax);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_segment_sum_multi(const dqrm_tables_t *tables, int32_t batch, int32_t num_batches,
                               const dqrm_segsum_batch_t *batches, size_t workspace_bytes, void *stream)
{
    int64_t R = 0;
    int32_t rc = check_tables(tables, false, &R);
    if (rc != DQRM_OK) return rc;
    if (!batches || num_batches < 1 || batch < 1) return DQRM_ERR_INVALID_ARG;
    if (num_batches > DQRM_MAX_DEDUPE_BATCHES) return DQRM_ERR_UNSUPPORTED;
    if ((int64_t)batch * tables->num_tables > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    const int T = tables->num_tables, D = tables->dim;
    int64_t max_n = 0;
    bool any_absmax = false;
    for (int i = 0; i < num_batches; ++i) {
        const dqrm_segsum_batch_t &b = batches[i];
        if (b.num_indices < 0) return DQRM_ERR_INVALID_ARG;
        if (b.num_indices > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
        if (!b.grad_out || !b.values || !b.workspace) return DQRM_ERR_INVALID_ARG;
        if (!aligned(b.grad_out, 16) || !aligned(b.values, 16) || !aligned(b.workspace, 256)) return DQRM_ERR_INVALID_ARG;
        if (workspace_bytes < ws_layout(T, D, b.num_indices).total) return DQRM_ERR_WORKSPACE_TOO_SMALL;
        max_n = std::max(max_n, b.num_indices);
        any_absmax = any_absmax || b.g_absmax != nullptr;
    }
    dqrm::SegMulti sm;
    dqrm::AbsmaxMulti am;
    std::memset(&sm, 0, sizeof(sm));
    std::memset(&am, 0, sizeof(am));
    for (int i = 0; i < num_batches; ++i) {
        const dqrm_segsum_batch_t &b = batches[i];
        dqrm::SegArgs &sa = sm.b[i];
        sa.grad_out = b.grad_out;
        sa.ws = ws_views(b.workspace, ws_layout(T, D, b.num_indices));
        sa.N = b.num_indices;
        sa.values = b.values;
        sa.g_absmax = b.g_absmax;
        sa.T = T, sa.B = batch, sa.D = D;
        am.slots[i] = sa.ws.absmax_slots;
        am.g_absmax[i] = b.g_absmax;
    }
    am.T = T;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int G = pow2ceil(D / 4);
    const int grid_sum = grid_for((max_n + 3) / 4 * G, dqrm::kSumThreads, dqrm::kSumBlocksPerCu);
    launch_segsum_multi(G, dim3(grid_sum, num_batches), st, sm);
    if (any_absmax)
        hipLaunchKernelGGL(dqrm::absmax_finalize_multi_kernel, dim3((T + 255) / 256, num_batches), dim3(256), 0, st, am);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_embbag_bwd(const dqrm_tables_t *tables, const int64_t *indices, const int64_t *offsets, int32_t batch,
                        int64_t num_indices, const float *grad_out, int32_t *sorted_pos, int64_t *uniq_rows,
                        int32_t *seg_offsets, int32_t *table_uniq_offsets, int32_t *num_unique, float *values,
                        float *g_absmax, void *workspace, size_t workspace_bytes, void *stream)
{
    // validate everything before the first launch
    if (!grad_out || !values || !g_absmax) return DQRM_ERR_INVALID_ARG;
    if (!aligned(grad_out, 16) || !aligned(values, 16)) return DQRM_ERR_INVALID_ARG;
    int32_t rc = dqrm_dedupe(tables, indices, offsets, batch, num_indices, sorted_pos, uniq_rows, seg_offsets,
                             table_uniq_offsets, num_unique, workspace, workspace_bytes, stream);
    if (rc != DQRM_OK) return rc;
    return dqrm_segment_sum(tables, batch, num_indices, grad_out, values, g_absmax, workspace, workspace_bytes, stream);
}

int32_t dqrm_embbag_bwd_noalloc(const dqrm_tables_t *tables, const int64_t *indices, const int64_t *offsets,
                                int32_t batch, int64_t num_indices, const float *grad_out, int32_t *sorted_pos,
                                int64_t *uniq_rows, int32_t *seg_offsets, int32_t *table_uniq_offsets,
                                int32_t *num_unique, float *values, float *g_absmax, void *stream)
{
    // the size check needs only the shape: do it before anything touches the device
    if (!tables) return DQRM_ERR_INVALID_ARG;
    if (tables->num_tables < 1 || tables->dim < 1 || batch < 1 || num_indices < 0) return DQRM_ERR_INVALID_ARG;
    const size_t need = dqrm_embbag_bwd_workspace_bytes(tables->num_tables, tables->dim, batch, num_indices);
    if (need == 0) return DQRM_ERR_UNSUPPORTED;
    if (need > (size_t)DQRM_NOALLOC_SCRATCH_BYTES) {
        std::snprintf(t_hip_error, sizeof(t_hip_error),
                      "dqrm_embbag_bwd_noalloc: this shape needs %zu bytes of scratch, the built-in array holds %zu",
                      need, (size_t)DQRM_NOALLOC_SCRATCH_BYTES);
        return DQRM_ERR_SCRATCH_LIMIT;
    }
    // every GPU holds its own copy of the array at its own address: ask once per device, with that device current
    constexpr int kMaxDevices = 64;
    static void *dev_ptr[kMaxDevices] = {};
    static std::mutex mu;
    int dev = 0;
    DQRM_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return DQRM_ERR_UNSUPPORTED;
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!dev_ptr[dev]) {
            void *p = nullptr;
            DQRM_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (!p || !aligned(p, 256)) return hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
            dev_ptr[dev] = p;
        }
        ws = dev_ptr[dev];
    }
    // nothing in the workspace has to start at zero: the dedupe kernels write every counter and slot they or
    // the segment sums read, so the previous call's contents do not matter
    return dqrm_embbag_bwd(tables, indices, offsets, batch, num_indices, grad_out, sorted_pos, uniq_rows, seg_offsets,
                           table_uniq_offsets, num_unique, values, g_absmax, ws, (size_t)DQRM_NOALLOC_SCRATCH_BYTES, stream);
}

int32_t dqrm_grad_quant_int8(int32_t num_tables, int32_t dim, int64_t capacity, const float *values,
                             const int32_t *table_uniq_offsets, const float *g_absmax, int8_t *gq, float *g_scale,
                             void *stream)
{
    if (num_tables < 1 || dim < 1 || capacity < 0) return DQRM_ERR_INVALID_ARG;
    if (!values || !table_uniq_offsets || !g_absmax || !gq || !g_scale) return DQRM_ERR_INVALID_ARG;
    if (num_tables > DQRM_MAX_TABLES || dim % 8 != 0 || dim > DQRM_MAX_DIM) return DQRM_ERR_UNSUPPORTED;
    if (capacity > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    if (!aligned(values, 16) || !aligned(gq, 4)) return DQRM_ERR_INVALID_ARG;
    if (capacity * (dim / 4) > kMaxRowQuarters) return DQRM_ERR_UNSUPPORTED;
    dqrm::QuantArgs a;
    a.values = values;
    a.tuo = table_uniq_offsets;
    a.g_absmax = g_absmax;
    a.gq = gq;
    a.g_scale = g_scale;
    a.capacity = capacity;
    a.T = num_tables;
    a.D = dim;
    a.by_q4 = dqrm::FastDiv::make((unsigned)(dim / 4));
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(dqrm::grad_quant_kernel, dim3(grid_for(capacity * (dim / 4), dqrm::kEwThreads, 8)),
                       dim3(dqrm::kEwThreads), dqrm::TableLds::bytes(num_tables), st, a);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_grad_quant_int8_multi(int32_t num_tables, int32_t dim, int32_t num_blocks,
                                   const dqrm_quant_block_t *blocks, void *stream)
{
    if (num_tables < 1 || dim < 1 || !blocks || num_blocks < 1) return DQRM_ERR_INVALID_ARG;
    if (num_tables > DQRM_MAX_TABLES || dim % 8 != 0 || dim > DQRM_MAX_DIM) return DQRM_ERR_UNSUPPORTED;
    if (num_blocks > DQRM_MAX_DEDUPE_BATCHES) return DQRM_ERR_UNSUPPORTED;
    int64_t max_cap = 0;
    for (int i = 0; i < num_blocks; ++i) {
        const dqrm_quant_block_t &b = blocks[i];
        if (b.capacity < 0) return DQRM_ERR_INVALID_ARG;
        if (!b.values || !b.table_uniq_offsets || !b.g_absmax || !b.gq || !b.g_scale) return DQRM_ERR_INVALID_ARG;
        if (b.capacity > kMaxIndices || b.capacity * (dim / 4) > kMaxRowQuarters) return DQRM_ERR_UNSUPPORTED;
        if (!aligned(b.values, 16) || !aligned(b.gq, 4)) return DQRM_ERR_INVALID_ARG;
        max_cap = std::max(max_cap, b.capacity);
    }
    dqrm::QuantMulti qm;
    std::memset(&qm, 0, sizeof(qm));
    for (int i = 0; i < num_blocks; ++i) {
        const dqrm_quant_block_t &b = blocks[i];
        dqrm::QuantArgs &a = qm.b[i];
        a.values = b.values;
        a.tuo = b.table_uniq_offsets;
        a.g_absmax = b.g_absmax;
        a.gq = b.gq;
        a.g_scale = b.g_scale;
        a.capacity = b.capacity;
        a.T = num_tables;
        a.D = dim;
        a.by_q4 = dqrm::FastDiv::make((unsigned)(dim / 4));
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(dqrm::grad_quant_multi_kernel,
                       dim3(grid_for(max_cap * (dim / 4), dqrm::kEwThreads, 8), num_blocks), dim3(dqrm::kEwThreads),
                       dqrm::TableLds::bytes(num_tables), st, qm);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_sparse_update(const dqrm_tables_t *tables, int64_t capacity, const int64_t *uniq_rows,
                           const int32_t *table_uniq_offsets, const int8_t *gq, const float *g_scale, float lr,
                           void *stream)
{
    if (!gq || !aligned(gq, 4)) return DQRM_ERR_INVALID_ARG;
    return sparse_update_impl(tables, capacity, uniq_rows, table_uniq_offsets, gq, nullptr, g_scale, lr, stream);
}

int32_t dqrm_sparse_update_sums(const dqrm_tables_t *tables, int64_t capacity, const int64_t *uniq_rows,
                                const int32_t *table_uniq_offsets, const int32_t *sums, const float *g_scale,
                                float lr, void *stream)
{
    if (!sums || !aligned(sums, 16)) return DQRM_ERR_INVALID_ARG;
    return sparse_update_impl(tables, capacity, uniq_rows, table_uniq_offsets, nullptr, sums, g_scale, lr, stream);
}

size_t dqrm_sparse_merge_workspace_bytes(int32_t num_tables, int32_t dim, int32_t num_blocks, int64_t max_total)
{
    if (num_tables < 1 || num_tables > DQRM_MAX_TABLES || dim < 8 || dim > DQRM_MAX_DIM || dim % 8 != 0 ||
        num_blocks < 1 || num_blocks > DQRM_MAX_DEDUPE_BATCHES || max_total < 0 || max_total > kMaxIndices)
        return 0;
    return merge_layout(num_tables, max_total).total;
}

int32_t dqrm_sparse_merge(const dqrm_tables_t *tables, int32_t num_blocks, const dqrm_sparse_block_t *blocks,
                          int64_t max_total, int64_t *uniq_rows, int32_t *table_uniq_offsets, int32_t *num_unique,
                          int32_t *sums, void *workspace, size_t workspace_bytes, void *stream)
{
    int64_t R = 0;
    int32_t rc = check_tables(tables, false, &R);
    if (rc != DQRM_OK) return rc;
    if (!blocks || num_blocks < 1 || max_total < 0) return DQRM_ERR_INVALID_ARG;
    if (num_blocks > DQRM_MAX_DEDUPE_BATCHES || max_total > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    const int T = tables->num_tables, D = tables->dim;
    if (max_total * (D / 4) > kMaxRowQuarters) return DQRM_ERR_UNSUPPORTED;
    if (!uniq_rows || !table_uniq_offsets || !num_unique || !sums || !workspace) return DQRM_ERR_INVALID_ARG;
    if (!aligned(sums, 16) || !aligned(workspace, 256)) return DQRM_ERR_INVALID_ARG;
    dqrm::MergeArgs ma;
    std::memset(&ma, 0, sizeof(ma));
    int64_t max_cap = 0;
    for (int k = 0; k < num_blocks; ++k) {
        const dqrm_sparse_block_t &b = blocks[k];
        if (!b.uniq_rows || !b.table_uniq_offsets || !b.gq || !aligned(b.gq, 4) || b.capacity < 0)
            return DQRM_ERR_INVALID_ARG;
        if (b.capacity >= (1LL << dqrm::kMergeSrcBits)) return DQRM_ERR_UNSUPPORTED;
        ma.uniq_rows[k] = b.uniq_rows, ma.tuo[k] = b.table_uniq_offsets, ma.gq[k] = b.gq, ma.capacity[k] = b.capacity;
        if (b.capacity > max_cap) max_cap = b.capacity;
    }
    const MergeLayout L = merge_layout(T, max_total);
    if (workspace_bytes < L.total) return DQRM_ERR_WORKSPACE_TOO_SMALL;
    char *ws = static_cast<char *>(workspace);
    ma.n = num_blocks, ma.T = T, ma.D = D, ma.max_total = (int)max_total;
    ma.base = reinterpret_cast<int32_t *>(ws + L.off_base);
    ma.sorted_src = reinterpret_cast<int32_t *>(ws + L.off_src);
    ma.head = reinterpret_cast<int32_t *>(ws + L.off_head);
    ma.local_excl = reinterpret_cast<int32_t *>(ws + L.off_excl);
    ma.table_heads = reinterpret_cast<int32_t *>(ws + L.off_table_heads);
    ma.uniq_rows_out = uniq_rows, ma.tuo_out = table_uniq_offsets, ma.num_unique = num_unique, ma.sums = sums;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const int per_block = (int)((max_cap + dqrm::kMergeThreads - 1) / dqrm::kMergeThreads);
    hipLaunchKernelGGL(dqrm::merge_rank_kernel, dim3(per_block < 1 ? 1 : per_block, num_blocks), dim3(dqrm::kMergeThreads),
                       dqrm::merge_rank_lds_bytes(T, num_blocks), st, ma);
    hipLaunchKernelGGL(dqrm::merge_scan_kernel, dim3(T), dim3(dqrm::kMergeScanThreads), 0, st, ma);
    hipLaunchKernelGGL(dqrm::merge_sum_kernel, dim3(grid_for(max_total * (D / 4), dqrm::kMergeThreads, 8)),
                       dim3(dqrm::kMergeThreads), dqrm::merge_sum_lds_bytes(T), st, ma);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_quant_update(const dqrm_tables_t *tables, int64_t capacity, int64_t num_indices, const float *values,
                          const int64_t *uniq_rows, const int32_t *table_uniq_offsets, float *g_absmax, int8_t *gq,
                          float *g_scale, float lr, void *workspace, size_t workspace_bytes, void *stream)
{
    int64_t R = 0;
    int32_t rc = check_tables(tables, false, &R);
    if (rc != DQRM_OK) return rc;
    if (capacity < 0 || num_indices < 0 || !values || !uniq_rows || !table_uniq_offsets || !g_absmax || !gq ||
        !g_scale || !workspace)
        return DQRM_ERR_INVALID_ARG;
    if (capacity > kMaxIndices || num_indices > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    if (!aligned(values, 16) || !aligned(gq, 4) || !aligned(workspace, 256)) return DQRM_ERR_INVALID_ARG;
    if (capacity * (tables->dim / 4) > kMaxRowQuarters) return DQRM_ERR_UNSUPPORTED;
    const WsLayout L = ws_layout(tables->num_tables, tables->dim, num_indices);
    if (workspace_bytes < L.total) return DQRM_ERR_WORKSPACE_TOO_SMALL;
    dqrm::QuantUpdateArgs a;
    a.u.master = tables->master;
    a.u.packed = tables->packed;
    a.u.w_scale = tables->w_scale;
    a.u.row_offsets = tables->row_offsets_dev;
    a.u.uniq_rows = uniq_rows;
    a.u.tuo = table_uniq_offsets;
    a.u.gq = nullptr;
    a.u.sums = nullptr;
    a.u.g_scale = nullptr;
    a.u.capacity = capacity;
    a.u.lr = lr;
    a.u.T = tables->num_tables;
    a.u.D = tables->dim;
    a.u.by_q4 = dqrm::FastDiv::make((unsigned)(a.u.D / 4));
    a.values = values;
    a.absmax_slots = ws_views(workspace, L).absmax_slots;
    a.g_absmax = g_absmax;
    a.gq_out = gq;
    a.g_scale_out = g_scale;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(dqrm::quant_update_kernel, dim3(grid_for(capacity * (a.u.D / 4), dqrm::kEwThreads, 8)),
                       dim3(dqrm::kEwThreads), dqrm::TableLds::bytes(a.u.T), st, a);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

} // extern "C"

// ---- the dense part of the train step ---------------------------------------------
namespace {

constexpr int kMaxMlpLayers = 16;
constexpr int kDenseMaxSplits = dqrm::kSgdMaxSlices; // slices of the batch dimension in the weight-gradient products

struct DenseLayout {
    // activations: bot_act[l] = output of bottom layer l, R = interaction output, top_act[l] = output of top
    // layer l (the last one is the logit); gradients w.r.t. the layers' pre-activations: bot_dz[l], top_dz[l]
    // (the last top one is the loss gradient), dR w.r.t. the interaction output; per-layer slices of the split
    // weight-gradient products: bot_part[l], top_part[l]
    size_t bot_act[kMaxMlpLayers], top_act[kMaxMlpLayers], R;
    size_t bot_dz[kMaxMlpLayers], top_dz[kMaxMlpLayers], dR;
    size_t bot_part[kMaxMlpLayers], top_part[kMaxMlpLayers];
    // the quantised variants: fake-quantised weights (layers in flat order), flat FP32 gradients, per-tensor maxima
    size_t wq, grads, gmax;
    size_t loss_terms; // per-sample loss
    size_t total;
};

// flat parameter order (see dqrm_dense_quant_t): top layers, then bottom layers
int64_t dense_param_count(const dqrm_dense_model_t *m)
{
    int64_t p = 0;
    for (int l = 0; l < m->top_layers; ++l) p += (int64_t)m->top_dims[l + 1] * (m->top_dims[l] + 1);
    for (int l = 0; l < m->bot_layers; ++l) p += (int64_t)m->bot_dims[l + 1] * (m->bot_dims[l] + 1);
    return p;
}

// Slices of the batch dimension in the weight-gradient products (all layers share one launch): as many as bring
// the launch's wave tiles to about one per SIMD of the chip -- more slices only add partial tiles to write and to
// add up again (Kaggle model at batch 2048: 2 slices 185 us per step, 4: 188, 8: 189, 16: 192) -- with at least
// two reduction slabs per slice, and at least two slices (the kernel stores partial tiles only when the reduction is
// split; a slice may be empty).
int dense_splits(const dqrm_dense_model_t *m, int batch)
{
    int64_t tiles = 0;
    for (int l = 0; l < m->bot_layers; ++l) tiles += (int64_t)((m->bot_dims[l + 1] + 31) / 32) * ((m->bot_dims[l] + 1 + 31) / 32);
    for (int l = 0; l < m->top_layers; ++l) tiles += (int64_t)((m->top_dims[l + 1] + 31) / 32) * ((m->top_dims[l] + 1 + 31) / 32);
    const int64_t simds = (int64_t)num_cus() * 4;
    int64_t s = (simds + tiles / 2) / std::max<int64_t>(tiles, 1);
    s = std::min<int64_t>(s, batch / (2 * dqrm::kGemmBK));
    return (int)std::max<int64_t>(2, std::min<int64_t>(s, kDenseMaxSplits));
}

int32_t check_dense_model(const dqrm_dense_model_t *m, int32_t batch)
{
    if (!m || batch < 1) return DQRM_ERR_INVALID_ARG;
    if (m->num_dense < 1 || m->num_tables < 1 || m->dim < 1 || m->bot_layers < 1 || m->top_layers < 1)
        return DQRM_ERR_INVALID_ARG;
    if (!m->bot_dims || !m->bot_w || !m->bot_b || !m->top_dims || !m->top_w || !m->top_b) return DQRM_ERR_INVALID_ARG;
    if (m->bot_layers > kMaxMlpLayers || m->top_layers > kMaxMlpLayers) return DQRM_ERR_UNSUPPORTED;
    const int V = m->num_tables + 1;
    if (V > 64 || (int64_t)V * m->dim > dqrm::kInterMaxZ) return DQRM_ERR_UNSUPPORTED;
    if (m->bot_dims[0] != m->num_dense || m->bot_dims[m->bot_layers] != m->dim) return DQRM_ERR_INVALID_ARG;
    if (m->top_dims[0] != m->dim + V * (V - 1) / 2 || m->top_dims[m->top_layers] != 1) return DQRM_ERR_INVALID_ARG;
    for (int l = 0; l <= m->bot_layers; ++l)
        if (m->bot_dims[l] < 1 || m->bot_dims[l] > 65536) return DQRM_ERR_UNSUPPORTED;
    for (int l = 0; l <= m->top_layers; ++l)
        if (m->top_dims[l] < 1 || m->top_dims[l] > 65536) return DQRM_ERR_UNSUPPORTED;
    for (int l = 0; l < m->bot_layers; ++l)
        if (!m->bot_w[l] || !m->bot_b[l]) return DQRM_ERR_INVALID_ARG;
    for (int l = 0; l < m->top_layers; ++l)
        if (!m->top_w[l] || !m->top_b[l]) return DQRM_ERR_INVALID_ARG;
    if ((int64_t)batch * 65536 > kMaxIndices) return DQRM_ERR_UNSUPPORTED;
    return DQRM_OK;
}

DenseLayout dense_layout(const dqrm_dense_model_t *m, int32_t batch)
{
    DenseLayout L{};
    size_t o = 0;
    auto take = [&](size_t floats) {
        size_t at = o;
        o = align_up(o + floats * sizeof(float), 256);
        return at;
    };
    const size_t splits = (size_t)dense_splits(m, batch);
    for (int l = 0; l < m->bot_layers; ++l) {
        L.bot_act[l] = take((size_t)batch * m->bot_dims[l + 1]);
        L.bot_dz[l] = take((size_t)batch * m->bot_dims[l + 1]);
        L.bot_part[l] = take(splits * (size_t)m->bot_dims[l + 1] * (m->bot_dims[l] + 1));
    }
    L.R = take((size_t)batch * m->top_dims[0]);
    L.dR = take((size_t)batch * m->top_dims[0]);
    for (int l = 0; l < m->top_layers; ++l) {
        L.top_act[l] = take((size_t)batch * m->top_dims[l + 1]);
        L.top_dz[l] = take((size_t)batch * m->top_dims[l + 1]);
        L.top_part[l] = take(splits * (size_t)m->top_dims[l + 1] * (m->top_dims[l] + 1));
    }
    const size_t P = (size_t)dense_param_count(m);
    L.wq = take(P);
    L.grads = take(P);
    L.gmax = take((size_t)dqrm::kMaxGradTensors * dqrm::kGradMaxSlots * dqrm::kGradMaxStride);
    L.loss_terms = take((size_t)batch);
    L.total = o;
    return L;
}

// A_MODE / B_MODE: how A / B lie in memory and are read (dqrm::kOpRC: the reduction index is the unit-stride one;
// kOpWide, kOpWideVec: the 32-wide index i / j is).  One launch for all problems of the group.
template <int A_MODE, int B_MODE>
hipError_t launch_gemm_group(hipStream_t st, dqrm::GemmGroup &grp)
{
    int tiles = 0;
    for (int q = 0; q < grp.count; ++q) {
        dqrm::GemmArgs &g = grp.p[q];
        if (g.b_ones_last && B_MODE != dqrm::kOpWide) return hipErrorInvalidValue; // only that form serves the virtual column
        g.tile_begin = tiles;
        tiles += ((g.M + 31) / 32) * ((g.N + 31) / 32) * g.splits;
    }
    grp.total_tiles = tiles;
    if (tiles == 0) return hipSuccess;
    if (grp.count > 1) {
        hipLaunchKernelGGL((dqrm::gemm_wave_group_kernel<A_MODE, B_MODE>),
                           dim3((tiles + dqrm::kGemmWaves - 1) / dqrm::kGemmWaves), dim3(dqrm::kGemmThreads), 0, st, grp);
        return hipGetLastError();
    }
    dqrm::GemmOne one;
    one.p = grp.p[0];
    one.total_tiles = tiles;
    // A product with fewer tiles than the chip has SIMDs (4 per CU) leaves some of them idle: let 2 or 4 waves
    // share a tile, each with a slice of the reduction (at least one pair of slabs each), up to one wave per
    // SIMD.  (Measured: beyond that, slices cost more than they bring.)
    one.kslices = 1;
    if (one.p.splits == 1) {
        const int pairs = one.p.K / (2 * dqrm::kGemmBK);
        while (one.kslices < 4 && tiles * one.kslices * 2 <= num_cus() * 4 && pairs >= one.kslices * 2) one.kslices *= 2;
    }
    const int waves = tiles * one.kslices;
    hipLaunchKernelGGL((dqrm::gemm_wave_kernel<A_MODE, B_MODE>), dim3((waves + dqrm::kGemmWaves - 1) / dqrm::kGemmWaves),
                       dim3(dqrm::kGemmThreads), 0, st, one);
    return hipGetLastError();
}

// Y[B][out] = act(X[B][in] * W[out][in]^T + b)
hipError_t linear_fwd(hipStream_t st, const float *X, const float *W, const float *b, float *Y, int B, int in, int out,
                bool relu)
{
    dqrm::GemmGroup grp{};
    dqrm::GemmArgs &g = grp.p[0];
    grp.count = 1;
    g.A = X, g.a_si = in, g.a_sr = 1;
    g.B = W, g.b_sr = 1, g.b_sj = in;
    g.C = Y, g.c_si = out, g.c_sj = 1;
    g.M = B, g.N = out, g.K = in;
    g.bias = b, g.relu = relu ? 1 : 0, g.splits = 1, g.k_per_split = in;
    return launch_gemm_group<dqrm::kOpRC, dqrm::kOpRC>(st, grp);
}

// dX[B][in] = (dZ[B][out] * W[out][in]) masked by (mask[B][in] > 0)
hipError_t linear_bwd_input(hipStream_t st, const float *dZ, const float *W, const float *mask, float *dX, int B, int in,
                      int out)
{
    dqrm::GemmGroup grp{};
    dqrm::GemmArgs &g = grp.p[0];
    grp.count = 1;
    g.A = dZ, g.a_si = out, g.a_sr = 1;
    g.B = W, g.b_sr = in, g.b_sj = 1;
    g.C = dX, g.c_si = in, g.c_sj = 1;
    g.M = B, g.N = in, g.K = out;
    g.mask = mask, g.splits = 1, g.k_per_split = out;
    return launch_gemm_group<dqrm::kOpRC, dqrm::kOpWideVec>(st, grp);
}

// One layer's weight-gradient product  [dZ^T * X | dZ^T * 1]  ([out][in + 1], the last column is the bias
// gradient) with the batch dimension cut into `splits` slices: partials[s][out][in + 1].
dqrm::GemmArgs weight_grad_problem(const float *dZ, const float *X, float *partials, int B, int in, int out, int splits)
{
    int per = (B + splits - 1) / splits;
    per = (per + dqrm::kGemmBK - 1) / dqrm::kGemmBK * dqrm::kGemmBK;
    dqrm::GemmArgs g{};
    g.A = dZ, g.a_si = 1, g.a_sr = out;
    g.B = X, g.b_sr = in, g.b_sj = 1, g.b_ones_last = 1;
    g.M = out, g.N = in + 1, g.K = B;
    g.splits = splits; // exactly the slices the workspace holds; slices past the batch come out as zeros
    g.k_per_split = per, g.P = partials;
    return g;
}

} // namespace

extern "C" {

size_t dqrm_dense_workspace_bytes(const dqrm_dense_model_t *model, int32_t batch)
{
    if (check_dense_model(model, batch) != DQRM_OK) return 0;
    return dense_layout(model, batch).total;
}

int64_t dqrm_dense_param_count(const dqrm_dense_model_t *model)
{
    if (check_dense_model(model, 1) != DQRM_OK) return -1;
    return dense_param_count(model);
}

int32_t dqrm_dense_step(const dqrm_dense_model_t *m, int32_t batch, const float *dense_x, const float *emb_out,
                        const float *labels, float lr, float *loss, float *grad_emb, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    return dqrm_dense_step_quant(m, nullptr, batch, dense_x, emb_out, labels, lr, loss, grad_emb, workspace,
                                 workspace_bytes, stream);
}

int32_t dqrm_dense_step_quant(const dqrm_dense_model_t *m, const dqrm_dense_quant_t *quant, int32_t batch,
                              const float *dense_x, const float *emb_out, const float *labels, float lr, float *loss,
                              float *grad_emb, void *workspace, size_t workspace_bytes, void *stream)
{
    int32_t rc = check_dense_model(m, batch);
    if (rc != DQRM_OK) return rc;
    const int wbits = quant ? quant->weight_bits : 0, gbits = quant ? quant->grad_bits : 0;
    if ((wbits != 0 && wbits != 4 && wbits != 8) || (gbits != 0 && gbits != 8)) return DQRM_ERR_UNSUPPORTED;
    if (gbits == 8 && !quant->grad_scale) return DQRM_ERR_INVALID_ARG;
    if (quant && quant->grad_buffer && gbits != 0) return DQRM_ERR_UNSUPPORTED; // FP32 gradient buffers only
    if (!dense_x || !emb_out || !labels || !loss || !grad_emb || !workspace || !aligned(workspace, 256))
        return DQRM_ERR_INVALID_ARG;
    const DenseLayout L = dense_layout(m, batch);
    if (workspace_bytes < L.total) return DQRM_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    auto F = [&](size_t off) { return reinterpret_cast<float *>(ws + off); };
    const int B = batch, T = m->num_tables, D = m->dim;

    // ---- the weights the forward and the input gradients use: the model's, or their fake-quantised copies
    const float *top_wf[kMaxMlpLayers], *bot_wf[kMaxMlpLayers];
    for (int l = 0; l < m->top_layers; ++l) top_wf[l] = m->top_w[l];
    for (int l = 0; l < m->bot_layers; ++l) bot_wf[l] = m->bot_w[l];
    if (wbits) {
        float *wq = quant->wq ? quant->wq : F(L.wq);
        dqrm::FqGroup fq{};
        fq.qmax = (float)((1 << (wbits - 1)) - 1);
        int rows = 0;
        auto flush_fq = [&]() -> hipError_t {
            if (fq.count == 0) return hipSuccess;
            fq.total_rows = rows;
            hipLaunchKernelGGL(dqrm::mlp_fake_quant_kernel, dim3((rows + 3) / 4), dim3(256), 0, st, fq);
            fq.count = 0;
            rows = 0;
            return hipGetLastError();
        };
        auto add_fq = [&](const float *W, const float **wf, int in, int out) -> hipError_t {
            hipError_t e = hipSuccess;
            if (fq.count == dqrm::kGemmMaxGroup) e = flush_fq();
            dqrm::FqLayer &q = fq.l[fq.count++];
            q.W = W, q.Wq = wq, q.out = out, q.in = in, q.row_begin = rows;
            rows += out;
            *wf = wq;
            wq += (size_t)out * in;
            return e;
        };
        for (int l = 0; l < m->top_layers; ++l)
            DQRM_HIP_CHECK(add_fq(m->top_w[l], &top_wf[l], m->top_dims[l], m->top_dims[l + 1]));
        for (int l = 0; l < m->bot_layers; ++l)
            DQRM_HIP_CHECK(add_fq(m->bot_w[l], &bot_wf[l], m->bot_dims[l], m->bot_dims[l + 1]));
        DQRM_HIP_CHECK(flush_fq());
    }

    // ---- forward
    // The bottom MLP's last layer rides along in the interaction kernels when its input is short enough for their LDS
    // (its product is tiny: 64 -> 16 in the paper's Kaggle model), and a first layer with a short reduction (the
    // 13 dense features) has a kernel of its own: both are all launch cost as products on the matrix cores.
    const int bl_last = m->bot_layers - 1;
    const bool ride = m->bot_dims[bl_last] <= dqrm::kInterMaxLinK;
    const float *x = dense_x;
    for (int l = 0; l < m->bot_layers - (ride ? 1 : 0); ++l) {
        const int in = m->bot_dims[l], out = m->bot_dims[l + 1];
        if (in <= dqrm::kSmallKMax && out % 4 == 0 && aligned(m->bot_b[l], 16)) {
            dqrm::SmallKArgs sk{};
            sk.X = x, sk.W = bot_wf[l], sk.bias = m->bot_b[l], sk.Y = F(L.bot_act[l]), sk.B = B, sk.N = out, sk.K = in, sk.relu = 1;
            hipLaunchKernelGGL(dqrm::linear_small_k_kernel, dim3((B + dqrm::kSmallKSamples - 1) / dqrm::kSmallKSamples),
                               dim3(dqrm::kSmallKThreads), 0, st, sk);
            DQRM_HIP_CHECK(hipGetLastError());
        } else {
            DQRM_HIP_CHECK(linear_fwd(st, x, bot_wf[l], m->bot_b[l], F(L.bot_act[l]), B, in, out, true));
        }
        x = F(L.bot_act[l]);
    }
    dqrm::InteractArgs ia{};
    ia.bot = ride ? F(L.bot_act[bl_last]) : x, ia.emb = emb_out, ia.R = F(L.R), ia.B = B, ia.T = T, ia.D = D;
    if (ride) {
        ia.lin_x = x, ia.lin_w = bot_wf[bl_last], ia.lin_b = m->bot_b[bl_last], ia.lin_y = F(L.bot_act[bl_last]);
        ia.lin_k = m->bot_dims[bl_last];
    }
    hipLaunchKernelGGL(dqrm::interact_fwd_kernel, dim3(B), dim3(dqrm::kInterThreads),
                       dqrm::interact_lds_bytes(T, D, false, ride ? ia.lin_k : 0), st, ia);
    x = F(L.R);
    const int last = m->top_layers - 1;
    for (int l = 0; l < last; ++l) {
        DQRM_HIP_CHECK(linear_fwd(st, x, top_wf[l], m->top_b[l], F(L.top_act[l]), B, m->top_dims[l], m->top_dims[l + 1], true));
        x = F(L.top_act[l]);
    }
    // the last layer (one output), the loss, and the gradient back to that layer's input in one kernel
    unsigned *gmax = reinterpret_cast<unsigned *>(ws + L.gmax);
    dqrm::HeadArgs ha{};
    ha.X = x, ha.w = top_wf[last], ha.bias = m->top_b[last], ha.y = labels;
    ha.z = F(L.top_act[last]), ha.dz = F(L.top_dz[last]), ha.terms = F(L.loss_terms);
    ha.dX = last > 0 ? F(L.top_dz[last - 1]) : F(L.dR);
    ha.relu_input = last > 0; // the input of top layer l > 0 is a ReLU output; the interaction output is not
    ha.B = B, ha.in = m->top_dims[last];
    ha.zero = gmax, ha.nzero = gbits ? dqrm::kMaxGradTensors * dqrm::kGradMaxSlots : 0, ha.zstride = dqrm::kGradMaxStride;
    hipLaunchKernelGGL(dqrm::head_kernel, dim3((B + 3) / 4), dim3(256), 0, st, ha);
    DQRM_HIP_CHECK(hipGetLastError());

    // ---- backward: the chain of input gradients first (dZ = gradient w.r.t. a layer's pre-activation) ...
    for (int l = last - 1; l >= 0; --l) {
        const float *in_act = l > 0 ? F(L.top_act[l - 1]) : F(L.R);
        float *dX = l > 0 ? F(L.top_dz[l - 1]) : F(L.dR);
        DQRM_HIP_CHECK(linear_bwd_input(st, F(L.top_dz[l]), top_wf[l], l > 0 ? in_act : nullptr, dX, B,
                                        m->top_dims[l], m->top_dims[l + 1]));
    }
    const float *bot_out = F(L.bot_act[bl_last]);
    ia.bot = bot_out, ia.dR = F(L.dR), ia.dbot = F(L.bot_dz[bl_last]), ia.demb = grad_emb, ia.bot_mask = bot_out;
    const bool ride_back = ride && bl_last > 0; // (a first layer's input gradient is not needed)
    if (ride_back) ia.lin_mask = F(L.bot_act[bl_last - 1]), ia.lin_dx = F(L.bot_dz[bl_last - 1]);
    hipLaunchKernelGGL(dqrm::interact_bwd_kernel, dim3(B), dim3(dqrm::kInterThreads), dqrm::interact_lds_bytes(T, D, true), st,
                       ia);
    for (int l = bl_last - (ride_back ? 1 : 0); l > 0; --l)
        DQRM_HIP_CHECK(linear_bwd_input(st, F(L.bot_dz[l]), bot_wf[l], F(L.bot_act[l - 1]), F(L.bot_dz[l - 1]), B,
                                        m->bot_dims[l], m->bot_dims[l + 1]));

    // ... then every layer's weight gradient in one launch and the SGD step in another (the input gradients
    // above used the weights of before the step)
    const int splits = dense_splits(m, B);
    dqrm::GemmGroup wg{};
    dqrm::SgdGroup sg{};
    sg.lr = lr;
    if (quant && quant->grad_buffer)
        sg.buffer = quant->grad_buffer, sg.buffer_add = quant->buffer_add != 0, sg.buffer_update = quant->buffer_update != 0;
    if (gbits) {
        sg.grads = quant->grads ? quant->grads : F(L.grads);
        sg.err = quant->grad_error;
        sg.codes = quant->grad_codes;
        sg.gmax_bits = gmax;
        sg.grad_scale = quant->grad_scale;
    }
    long long flat = 0;
    int tensor = 0;
    hipError_t launch_err = hipSuccess;
    auto flush = [&](bool ends_step) {
        if (wg.count == 0 && !ends_step) return;
        if (ends_step) sg.loss_terms = F(L.loss_terms), sg.loss = loss, sg.batch = B; // one more block
        hipError_t e = launch_gemm_group<dqrm::kOpWide, dqrm::kOpWide>(st, wg);
        if (e != hipSuccess && launch_err == hipSuccess) launch_err = e;
        const unsigned blocks = (unsigned)std::min<long long>((sg.total + 255) / 256, 2048);
        const dim3 last_grid(blocks + (ends_step ? 1u : 0u));
        if (gbits) {
            if (blocks) hipLaunchKernelGGL(dqrm::grad_sum_absmax_kernel, dim3(blocks), dim3(256), 0, st, sg);
            hipLaunchKernelGGL(dqrm::grad_quant_ec_kernel, last_grid, dim3(256), 0, st, sg);
        } else {
            hipLaunchKernelGGL(dqrm::sgd_from_partials_kernel, last_grid, dim3(256), 0, st, sg);
        }
        e = hipGetLastError();
        if (e != hipSuccess && launch_err == hipSuccess) launch_err = e;
        wg.count = 0;
        sg.count = 0;
        sg.total = 0;
    };
    auto add_layer = [&](const float *dZ, const float *X, float *W, float *b, float *part, int in, int out) {
        if (wg.count == dqrm::kGemmMaxGroup) flush(false);
        const dqrm::GemmArgs g = weight_grad_problem(dZ, X, part, B, in, out, splits);
        wg.p[wg.count++] = g;
        dqrm::SgdLayer &s = sg.l[sg.count++];
        s.P = part, s.W = W, s.b = b, s.S = g.splits, s.out = out, s.in = in, s.elem_begin = sg.total;
        s.flat_begin = flat, s.tensor0 = tensor;
        sg.total += (long long)out * (in + 1);
        flat += (long long)out * (in + 1);
        tensor += 2;
    };
    for (int l = 0; l < m->top_layers; ++l)
        add_layer(F(L.top_dz[l]), l > 0 ? F(L.top_act[l - 1]) : F(L.R), m->top_w[l], m->top_b[l], F(L.top_part[l]),
                  m->top_dims[l], m->top_dims[l + 1]);
    for (int l = 0; l < m->bot_layers; ++l)
        add_layer(F(L.bot_dz[l]), l > 0 ? F(L.bot_act[l - 1]) : dense_x, m->bot_w[l], m->bot_b[l], F(L.bot_part[l]),
                  m->bot_dims[l], m->bot_dims[l + 1]);
    flush(true);
    DQRM_HIP_CHECK(launch_err);
    DQRM_HIP_CHECK(hipGetLastError());
    return DQRM_OK;
}

int32_t dqrm_check_status(void *stream, int32_t *first_bad_table, int64_t *first_bad_index)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    DQRM_HIP_CHECK(hipStreamSynchronize(st));
    dqrm::DeviceStatus h;
    DQRM_HIP_CHECK(hipMemcpyFromSymbol(&h, HIP_SYMBOL(dqrm::g_status), sizeof(h), 0, hipMemcpyDeviceToHost));
    if (h.code != 0) {
        dqrm::DeviceStatus z{0, 0, 0};
        DQRM_HIP_CHECK(hipMemcpyToSymbol(HIP_SYMBOL(dqrm::g_status), &z, sizeof(z), 0, hipMemcpyHostToDevice));
    }
    if (first_bad_table) *first_bad_table = h.code ? h.table : -1;
    if (first_bad_index) *first_bad_index = h.code ? h.value : -1;
    return h.code;
}


} // extern "C"
