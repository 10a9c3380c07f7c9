// Merging sparse gradient blocks (simulated data parallelism on one device, the appendix
// "Simulated Data Parallelism Environment": the gradients of several micro-batches
// are added into one buffer before the weights are updated; the same operation
// adds the integer gradients that an all-reduce would deliver, distributed-training
// appendix).  A block is one micro-batch's sparse gradient after INT8 quantisation:
// table-local unique rows (ascending inside each table), per-table offsets, INT8
// codes.  The result is the union of the rows, table by table in ascending order,
// with the codes added as 32-bit integers - exact, so no order matters.
//
// The blocks are sorted already, so nothing is sorted again: the place of a row in
// the merged list of its table is its own index plus, for every other block, the
// number of that block's rows below it (a binary search; equal rows of earlier
// blocks count as below).  Every row of every block finds its place on its own, so
// the whole chip works on the merge, not one workgroup per table.
//   merge_rank_kernel   place of every block row, source word and "first of its row" flag
//   merge_scan_kernel   per table: number of first-of-row flags before each place
//   merge_sum_kernel    per unique row: the members' code words added up
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

constexpr int kMergeSrcBits = 28; // a source word = block << 28 | row inside the block
constexpr int kMergeThreads = 256;
constexpr int kMergeWaves = kMergeThreads / kWave;
constexpr int kMergeBlocks = DQRM_MAX_DEDUPE_BATCHES;

struct MergeArgs {
    const int64_t *uniq_rows[kMergeBlocks];
    const int32_t *tuo[kMergeBlocks];
    const int8_t *gq[kMergeBlocks];
    int64_t capacity[kMergeBlocks]; // rows allocated per block (< 2^28)
    int n, T, D;
    int max_total;        // rows allocated in the lists below and in the outputs
    // workspace
    int32_t *base;        // [T + 1] first place of each table in the merged list
    int32_t *sorted_src;  // [max_total] source word of the block row at each place
    int32_t *head;        // [max_total] 1: no earlier block has this row (the place starts a unique row)
    int32_t *local_excl;  // [max_total] flags before this place inside its table
    int32_t *table_heads; // [T] unique rows per table
    // outputs
    int64_t *uniq_rows_out; // [max_total]
    int32_t *tuo_out;       // [T + 1]
    int32_t *num_unique;    // [1]
    int32_t *sums;          // [max_total][D]
};

// dynamic LDS of merge_rank_kernel: the blocks' table offsets and the merged list's table offsets
inline size_t merge_rank_lds_bytes(int T, int n) { return sizeof(int) * ((size_t)n * (T + 1) + (size_t)(T + 1)); }
// ... of merge_sum_kernel: the merged list's table offsets by place and by unique row
inline size_t merge_sum_lds_bytes(int T) { return sizeof(int) * 2 * (size_t)(T + 1); }

// exclusive scan of v[0 .. count) (LDS) into out[0 .. count], by the whole block, out[count] = sum clamped to `cap`
__device__ __forceinline__ void merge_block_scan(const int *v, int *out, int count, int cap, int *s_w)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    int carry = 0;
    for (int c0 = 0; c0 < count; c0 += kMergeThreads) {
        const int i = c0 + (int)threadIdx.x;
        const int x = i < count ? v[i] : 0;
        int total;
        const int ex = block_excl_scan_add<kMergeWaves>(x, lane, wave, s_w, &total);
        if (i < count) out[i] = min(carry + ex, cap);
        carry = min(carry + total, cap);
        __syncthreads();
    }
    if (threadIdx.x == 0) out[count] = carry;
    __syncthreads();
}

__global__ __launch_bounds__(kMergeThreads) void merge_rank_kernel(MergeArgs a)
{
    extern __shared__ int merge_lds[];
    __shared__ int s_bad[kMergeBlocks];
    __shared__ int s_w[kMergeWaves];
    __shared__ int s_tot[DQRM_MAX_TABLES];
    const int T = a.T, n = a.n, k = blockIdx.y;
    int *s_tuo = merge_lds;             // [n][T + 1]
    int *s_base = merge_lds + n * (T + 1); // [T + 1]
    for (int e = threadIdx.x; e < n * (T + 1); e += kMergeThreads) s_tuo[e] = a.tuo[e / (T + 1)][e % (T + 1)];
    if (threadIdx.x < kMergeBlocks) s_bad[threadIdx.x] = 0;
    __syncthreads();
    // a block whose offsets do not start at 0, go backwards or pass its capacity contributes nothing
    for (int e = threadIdx.x; e < n * T; e += kMergeThreads) {
        const int j = e / T, t = e - j * T;
        const int b = s_tuo[j * (T + 1) + t], en = s_tuo[j * (T + 1) + t + 1];
        if ((t == 0 && b != 0) || en < b || (int64_t)en > a.capacity[j]) s_bad[j] = 1;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < n * (T + 1); e += kMergeThreads)
        if (s_bad[e / (T + 1)]) s_tuo[e] = 0;
    if (blockIdx.x == 0 && k == 0 && threadIdx.x < (unsigned)n && s_bad[threadIdx.x])
        report(DQRM_ERR_BAD_OFFSETS, 0, threadIdx.x);
    __syncthreads();
    // where each table starts in the merged list
    for (int t = threadIdx.x; t < T; t += kMergeThreads) {
        int c = 0;
        for (int j = 0; j < n; ++j) c += s_tuo[j * (T + 1) + t + 1] - s_tuo[j * (T + 1) + t];
        s_tot[t] = c;
    }
    __syncthreads();
    merge_block_scan(s_tot, s_base, T, 0x7FFFFFFF, s_w);
    if (blockIdx.x == 0 && k == 0) {
        for (int t = threadIdx.x; t <= T; t += kMergeThreads) a.base[t] = min(s_base[t], a.max_total);
        if (threadIdx.x == 0 && s_base[T] > a.max_total) report(DQRM_ERR_CAPACITY, 0, s_base[T]);
    }

    const int *my = s_tuo + k * (T + 1);
    const int i = (int)blockIdx.x * kMergeThreads + (int)threadIdx.x;
    const bool live = i < my[T];
    // (a thread without a row goes through the searches with empty ranges: the loop bounds stay wave-uniform)
    const int t = live ? table_of(my, T, i) : 0;
    const int64_t r = live ? a.uniq_rows[k][i] : 0;
    if (live && i > my[t] && a.uniq_rows[k][i - 1] >= r) report(DQRM_ERR_BAD_OFFSETS, t, i); // not ascending
    int lo[kMergeBlocks], hi[kMergeBlocks];
#pragma unroll
    for (int j = 0; j < kMergeBlocks; ++j) {
        const bool on = live && j < n && j != k;
        lo[j] = on ? s_tuo[j * (T + 1) + t] : 0;
        hi[j] = on ? s_tuo[j * (T + 1) + t + 1] : 0;
    }
    // lower bound of r in every other block's rows of table t, all searches in step
    for (int step = 0; step < 32; ++step) {
        bool any = false;
#pragma unroll
        for (int j = 0; j < kMergeBlocks; ++j) any |= lo[j] < hi[j];
        if (!__any(any)) break;
        int64_t v[kMergeBlocks];
        int mid[kMergeBlocks];
#pragma unroll
        for (int j = 0; j < kMergeBlocks; ++j) {
            mid[j] = (lo[j] + hi[j]) >> 1;
            v[j] = (j < n && lo[j] < hi[j]) ? a.uniq_rows[j][mid[j]] : 0;
        }
#pragma unroll
        for (int j = 0; j < kMergeBlocks; ++j) {
            if (lo[j] < hi[j]) {
                if (v[j] < r)
                    lo[j] = mid[j] + 1;
                else
                    hi[j] = mid[j];
            }
        }
    }
    int place = i - my[t];
    bool first = true;
#pragma unroll
    for (int j = 0; j < kMergeBlocks; ++j) {
        if (live && j < n && j != k) {
            const int beg = s_tuo[j * (T + 1) + t], end = s_tuo[j * (T + 1) + t + 1];
            const bool present = lo[j] < end && a.uniq_rows[j][lo[j]] == r;
            place += lo[j] - beg + ((j < k && present) ? 1 : 0);
            if (j < k && present) first = false;
        }
    }
    if (!live) return;
    const long long P = (long long)s_base[t] + place;
    if (P >= a.max_total) return; // reported above
    a.sorted_src[P] = (int32_t)(((unsigned)k << kMergeSrcBits) | (unsigned)i);
    a.head[P] = first ? 1 : 0;
}

constexpr int kMergeScanThreads = 1024, kMergeScanPer = 4;

__global__ __launch_bounds__(kMergeScanThreads) void merge_scan_kernel(MergeArgs a)
{
    __shared__ int s_w[kMergeScanThreads / kWave];
    const int t = blockIdx.x;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int b0 = a.base[t], b1 = a.base[t + 1];
    int carry = 0;
    for (int c0 = b0; c0 < b1; c0 += kMergeScanThreads * kMergeScanPer) {
        const int P0 = c0 + (int)threadIdx.x * kMergeScanPer; // kMergeScanPer consecutive places per thread
        int h[kMergeScanPer], mine = 0;
#pragma unroll
        for (int q = 0; q < kMergeScanPer; ++q) {
            h[q] = a.head[min(P0 + q, b1 - 1)] != 0 && P0 + q < b1 ? 1 : 0;
            mine += h[q];
        }
        int total;
        int ex = carry + block_excl_scan_add<kMergeScanThreads / kWave>(mine, lane, wave, s_w, &total);
#pragma unroll
        for (int q = 0; q < kMergeScanPer; ++q) {
            if (P0 + q < b1) a.local_excl[P0 + q] = ex;
            ex += h[q];
        }
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) a.table_heads[t] = carry;
}

__global__ __launch_bounds__(kMergeThreads) void merge_sum_kernel(MergeArgs a)
{
    extern __shared__ int merge_lds[];
    __shared__ const int *s_gq[kMergeBlocks];
    __shared__ const int64_t *s_rows[kMergeBlocks];
    __shared__ int s_cap[kMergeBlocks];
    __shared__ int s_w[kMergeWaves];
    __shared__ int s_heads[DQRM_MAX_TABLES];
    const int T = a.T;
    int *s_base = merge_lds, *s_tuo = merge_lds + (T + 1);
    if (threadIdx.x < kMergeBlocks) {
        const int j = threadIdx.x < (unsigned)a.n ? threadIdx.x : 0;
        s_gq[threadIdx.x] = reinterpret_cast<const int *>(a.gq[j]);
        s_rows[threadIdx.x] = a.uniq_rows[j];
        s_cap[threadIdx.x] = threadIdx.x < (unsigned)a.n ? (int)a.capacity[j] : 0;
    }
    for (int t = threadIdx.x; t <= T; t += kMergeThreads) s_base[t] = a.base[t];
    for (int t = threadIdx.x; t < T; t += kMergeThreads) s_heads[t] = a.table_heads[t];
    __syncthreads();
    merge_block_scan(s_heads, s_tuo, T, a.max_total, s_w);
    if (blockIdx.x == 0) {
        for (int t = threadIdx.x; t <= T; t += kMergeThreads) a.tuo_out[t] = s_tuo[t];
        if (threadIdx.x == 0) *a.num_unique = s_tuo[T];
    }
    const int q4 = a.D / 4;
    const long long total = (long long)s_base[T] * q4;
    for (long long e = (long long)blockIdx.x * kMergeThreads + threadIdx.x; e < total;
         e += (long long)gridDim.x * kMergeThreads) {
        const int P = (int)(e / q4), c4 = (int)(e - (long long)P * q4);
        if (a.head[P] == 0) continue;
        const int t = table_of(s_base, T, P);
        const int u = s_tuo[t] + a.local_excl[P];
        if (u < 0 || u >= a.max_total) continue;
        const int end = s_base[t + 1];
        // the row's members: this place and the following ones up to the next flag (one per block at most);
        // flags, source words and then code words are requested together, places past the row re-read its first
        int hd[kMergeBlocks], src[kMergeBlocks];
#pragma unroll
        for (int m = 0; m < kMergeBlocks; ++m) {
            const int Q = min(P + m, end - 1);
            hd[m] = a.head[Q];
            src[m] = a.sorted_src[Q];
        }
        int members = 1;
#pragma unroll
        for (int m = 1; m < kMergeBlocks; ++m)
            if (members == m && P + m < end && hd[m] == 0) members = m + 1;
        int word[kMergeBlocks];
        bool ok[kMergeBlocks];
#pragma unroll
        for (int m = 0; m < kMergeBlocks; ++m) {
            const unsigned k = (unsigned)src[m] >> kMergeSrcBits, idx = (unsigned)src[m] & ((1u << kMergeSrcBits) - 1u);
            ok[m] = m < members && k < (unsigned)a.n && idx < (unsigned)s_cap[k]; // (else: a place no valid block row claimed)
            const unsigned kk = ok[m] ? k : (unsigned)src[0] >> kMergeSrcBits;
            const unsigned ii = ok[m] ? idx : (unsigned)src[0] & ((1u << kMergeSrcBits) - 1u);
            word[m] = 0;
            if (ok[0]) word[m] = s_gq[kk][(long long)ii * q4 + c4];
        }
        int4 s = make_int4(0, 0, 0, 0);
#pragma unroll
        for (int m = 0; m < kMergeBlocks; ++m) {
            if (ok[m]) {
                s.x += (int)(signed char)(word[m] & 0xFF);
                s.y += (int)(signed char)((word[m] >> 8) & 0xFF);
                s.z += (int)(signed char)((word[m] >> 16) & 0xFF);
                s.w += word[m] >> 24;
            }
        }
        long long row = 0;
        if (ok[0] && c4 == 0) row = s_rows[(unsigned)src[0] >> kMergeSrcBits][(unsigned)src[0] & ((1u << kMergeSrcBits) - 1u)];
        reinterpret_cast<int4 *>(a.sums)[(long long)u * q4 + c4] = s;
        if (c4 == 0) a.uniq_rows_out[u] = row;
    }
}

} // namespace dqrm
