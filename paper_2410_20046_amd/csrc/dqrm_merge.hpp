// Merging sparse gradient blocks (simulated data parallelism on one device, the appendix
// "Simulated Data Parallelism Environment": the gradients of several micro-batches
// are added into one buffer before the weights are updated; the same operation
// adds the integer gradients that an all-reduce would deliver, distributed-training
// appendix).  A block is one micro-batch's sparse gradient after INT8 quantisation:
// table-local unique rows, per-table offsets, INT8 codes.  The result is the union
// of the rows with the codes added as 32-bit integers - exact, so no order matters.
//
// Three steps: merge_layout_kernel lays the blocks' rows out table by table (block
// after block inside a table) with a CSR over (table, block) and remembers where
// every row came from; the sort-and-segment kernels of dqrm_dedupe run on that
// list (one "bag" per block); merge_sum_kernel adds, for every unique row, the
// code rows of the segment's members.
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

constexpr int kMergeSrcBits = 28; // a source word = block << 28 | row inside the block

struct MergeArgs {
    const int64_t *uniq_rows[DQRM_MAX_DEDUPE_BATCHES];
    const int32_t *tuo[DQRM_MAX_DEDUPE_BATCHES];
    const int8_t *gq[DQRM_MAX_DEDUPE_BATCHES];
    int64_t capacity[DQRM_MAX_DEDUPE_BATCHES]; // rows allocated per block (< 2^28)
    int n, T, D;
    int64_t max_total;    // rows allocated in the lists below and in the outputs
    int64_t *cat_rows;    // [max_total] the blocks' rows, table-major
    int64_t *cat_offsets; // [T * n + 1] piece (t, k) = cat_rows[cat_offsets[t * n + k] .. cat_offsets[t * n + k + 1])
    int32_t *cat_src;     // [max_total] source word of every entry of cat_rows
    const int32_t *sorted_pos;  // from the sort: position in cat_rows of every sorted entry
    const int32_t *seg_offsets; // [U + 1] (the last entry is not used: the list may be shorter than max_total)
    const int32_t *num_unique;
    int32_t *sums;        // [max_total][D] out
};

// rows of piece q = (table q / n, block q % n), or 0 if the block's offsets are unusable
__device__ __forceinline__ int merge_piece_count(const MergeArgs &a, int q, int *begin)
{
    const int t = q / a.n, k = q - t * a.n;
    const int b = a.tuo[k][t], e = a.tuo[k][t + 1];
    *begin = b;
    if (b < 0 || e < b || (int64_t)e > a.capacity[k]) return -1;
    return e - b;
}

__global__ __launch_bounds__(256) void merge_layout_kernel(MergeArgs a)
{
    __shared__ long long s_part[256];
    const int p = blockIdx.x, pieces = a.T * a.n;
    // first entry of this piece = rows of all pieces before it (every workgroup adds them up itself: T * n is small)
    long long before = 0;
    for (int q = threadIdx.x; q < p; q += 256) {
        int b;
        const int c = merge_piece_count(a, q, &b);
        before += c > 0 ? c : 0;
    }
    s_part[threadIdx.x] = before;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) s_part[threadIdx.x] += s_part[threadIdx.x + w];
        __syncthreads();
    }
    long long start = s_part[0];
    int begin;
    int cnt = merge_piece_count(a, p, &begin);
    const int t = p / a.n, k = p - t * a.n;
    if (cnt < 0) {
        if (threadIdx.x == 0) report(DQRM_ERR_BAD_OFFSETS, t, k);
        cnt = 0;
    }
    if (start + cnt > a.max_total) { // the outputs cannot hold the blocks: what does not fit is left out
        if (threadIdx.x == 0) report(DQRM_ERR_CAPACITY, t, start + cnt);
        start = start < a.max_total ? start : a.max_total;
        cnt = (int)(a.max_total - start);
    }
    if (threadIdx.x == 0) {
        a.cat_offsets[p] = start;
        if (p == pieces - 1) a.cat_offsets[pieces] = start + cnt;
    }
    const int64_t *rows = a.uniq_rows[k] + begin;
    for (int i = threadIdx.x; i < cnt; i += 256) {
        a.cat_rows[start + i] = rows[i];
        a.cat_src[start + i] = (int32_t)(((unsigned)k << kMergeSrcBits) | (unsigned)(begin + i));
    }
}

__global__ __launch_bounds__(256) void merge_sum_kernel(MergeArgs a)
{
    __shared__ const int *s_gq[DQRM_MAX_DEDUPE_BATCHES];
    if (threadIdx.x < DQRM_MAX_DEDUPE_BATCHES)
        s_gq[threadIdx.x] = reinterpret_cast<const int *>(a.gq[threadIdx.x < (unsigned)a.n ? threadIdx.x : 0]);
    __syncthreads();
    const int q4 = a.D / 4;
    const long long total_in = a.cat_offsets[a.T * a.n];
    long long U = *a.num_unique;
    U = U < 0 ? 0 : (U > a.max_total ? a.max_total : U);
    const long long total = U * q4;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const long long u = e / q4;
        const int c4 = (int)(e - u * q4);
        long long beg = a.seg_offsets[u], end = u + 1 < U ? (long long)a.seg_offsets[u + 1] : total_in;
        beg = beg < 0 ? 0 : beg;
        end = end > total_in ? total_in : end;
        int4 s = make_int4(0, 0, 0, 0);
        for (long long p = beg; p < end; ++p) {
            int pos = a.sorted_pos[p];
            pos = pos < 0 ? 0 : (pos >= total_in ? (int)(total_in - 1) : pos);
            const unsigned src = (unsigned)a.cat_src[pos];
            const unsigned k = src >> kMergeSrcBits, idx = src & ((1u << kMergeSrcBits) - 1u);
            const int word = s_gq[k][(long long)idx * q4 + c4];
            s.x += (int)(signed char)(word & 0xFF);
            s.y += (int)(signed char)((word >> 8) & 0xFF);
            s.z += (int)(signed char)((word >> 16) & 0xFF);
            s.w += word >> 24;
        }
        reinterpret_cast<int4 *>(a.sums)[e] = s;
    }
}

} // namespace dqrm
