// Forward: gather -> INT4 fake-quant -> sum-pool (Sec. 3.1 and Sec. 4.1 of the paper).
//
// A workgroup owns kFwdTile consecutive output slots (slot = b * T + t, i.e. a
// contiguous piece of `out`).  It works in three phases, each one memory round
// trip deep, so the dependent chain offsets -> index -> row is paid once per
// workgroup and not once per bag:
//   A  thread i reads the extent of slot i's bag and the bag's first index,
//      checks them, and leaves the row address and the table scale in LDS;
//   B  groups of G = pow2ceil(D/4) lanes walk the slots; lane l of a group owns
//      columns 4l..4l+3 (one 16-byte access per row).  The first rows of a whole
//      batch of slots are requested before any is used;
//   C  the bag's remaining lookups (none in the usual one-index-per-bag batch)
//      are added in order, and the pooled row is stored.
// The per-column sum is the plain left-to-right sum over the bag, so no
// cross-lane reduction is needed and the result does not depend on the mapping.
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

#ifndef DQRM_FWD_TILE
#define DQRM_FWD_TILE 128
#endif
#ifndef DQRM_FWD_BATCH
#define DQRM_FWD_BATCH 16
#endif
constexpr int kFwdTile = DQRM_FWD_TILE;   // output slots per workgroup
constexpr int kFwdThreads = kFwdTile;     // phase A is one slot per thread
constexpr int kFwdBatch = DQRM_FWD_BATCH; // first rows in flight per lane

struct FwdArgs {
    const float *master;
    const uint8_t *packed;
    const float *w_scale;
    const int64_t *row_offsets;
    const int64_t *indices;
    const int64_t *offsets;
    float *out;
    int8_t *codes;
    int64_t num_indices;
    int64_t num_bags; // T * B
    int T, B, D;
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

// codes of 4 consecutive elements of one row, as floats
template <bool PACKED>
__device__ __forceinline__ float4 load_codes(const FwdArgs &a, int64_t row, int col, float s)
{
    float4 q;
    if (PACKED) {
        unsigned v = *reinterpret_cast<const unsigned short *>(a.packed + row * (a.D >> 1) + (col >> 1));
        q.x = (float)nibble_code(v);
        q.y = (float)nibble_code(v >> 4);
        q.z = (float)nibble_code(v >> 8);
        q.w = (float)nibble_code(v >> 12);
    } else {
        float4 w = *reinterpret_cast<const float4 *>(a.master + row * a.D + col);
        q.x = int4_code(w.x, s);
        q.y = int4_code(w.y, s);
        q.z = int4_code(w.z, s);
        q.w = int4_code(w.w, s);
    }
    return q;
}

__device__ __forceinline__ void store_codes(int8_t *codes, int64_t i, int D, int col, float4 q)
{
    char4 c = make_char4((signed char)(int)q.x, (signed char)(int)q.y, (signed char)(int)q.z, (signed char)(int)q.w);
    *reinterpret_cast<char4 *>(codes + i * D + col) = c;
}

template <int G, bool PACKED>
__global__ __launch_bounds__(kFwdThreads) void embbag_fwd_kernel(FwdArgs a)
{
    __shared__ int64_t s_row[kFwdTile]; // absolute row of the bag's first lookup, -1 if none / invalid
    __shared__ int64_t s_beg[kFwdTile]; // position of the bag's first lookup
    __shared__ int s_len[kFwdTile];     // lookups in the bag
    __shared__ int s_tab[kFwdTile];
    __shared__ float s_scale[kFwdTile];

    const int tid = threadIdx.x;
    const int64_t slot0 = (int64_t)blockIdx.x * kFwdTile;

    // ---- phase A: one slot per thread ------------------------------------------
    {
        const int64_t o = slot0 + tid;
        int64_t row = -1, beg = 0;
        int len = 0, t = 0;
        float sc = 1.0f;
        if (o < a.num_bags) {
            const unsigned b = (unsigned)o / (unsigned)a.T; // num_bags < 2^31 (checked on the host)
            t = (int)((unsigned)o - b * (unsigned)a.T);
            const int64_t bag = (int64_t)t * a.B + b;
            int64_t s = a.offsets[bag], e = a.offsets[bag + 1];
            if (s < 0 || e > a.num_indices || s > e) {
                report(DQRM_ERR_BAD_OFFSETS, t, bag);
                s = e = 0;
            }
            if (e - s > 0x7fffffff) e = s + 0x7fffffff;
            beg = s;
            len = (int)(e - s);
            sc = a.w_scale[t];
            if (len > 0) {
                const int64_t idx = a.indices[s];
                const int64_t r0 = a.row_offsets[t], r1 = a.row_offsets[t + 1];
                if (idx >= 0 && idx < r1 - r0)
                    row = r0 + idx;
                else
                    report(DQRM_ERR_INDEX_OUT_OF_RANGE, t, idx);
            }
        }
        s_row[tid] = row;
        s_beg[tid] = beg;
        s_len[tid] = len;
        s_tab[tid] = t;
        s_scale[tid] = sc;
    }
    __syncthreads();

    // ---- phases B and C ------------------------------------------------------------
    constexpr int kGroups = kFwdThreads / G;   // groups per workgroup
    constexpr int kIters = kFwdTile / kGroups; // slots per group (= G)
    constexpr int kBatch = kIters < kFwdBatch ? kIters : kFwdBatch;
    const int lg = tid & (G - 1);
    const int grp = tid / G;
    const int col = lg * 4;
    const bool col_ok = col < a.D;

    for (int k0 = 0; k0 < kIters; k0 += kBatch) {
        float4 q[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) { // B: request the first rows of the whole batch
            const int i = (k0 + k) * kGroups + grp;
            const int64_t row = s_row[i];
            q[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row >= 0 && col_ok) q[k] = load_codes<PACKED>(a, row, col, s_scale[i]);
        }
#pragma unroll
        for (int k = 0; k < kBatch; ++k) { // C: pool and store
            const int i = (k0 + k) * kGroups + grp;
            const int64_t o = slot0 + i;
            if (o >= a.num_bags) continue;
            const float s = s_scale[i];
            const int len = s_len[i];
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            if (s_row[i] >= 0) {
                acc.x = acc.x + s * q[k].x;
                acc.y = acc.y + s * q[k].y;
                acc.z = acc.z + s * q[k].z;
                acc.w = acc.w + s * q[k].w;
                if (a.codes && col_ok) store_codes(a.codes, s_beg[i], a.D, col, q[k]);
            }
            if (len > 1) {
                const int t = s_tab[i];
                const int64_t r0 = a.row_offsets[t], r1 = a.row_offsets[t + 1];
                const int64_t beg = s_beg[i];
                for (int64_t p = beg + 1; p < beg + len; ++p) {
                    const int64_t idx = a.indices[p];
                    if (idx < 0 || idx >= r1 - r0) {
                        if (lg == 0) report(DQRM_ERR_INDEX_OUT_OF_RANGE, t, idx);
                        continue;
                    }
                    if (col_ok) {
                        const float4 qq = load_codes<PACKED>(a, r0 + idx, col, s);
                        acc.x = acc.x + s * qq.x;
                        acc.y = acc.y + s * qq.y;
                        acc.z = acc.z + s * qq.z;
                        acc.w = acc.w + s * qq.w;
                        if (a.codes) store_codes(a.codes, p, a.D, col, qq);
                    }
                }
            }
            if (col_ok) {
                // `out` is written once and not read again by this library: stream it past the caches
                f32x4 v = {acc.x, acc.y, acc.z, acc.w};
                __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(a.out + o * a.D + col));
            }
        }
    }
}

} // namespace dqrm
