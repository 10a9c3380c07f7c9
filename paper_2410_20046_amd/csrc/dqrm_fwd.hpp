// Forward: gather -> INT4 fake-quant -> sum-pool (Sec. 3.1 and Sec. 4.1 of the paper).
//
// A group of G = pow2ceil(D/4) lanes owns one bag; lane l of the group owns the
// four columns 4l..4l+3 (one 16-byte access per row).  The bag's lookups are
// walked in order, so the per-column sum is the plain left-to-right sum and no
// cross-lane reduction is needed.  Each group handles kBagsPerGroup bags whose
// first rows are all requested before any is used, to keep enough bytes in
// flight per CU to cover HBM latency with one-lookup bags.
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

constexpr int kFwdThreads = 256;
constexpr int kBagsPerGroup = 4;

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

// dequantised value of 4 consecutive elements of one row
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
    const int lg = threadIdx.x & (G - 1);
    const int col = lg * 4;
    const bool col_ok = col < a.D;
    const int64_t group = ((int64_t)blockIdx.x * kFwdThreads + threadIdx.x) / G;
    const int64_t bag0 = group * kBagsPerGroup;
    if (bag0 >= a.num_bags) return;

    int64_t beg[kBagsPerGroup], end[kBagsPerGroup], row[kBagsPerGroup];
    int tab[kBagsPerGroup];
    float sc[kBagsPerGroup];

    // 1. bag extents (clamped so that every later access is in range)
#pragma unroll
    for (int k = 0; k < kBagsPerGroup; ++k) {
        int64_t bag = bag0 + k;
        beg[k] = end[k] = 0;
        tab[k] = 0;
        if (bag < a.num_bags) {
            int64_t s = a.offsets[bag], e = a.offsets[bag + 1];
            tab[k] = (int)(bag / a.B);
            if (s < 0 || e > a.num_indices || s > e) {
                if (lg == 0) report(DQRM_ERR_BAD_OFFSETS, tab[k], bag);
                s = e = 0;
            }
            beg[k] = s;
            end[k] = e;
        }
    }
    // 2. first index of every bag, its table's row base and scale
#pragma unroll
    for (int k = 0; k < kBagsPerGroup; ++k) {
        row[k] = -1;
        sc[k] = 1.0f;
        if (beg[k] < end[k]) {
            int64_t idx = a.indices[beg[k]];
            int64_t r0 = a.row_offsets[tab[k]], r1 = a.row_offsets[tab[k] + 1];
            sc[k] = a.w_scale[tab[k]];
            if (idx >= 0 && idx < r1 - r0)
                row[k] = r0 + idx;
            else if (lg == 0)
                report(DQRM_ERR_INDEX_OUT_OF_RANGE, tab[k], idx);
        }
    }
    // 3. first rows, all requested before any is consumed
    float4 q[kBagsPerGroup];
#pragma unroll
    for (int k = 0; k < kBagsPerGroup; ++k) {
        q[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row[k] >= 0 && col_ok) q[k] = load_codes<PACKED>(a, row[k], col, sc[k]);
    }
    // 4. pool, then the bag's remaining lookups (none when every bag has one index)
#pragma unroll
    for (int k = 0; k < kBagsPerGroup; ++k) {
        int64_t bag = bag0 + k;
        if (bag >= a.num_bags) break;
        const float s = sc[k];
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row[k] >= 0) {
            acc.x = acc.x + s * q[k].x;
            acc.y = acc.y + s * q[k].y;
            acc.z = acc.z + s * q[k].z;
            acc.w = acc.w + s * q[k].w;
            if (a.codes && col_ok) store_codes(a.codes, beg[k], a.D, col, q[k]);
        }
        if (end[k] - beg[k] > 1) {
            const int64_t r0 = a.row_offsets[tab[k]], r1 = a.row_offsets[tab[k] + 1];
            for (int64_t i = beg[k] + 1; i < end[k]; ++i) {
                int64_t idx = a.indices[i];
                if (idx < 0 || idx >= r1 - r0) {
                    if (lg == 0) report(DQRM_ERR_INDEX_OUT_OF_RANGE, tab[k], idx);
                    continue;
                }
                if (col_ok) {
                    float4 qq = load_codes<PACKED>(a, r0 + idx, col, s);
                    acc.x = acc.x + s * qq.x;
                    acc.y = acc.y + s * qq.y;
                    acc.z = acc.z + s * qq.z;
                    acc.w = acc.w + s * qq.w;
                    if (a.codes) store_codes(a.codes, i, a.D, col, qq);
                }
            }
        }
        if (col_ok) {
            const int t = tab[k];
            const int64_t b = bag - (int64_t)t * a.B;
            *reinterpret_cast<float4 *>(a.out + (b * a.T + t) * a.D + col) = acc;
        }
    }
}

} // namespace dqrm
