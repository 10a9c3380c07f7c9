// INT8 quantisation of the sparse gradient's values and the sparse SGD row
// update (gradient-quantisation appendix of the paper), plus the whole-table
// passes: find-scale (Sec. 3.2) and INT4 packing.
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

constexpr int kEwThreads = 256;

// ---- B4: values -> INT8 codes, one scale per table ---------------------------
struct QuantArgs {
    const float *values;
    const int32_t *tuo;
    const float *g_absmax;
    int8_t *gq;
    float *g_scale;
    int64_t capacity;
    int T, D;
};

__global__ __launch_bounds__(kEwThreads) void grad_quant_kernel(QuantArgs a)
{
    __shared__ int s_tuo[DQRM_MAX_TABLES + 1];
    __shared__ float s_gs[DQRM_MAX_TABLES];
    const int T = a.T;
    for (int k = threadIdx.x; k <= T; k += kEwThreads) {
        s_tuo[k] = a.tuo[k];
        if (k < T) {
            const float gs = scale_from_absmax(a.g_absmax[k], 127.0f);
            s_gs[k] = gs;
            if (blockIdx.x == 0) a.g_scale[k] = gs;
        }
    }
    __syncthreads();
    int64_t U = s_tuo[T];
    U = U < 0 ? 0 : (U > a.capacity ? a.capacity : U);
    const int q4 = a.D >> 2; // float4 per row
    const int64_t total = U * q4;
    for (int64_t e = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kEwThreads) {
        const int64_t u = e / q4;
        const int t = table_of(s_tuo, T, (int)u);
        const float gs = s_gs[t];
        const float4 v = reinterpret_cast<const float4 *>(a.values)[e];
        char4 c = make_char4((signed char)(int)int8_code(v.x, gs), (signed char)(int)int8_code(v.y, gs),
                             (signed char)(int)int8_code(v.z, gs), (signed char)(int)int8_code(v.w, gs));
        reinterpret_cast<char4 *>(a.gq)[e] = c;
    }
}

// ---- B5: dequantise, SGD on the master rows, re-encode the packed mirror -------
struct UpdateArgs {
    float *master;
    uint8_t *packed;
    const float *w_scale;
    const int64_t *row_offsets;
    const int64_t *uniq_rows;
    const int32_t *tuo;
    const int8_t *gq;
    const float *g_scale;
    int64_t capacity;
    float lr;
    int T, D;
};

__global__ __launch_bounds__(kEwThreads) void sparse_update_kernel(UpdateArgs a)
{
    __shared__ int s_tuo[DQRM_MAX_TABLES + 1];
    const int T = a.T;
    for (int k = threadIdx.x; k <= T; k += kEwThreads) s_tuo[k] = a.tuo[k];
    __syncthreads();
    int64_t U = s_tuo[T];
    U = U < 0 ? 0 : (U > a.capacity ? a.capacity : U);
    const int q4 = a.D >> 2;
    const int64_t total = U * q4;
    for (int64_t e = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kEwThreads) {
        const int64_t u = e / q4;
        const int c4 = (int)(e - u * q4);
        const int t = table_of(s_tuo, T, (int)u);
        const int64_t r0 = a.row_offsets[t], r1 = a.row_offsets[t + 1];
        const int64_t lr_row = a.uniq_rows[u];
        if (lr_row < 0 || lr_row >= r1 - r0) {
            if (c4 == 0) report(DQRM_ERR_INDEX_OUT_OF_RANGE, t, lr_row);
            continue;
        }
        const int64_t row = r0 + lr_row;
        const float gs = a.g_scale[t];
        const char4 c = reinterpret_cast<const char4 *>(a.gq)[e];
        float4 *wp = reinterpret_cast<float4 *>(a.master + row * a.D) + c4;
        float4 w = *wp;
        // g = g_scale * code; w <- w - lr * g, each operation rounded on its own
        w.x = w.x - a.lr * (gs * (float)c.x);
        w.y = w.y - a.lr * (gs * (float)c.y);
        w.z = w.z - a.lr * (gs * (float)c.z);
        w.w = w.w - a.lr * (gs * (float)c.w);
        *wp = w;
        if (a.packed) {
            const float ws = a.w_scale[t];
            const unsigned p = pack4(int4_code(w.x, ws), int4_code(w.y, ws), int4_code(w.z, ws), int4_code(w.w, ws));
            *reinterpret_cast<unsigned short *>(a.packed + row * (a.D >> 1) + c4 * 2) = (unsigned short)p;
        }
    }
}

// ---- B4 + B5 in one pass ---------------------------------------------------------
// Same results as grad_quant_kernel followed by sparse_update_kernel (and as the
// fold of the per-table maxima that ends the segment sums): every block folds
// the maxima itself, then each thread quantises four gradient values, stores
// their INT8 codes, and applies the dequantised step to its four master weights.
struct QuantUpdateArgs {
    UpdateArgs u;             // u.gq / u.g_scale are written here, not read
    const float *values;
    float *absmax_slots;       // [T][kAbsmaxSlots], see absmax_slot()
    float *g_absmax;           // [T] out
    int8_t *gq_out;
    float *g_scale_out;
};

constexpr int kQuPerThread = 4; // float4 elements a thread has in flight

__global__ __launch_bounds__(kEwThreads) void quant_update_kernel(QuantUpdateArgs a)
{
    __shared__ int s_tuo[DQRM_MAX_TABLES + 1];
    __shared__ float s_gs[DQRM_MAX_TABLES];
    const int T = a.u.T;
    for (int k = threadIdx.x; k <= T; k += kEwThreads) {
        s_tuo[k] = a.u.tuo[k];
        if (k < T) {
            float v[kAbsmaxSlots];
#pragma unroll
            for (int q = 0; q < kAbsmaxSlots; ++q) v[q] = *absmax_slot(a.absmax_slots, k, q);
            float m = 0.0f;
#pragma unroll
            for (int q = 0; q < kAbsmaxSlots; ++q) m = fmaxf(m, v[q]);
            const float gs = scale_from_absmax(m, 127.0f);
            s_gs[k] = gs;
            if (blockIdx.x == 0) {
                a.g_absmax[k] = m;
                a.g_scale_out[k] = gs;
            }
        }
    }
    __syncthreads();
    int64_t U = s_tuo[T];
    U = U < 0 ? 0 : (U > a.u.capacity ? a.u.capacity : U);
    const int D = a.u.D, q4 = D >> 2;
    const int64_t total = U * q4;
    const int64_t nthreads = (int64_t)gridDim.x * kEwThreads;
    for (int64_t e0 = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; e0 < total; e0 += nthreads * kQuPerThread) {
        // 1. gradient values and row ids of all elements of the batch
        float4 v[kQuPerThread];
        int64_t row[kQuPerThread];
        int tab[kQuPerThread], c4[kQuPerThread];
#pragma unroll
        for (int k = 0; k < kQuPerThread; ++k) {
            const int64_t e = e0 + k * nthreads;
            row[k] = -1;
            tab[k] = 0;
            c4[k] = 0;
            v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (e < total) {
                const int64_t u = e / q4;
                c4[k] = (int)(e - u * q4);
                tab[k] = table_of(s_tuo, T, (int)u);
                v[k] = reinterpret_cast<const float4 *>(a.values)[e];
                row[k] = a.u.uniq_rows[u];
            }
        }
        // 2. their master weights
        float4 w[kQuPerThread];
#pragma unroll
        for (int k = 0; k < kQuPerThread; ++k) {
            const int64_t e = e0 + k * nthreads;
            w[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (e < total) {
                const int64_t r0 = a.u.row_offsets[tab[k]], r1 = a.u.row_offsets[tab[k] + 1];
                if (row[k] < 0 || row[k] >= r1 - r0) {
                    if (c4[k] == 0) report(DQRM_ERR_INDEX_OUT_OF_RANGE, tab[k], row[k]);
                    row[k] = -1;
                } else {
                    row[k] += r0;
                    w[k] = reinterpret_cast<const float4 *>(a.u.master + row[k] * D)[c4[k]];
                }
            }
        }
        // 3. quantise, store the codes, step, re-encode
#pragma unroll
        for (int k = 0; k < kQuPerThread; ++k) {
            const int64_t e = e0 + k * nthreads;
            if (e >= total) continue;
            const float gs = s_gs[tab[k]];
            const char4 c = make_char4((signed char)(int)int8_code(v[k].x, gs), (signed char)(int)int8_code(v[k].y, gs),
                                       (signed char)(int)int8_code(v[k].z, gs), (signed char)(int)int8_code(v[k].w, gs));
            reinterpret_cast<char4 *>(a.gq_out)[e] = c;
            if (row[k] < 0) continue;
            // g = g_scale * code; w <- w - lr * g, each operation rounded on its own
            float4 x = w[k];
            x.x = x.x - a.u.lr * (gs * (float)c.x);
            x.y = x.y - a.u.lr * (gs * (float)c.y);
            x.z = x.z - a.u.lr * (gs * (float)c.z);
            x.w = x.w - a.u.lr * (gs * (float)c.w);
            reinterpret_cast<float4 *>(a.u.master + row[k] * D)[c4[k]] = x;
            if (a.u.packed) {
                const float ws = a.u.w_scale[tab[k]];
                const unsigned p = pack4(int4_code(x.x, ws), int4_code(x.y, ws), int4_code(x.z, ws), int4_code(x.w, ws));
                *reinterpret_cast<unsigned short *>(a.u.packed + row[k] * (D >> 1) + c4[k] * 2) = (unsigned short)p;
            }
        }
    }
}

// ---- S0: per-table absmax of the master table ----------------------------------
__global__ void fill_u32_kernel(unsigned *p, unsigned v, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// absmax_bits[t] (zeroed before) <- max |master_t|, as the bit pattern of a non-negative float
__global__ __launch_bounds__(kEwThreads) void table_absmax_kernel(const float *__restrict__ master,
                                                                  const int64_t *__restrict__ row_offsets, int T, int D,
                                                                  float *absmax)
{
    __shared__ int64_t s_ro[DQRM_MAX_TABLES + 1];
    for (int k = threadIdx.x; k <= T; k += kEwThreads) s_ro[k] = row_offsets[k];
    __syncthreads();
    const int q4 = D >> 2;
    const int64_t total = s_ro[T] * q4;
    const int64_t per_block = (total + gridDim.x - 1) / gridDim.x;
    const int64_t beg = (int64_t)blockIdx.x * per_block;
    const int64_t end = beg + per_block < total ? beg + per_block : total;
    int cur_t = -1;
    int64_t cur_end = -1; // first float4 past the current table
    float cur_max = 0.0f;
    for (int64_t e = beg + threadIdx.x; e < end; e += kEwThreads) {
        if (e >= cur_end) {
            if (cur_t >= 0 && cur_max > 0.0f) atomic_max_nonneg(absmax + cur_t, cur_max);
            cur_t = table_of(s_ro, T, e / q4);
            cur_end = s_ro[cur_t + 1] * q4;
            cur_max = 0.0f;
        }
        const float4 w = reinterpret_cast<const float4 *>(master)[e];
        cur_max = fmaxf(cur_max, fmaxf(fmaxf(fabsf(w.x), fabsf(w.y)), fmaxf(fabsf(w.z), fabsf(w.w))));
    }
    const int tt = wave_max_int(cur_t);
    if (__all(cur_t < 0 || cur_t == tt)) {
        const float m = wave_max(cur_max);
        if ((threadIdx.x & (kWave - 1)) == 0 && tt >= 0 && m > 0.0f) atomic_max_nonneg(absmax + tt, m);
    } else if (cur_t >= 0 && cur_max > 0.0f) {
        atomic_max_nonneg(absmax + cur_t, cur_max);
    }
}

__global__ void finalize_scale_kernel(float *w_scale, int T)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) w_scale[t] = scale_from_absmax(w_scale[t], 7.0f);
}

// ---- S1: encode every row of the master table into the packed mirror ------------
__global__ __launch_bounds__(kEwThreads) void pack_int4_kernel(const float *__restrict__ master,
                                                               const int64_t *__restrict__ row_offsets,
                                                               const float *__restrict__ w_scale, int T, int D,
                                                               uint8_t *__restrict__ packed)
{
    __shared__ int64_t s_ro[DQRM_MAX_TABLES + 1];
    __shared__ float s_ws[DQRM_MAX_TABLES];
    for (int k = threadIdx.x; k <= T; k += kEwThreads) {
        s_ro[k] = row_offsets[k];
        if (k < T) s_ws[k] = w_scale[k];
    }
    __syncthreads();
    const int q8 = D >> 3; // groups of 8 elements per row -> 4 packed bytes each
    const int64_t total = s_ro[T] * q8;
    int cur_t = -1;
    int64_t cur_end = -1;
    float ws = 1.0f;
    for (int64_t e = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kEwThreads) {
        if (e >= cur_end) {
            cur_t = table_of(s_ro, T, e / q8);
            cur_end = s_ro[cur_t + 1] * q8;
            ws = s_ws[cur_t];
        }
        const float4 a = reinterpret_cast<const float4 *>(master)[2 * e];
        const float4 b = reinterpret_cast<const float4 *>(master)[2 * e + 1];
        const unsigned lo = pack4(int4_code(a.x, ws), int4_code(a.y, ws), int4_code(a.z, ws), int4_code(a.w, ws));
        const unsigned hi = pack4(int4_code(b.x, ws), int4_code(b.y, ws), int4_code(b.z, ws), int4_code(b.w, ws));
        reinterpret_cast<unsigned *>(packed)[e] = lo | (hi << 16);
    }
}

} // namespace dqrm
