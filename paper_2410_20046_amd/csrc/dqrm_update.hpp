// INT8 quantisation of the sparse gradient's values and the sparse SGD row
// update (gradient-quantisation appendix of the paper), plus the whole-table
// passes: find-scale (Sec. 3.2) and INT4 packing.
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

constexpr int kEwThreads = 256;

// Per-table constants of the element-wise kernels, in dynamic LDS:
// [T+1] int tuo | [T] Scale gradient | [T] Scale weight | [T+1] int64 row offsets
struct TableLds {
    int *tuo;
    Scale *gs, *ws;
    int64_t *r0;
    __device__ __forceinline__ explicit TableLds(unsigned char *base, int T)
    {
        r0 = reinterpret_cast<int64_t *>(base);
        gs = reinterpret_cast<Scale *>(r0 + (T + 1));
        ws = gs + T;
        tuo = reinterpret_cast<int *>(ws + T);
    }
    __host__ __device__ static size_t bytes(int T) { return (size_t)(T + 1) * 8 + (size_t)T * 16 + (size_t)(T + 1) * 4; }
};

// One float4 of one unique row: which row, which table, which quarter-row.
struct RowElem {
    unsigned e;  // float4 index into values / char4 index into gq
    int u, t, c4;
};

// the element's position; e < total <= capacity * D / 4 < 2^31
__device__ __forceinline__ RowElem row_elem(unsigned e, FastDiv by_q4, const TableLds &L, int T)
{
    RowElem r;
    r.e = e;
    r.u = (int)by_q4.div(e);
    r.c4 = (int)(e - (unsigned)r.u * by_q4.d);
    r.t = table_of(L.tuo, T, r.u);
    return r;
}

__device__ __forceinline__ unsigned clamp_u(const int *tuo, int T, int64_t capacity)
{
    int64_t U = tuo[T];
    return (unsigned)(U < 0 ? 0 : (U > capacity ? capacity : U));
}

// ---- B4: values -> INT8 codes, one scale per table ---------------------------
struct QuantArgs {
    const float *values;
    const int32_t *tuo;
    const float *g_absmax;
    int8_t *gq;
    float *g_scale;
    int64_t capacity;
    FastDiv by_q4;
    int T, D;
};

__device__ __forceinline__ void grad_quant_body(const QuantArgs &a)
{
    extern __shared__ __align__(16) unsigned char s_dyn[];
    const TableLds L(s_dyn, a.T);
    const int T = a.T;
    for (int k = threadIdx.x; k <= T; k += kEwThreads) {
        L.tuo[k] = a.tuo[k];
        if (k < T) {
            const float gs = scale_from_absmax(a.g_absmax[k], 127.0f);
            L.gs[k] = Scale(gs);
            if (blockIdx.x == 0) a.g_scale[k] = gs;
        }
    }
    __syncthreads();
    const unsigned total = clamp_u(L.tuo, T, a.capacity) * a.by_q4.d;
    for (unsigned e = blockIdx.x * kEwThreads + threadIdx.x; e < total; e += gridDim.x * kEwThreads) {
        const RowElem r = row_elem(e, a.by_q4, L, T);
        const Scale gs = L.gs[r.t];
        const float4 v = reinterpret_cast<const float4 *>(a.values)[e];
        // the caller's g_absmax may be smaller than the values' (then codes clamp): guarded quotient
        reinterpret_cast<unsigned *>(a.gq)[e] =
            pack_bytes(int8_code(v.x, gs), int8_code(v.y, gs), int8_code(v.z, gs), int8_code(v.w, gs));
    }
}

__global__ __launch_bounds__(kEwThreads) void grad_quant_kernel(QuantArgs a)
{
    grad_quant_body(a);
}

// several blocks of values in one launch (blockIdx.y picks the block), for the same reason as the segment sums
struct QuantMulti {
    QuantArgs b[DQRM_MAX_DEDUPE_BATCHES];
};

__global__ __launch_bounds__(kEwThreads) void grad_quant_multi_kernel(QuantMulti m)
{
    grad_quant_body(m.b[blockIdx.y]);
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
    const int32_t *sums; // instead of gq: 32-bit sums of the codes of several blocks (merged sparse gradients)
    const float *g_scale;
    int64_t capacity;
    FastDiv by_q4;
    float lr;
    int T, D;
};

// w <- w - lr * (gs * code), each operation rounded on its own; returns the new weights
__device__ __forceinline__ float4 sgd_step(float4 w, int c0, int c1, int c2, int c3, float gs, float lr)
{
    w.x = w.x - lr * (gs * (float)c0);
    w.y = w.y - lr * (gs * (float)c1);
    w.z = w.z - lr * (gs * (float)c2);
    w.w = w.w - lr * (gs * (float)c3);
    return w;
}

__device__ __forceinline__ unsigned short encode4(float4 w, Scale ws)
{
    return (unsigned short)pack4(int4_code(w.x, ws), int4_code(w.y, ws), int4_code(w.z, ws), int4_code(w.w, ws));
}

__global__ __launch_bounds__(kEwThreads) void sparse_update_kernel(UpdateArgs a)
{
    extern __shared__ __align__(16) unsigned char s_dyn[];
    const TableLds L(s_dyn, a.T);
    const int T = a.T;
    for (int k = threadIdx.x; k <= T; k += kEwThreads) {
        L.tuo[k] = a.tuo[k];
        L.r0[k] = a.row_offsets[k];
        if (k < T) {
            L.gs[k].s = a.g_scale[k];
            if (a.packed) L.ws[k] = Scale(a.w_scale[k]);
        }
    }
    __syncthreads();
    const unsigned total = clamp_u(L.tuo, T, a.capacity) * a.by_q4.d;
    const int q4 = (int)a.by_q4.d;
    for (unsigned e = blockIdx.x * kEwThreads + threadIdx.x; e < total; e += gridDim.x * kEwThreads) {
        const RowElem r = row_elem(e, a.by_q4, L, T);
        const int64_t r0 = L.r0[r.t], r1 = L.r0[r.t + 1];
        const int64_t lr_row = a.uniq_rows[r.u];
        if (lr_row < 0 || lr_row >= r1 - r0) {
            if (r.c4 == 0) report(DQRM_ERR_INDEX_OUT_OF_RANGE, r.t, lr_row);
            continue;
        }
        const int64_t row = r0 + lr_row;
        int4 c;
        if (a.sums) {
            c = reinterpret_cast<const int4 *>(a.sums)[e];
        } else {
            const char4 c8 = reinterpret_cast<const char4 *>(a.gq)[e];
            c = make_int4(c8.x, c8.y, c8.z, c8.w);
        }
        float4 *wp = reinterpret_cast<float4 *>(a.master) + row * q4 + r.c4;
        const float4 w = sgd_step(*wp, c.x, c.y, c.z, c.w, L.gs[r.t].s, a.lr);
        *wp = w;
        if (a.packed)
            reinterpret_cast<unsigned short *>(a.packed)[row * q4 + r.c4] = encode4(w, L.ws[r.t]);
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

constexpr int kQuPerThread = 2; // float4 elements a thread has in flight

__global__ __launch_bounds__(kEwThreads) void quant_update_kernel(QuantUpdateArgs a)
{
    extern __shared__ __align__(16) unsigned char s_dyn[];
    const int T = a.u.T;
    const TableLds L(s_dyn, T);
    for (int k = threadIdx.x; k <= T; k += kEwThreads) {
        L.tuo[k] = a.u.tuo[k];
        L.r0[k] = a.u.row_offsets[k];
        if (k < T) {
            float v[kAbsmaxSlots];
#pragma unroll
            for (int q = 0; q < kAbsmaxSlots; ++q) v[q] = *absmax_slot(a.absmax_slots, k, q);
            float m = 0.0f;
#pragma unroll
            for (int q = 0; q < kAbsmaxSlots; ++q) m = fmaxf(m, v[q]);
            const float gs = scale_from_absmax(m, 127.0f);
            L.gs[k] = Scale(gs);
            if (a.u.packed) L.ws[k] = Scale(a.u.w_scale[k]);
            if (blockIdx.x == 0) {
                a.g_absmax[k] = m;
                a.g_scale_out[k] = gs;
            }
        }
    }
    __syncthreads();
    const unsigned total = clamp_u(L.tuo, T, a.u.capacity) * a.u.by_q4.d;
    const int q4 = (int)a.u.by_q4.d;
    const unsigned nthreads = gridDim.x * kEwThreads;
    // e0 + 3 * nthreads < 2^32: total < 2^31 and nthreads <= 2^19 (host)
    for (unsigned e0 = blockIdx.x * kEwThreads + threadIdx.x; e0 < total; e0 += nthreads * kQuPerThread) {
        // 1. gradient values and row ids of all elements of the batch
        RowElem r[kQuPerThread];
        float4 v[kQuPerThread];
        int64_t row[kQuPerThread];
#pragma unroll
        for (int k = 0; k < kQuPerThread; ++k) {
            const unsigned e = e0 + k * nthreads;
            row[k] = -1;
            v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            r[k] = row_elem(e < total ? e : 0u, a.u.by_q4, L, T);
            if (e < total) {
                v[k] = reinterpret_cast<const float4 *>(a.values)[e];
                row[k] = a.u.uniq_rows[r[k].u];
            }
        }
        // 2. their master weights
        float4 w[kQuPerThread];
#pragma unroll
        for (int k = 0; k < kQuPerThread; ++k) {
            const unsigned e = e0 + k * nthreads;
            w[k] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (e < total) {
                const int64_t r0 = L.r0[r[k].t], r1 = L.r0[r[k].t + 1];
                if (row[k] < 0 || row[k] >= r1 - r0) {
                    if (r[k].c4 == 0) report(DQRM_ERR_INDEX_OUT_OF_RANGE, r[k].t, row[k]);
                    row[k] = -1;
                } else {
                    row[k] = (r0 + row[k]) * q4 + r[k].c4; // float4 index into the master table
                    w[k] = reinterpret_cast<const float4 *>(a.u.master)[row[k]];
                }
            }
        }
        // 3. quantise, store the codes, step, re-encode
#pragma unroll
        for (int k = 0; k < kQuPerThread; ++k) {
            const unsigned e = e0 + k * nthreads;
            if (e >= total) continue;
            const Scale gs = L.gs[r[k].t];
            // the scale comes from the maximum of these very values: no quotient beyond 127 (1 + 2^-23)
            const int c0 = int8_code_fresh(v[k].x, gs), c1 = int8_code_fresh(v[k].y, gs);
            const int c2 = int8_code_fresh(v[k].z, gs), c3 = int8_code_fresh(v[k].w, gs);
            reinterpret_cast<unsigned *>(a.gq_out)[e] = pack_bytes(c0, c1, c2, c3);
            if (row[k] < 0) continue;
            const float4 x = sgd_step(w[k], c0, c1, c2, c3, gs.s, a.u.lr);
            reinterpret_cast<float4 *>(a.u.master)[row[k]] = x;
            if (a.u.packed) reinterpret_cast<unsigned short *>(a.u.packed)[row[k]] = encode4(x, L.ws[r[k].t]);
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
// A thread takes kPackPerThread groups of 8 elements (32 bytes in, 4 bytes out each) per round, all requested
// before the first is encoded; consecutive threads take consecutive groups.
constexpr int kPackPerThread = 4;

__global__ __launch_bounds__(kEwThreads) void pack_int4_kernel(const float *__restrict__ master,
                                                               const int64_t *__restrict__ row_offsets,
                                                               const float *__restrict__ w_scale, int T, int D,
                                                               uint8_t *__restrict__ packed)
{
    __shared__ int64_t s_ro[DQRM_MAX_TABLES + 1];
    __shared__ Scale s_ws[DQRM_MAX_TABLES];
    for (int k = threadIdx.x; k <= T; k += kEwThreads) {
        s_ro[k] = row_offsets[k];
        if (k < T) s_ws[k] = Scale(w_scale[k]);
    }
    __syncthreads();
    const int q8 = D >> 3; // groups of 8 elements per row -> 4 packed bytes each
    const int64_t total = s_ro[T] * q8;
    int cur_t = -1;
    int64_t cur_end = -1;
    Scale ws(1.0f);
    const int64_t stride = (int64_t)gridDim.x * kEwThreads;
    for (int64_t e0 = (int64_t)blockIdx.x * kEwThreads + threadIdx.x; e0 < total; e0 += stride * kPackPerThread) {
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        f32x4 lo4[kPackPerThread], hi4[kPackPerThread];
#pragma unroll
        for (int k = 0; k < kPackPerThread; ++k) {
            const int64_t e = e0 + k * stride;
            if (e < total) {
                lo4[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(master) + 2 * e);
                hi4[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(master) + 2 * e + 1);
            }
        }
#pragma unroll
        for (int k = 0; k < kPackPerThread; ++k) {
            const int64_t e = e0 + k * stride;
            if (e >= total) break;
            if (e >= cur_end) {
                cur_t = table_of(s_ro, T, e / q8);
                cur_end = s_ro[cur_t + 1] * q8;
                ws = s_ws[cur_t];
            }
            const f32x4 a = lo4[k], b = hi4[k];
            const unsigned lo = pack4(int4_code(a[0], ws), int4_code(a[1], ws), int4_code(a[2], ws), int4_code(a[3], ws));
            const unsigned hi = pack4(int4_code(b[0], ws), int4_code(b[1], ws), int4_code(b[2], ws), int4_code(b[3], ws));
            __builtin_nontemporal_store(lo | (hi << 16), reinterpret_cast<unsigned *>(packed) + e);
        }
    }
}

} // namespace dqrm
