// Device-side helpers shared by the DQRM kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dqrm.h"

// one rounding per operation everywhere: results are compared bit for bit
#pragma clang fp contract(off)

namespace dqrm {

constexpr int kWave = 64;

// ---- per-device status word ------------------------------------------------
// Kernels record the first data-dependent problem here (they never act on the
// offending data); dqrm_check_status() copies it out and clears it.
struct DeviceStatus {
    int code;
    int table;
    long long value;
};
__device__ DeviceStatus g_status;

__device__ __forceinline__ void report(int code, int table, long long value)
{
    if (atomicCAS(&g_status.code, 0, code) == 0) {
        g_status.table = table;
        g_status.value = value;
    }
}

// ---- the quantiser -----------------------------------------------------------
// scale = max(absmax / qmax, 1e-8); code = clamp(rint(x / scale), lo, hi).
// IEEE division (hipcc rounds fp32 division correctly unless told otherwise),
// round-half-even (v_rndne_f32), one rounding per operation.
__device__ __forceinline__ float scale_from_absmax(float absmax, float qmax)
{
    return fmaxf(absmax / qmax, 1e-8f);
}

__device__ __forceinline__ float code_f(float x, float scale, float lo, float hi)
{
    return fminf(fmaxf(rintf(x / scale), lo), hi);
}

__device__ __forceinline__ float int4_code(float w, float s) { return code_f(w, s, -8.0f, 7.0f); }
__device__ __forceinline__ float int8_code(float g, float s) { return code_f(g, s, -128.0f, 127.0f); }

// sign-extend the low 4 bits of v
__device__ __forceinline__ int nibble_code(unsigned v) { return (int)((v & 0xFu) ^ 8u) - 8; }

// four codes -> two bytes, element 0 in the low nibble of byte 0
__device__ __forceinline__ unsigned pack4(float q0, float q1, float q2, float q3)
{
    return ((unsigned)(int)q0 & 0xFu) | (((unsigned)(int)q1 & 0xFu) << 4) | (((unsigned)(int)q2 & 0xFu) << 8) |
           (((unsigned)(int)q3 & 0xFu) << 12);
}

// ---- wave / block primitives ---------------------------------------------------
__device__ __forceinline__ int lane_id() { return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)); }

// DPP moves: lanes whose source lies outside the row (or whose row is masked
// off) receive `identity`.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int dpp_or(int identity, int v)
{
    return __builtin_amdgcn_update_dpp(identity, v, kCtrl, kRowMask, 0xF, false);
}

constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;

// inclusive scans over the 64 lanes of a wave: four shifts inside each row of
// 16 lanes, then the row totals are passed on to the following rows
__device__ __forceinline__ int wave_incl_scan_add(int v, int /*lane*/)
{
    v += dpp_or<kDppRowShr1, 0xF>(0, v);
    v += dpp_or<kDppRowShr2, 0xF>(0, v);
    v += dpp_or<kDppRowShr4, 0xF>(0, v);
    v += dpp_or<kDppRowShr8, 0xF>(0, v);
    v += dpp_or<kDppRowBcast15, 0xA>(0, v);
    v += dpp_or<kDppRowBcast31, 0xC>(0, v);
    return v;
}

// values must be >= -1 (the identity used for lanes without a source)
__device__ __forceinline__ int wave_incl_scan_max(int v, int /*lane*/)
{
    v = max(v, dpp_or<kDppRowShr1, 0xF>(-1, v));
    v = max(v, dpp_or<kDppRowShr2, 0xF>(-1, v));
    v = max(v, dpp_or<kDppRowShr4, 0xF>(-1, v));
    v = max(v, dpp_or<kDppRowShr8, 0xF>(-1, v));
    v = max(v, dpp_or<kDppRowBcast15, 0xA>(-1, v));
    v = max(v, dpp_or<kDppRowBcast31, 0xC>(-1, v));
    return v;
}

__device__ __forceinline__ int wave_last(int v) { return __builtin_amdgcn_readlane(v, kWave - 1); }

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, kWave));
    return v;
}

__device__ __forceinline__ int wave_max_int(int v)
{
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) v = max(v, __shfl_xor(v, d, kWave));
    return v;
}

// lanes of the wave whose 8-bit digit equals mine (all 64 lanes must be active)
__device__ __forceinline__ unsigned long long match_any8(unsigned d)
{
    unsigned long long m = ~0ull;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        bool bit = (d >> b) & 1u;
        unsigned long long bal = __ballot(bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}

// largest t in [0, T) with offs[t] <= x, for a non-decreasing offs[0..T] with
// offs[0] <= x; tables with no entries (offs[t] == offs[t+1]) are skipped
// because the search is an upper bound.
template <typename OffT, typename X>
__device__ __forceinline__ int table_of(const OffT *offs, int T, X x)
{
    int lo = 0, hi = T; // invariant: offs[lo] <= x, answer in [lo, hi)
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if ((X)offs[mid] <= x)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

// non-negative floats order like their bit patterns
__device__ __forceinline__ void atomic_max_nonneg(float *addr, float v)
{
    atomicMax(reinterpret_cast<unsigned *>(addr), __float_as_uint(v));
}

// Per-table maxima are first gathered in kAbsmaxSlots separate cache lines per
// table (workgroups pick a slot by their index), so that atomics from thousands
// of workgroups do not all queue on one line; a last small kernel folds them.
constexpr int kAbsmaxSlots = 16;
constexpr int kAbsmaxStride = 32; // floats between slots = 128 bytes

__device__ __forceinline__ float *absmax_slot(float *slots, int t, int k)
{
    return slots + ((int64_t)t * kAbsmaxSlots + k) * kAbsmaxStride;
}

} // namespace dqrm
