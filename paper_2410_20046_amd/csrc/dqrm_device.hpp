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
// scale = max(absmax / qmax, 1e-8); code = clamp(rint(x / scale), lo, hi) with
// the IEEE quotient, round-half-even (v_rndne_f32), one rounding per operation.
__device__ __forceinline__ float scale_from_absmax(float absmax, float qmax)
{
    return fmaxf(absmax / qmax, 1e-8f);
}

// One scale and its correctly rounded reciprocal (one IEEE division per table,
// not one per element).
struct Scale {
    float s, y;
    Scale() = default;
    __device__ __forceinline__ explicit Scale(float scale) : s(scale), y(1.0f / scale) {}
    __device__ __forceinline__ Scale(float scale, float recip) : s(scale), y(recip) {}
};

// x / s rounded to nearest, as the division instruction sequence would give it,
// from y = RN(1 / s).  q0 = x * y is within two units in the last place of the
// quotient; the remainder x - s * q is exact in one fused operation, and adding
// remainder * y first gives a faithful quotient and then the correctly rounded
// one (Markstein's correction step, twice).  Needs no overflow and an exactly
// representable remainder: scales are >= 1e-8, so a quotient that can reach 0.5
// has a normal x, and smaller quotients round to code 0 whatever their last bits
// are.  GUARD: quotients beyond 1e6 in magnitude (possible only with a scale the
// data has outgrown) are left as x * y, far out in the clamped range, so that the
// correction never sees an infinity.
template <bool GUARD>
__device__ __forceinline__ float quotient(float x, Scale sc)
{
    const float q0 = x * sc.y;
    float q = __builtin_fmaf(__builtin_fmaf(-sc.s, q0, x), sc.y, q0);
    q = __builtin_fmaf(__builtin_fmaf(-sc.s, q, x), sc.y, q);
    if (GUARD) q = __builtin_fabsf(q0) < 1e6f ? q : q0;
    return q;
}

// the code as an integer in [lo, hi]
template <bool GUARD>
__device__ __forceinline__ int code_i(float x, Scale sc, float lo, float hi)
{
    return (int)__builtin_amdgcn_fmed3f(__builtin_rintf(quotient<GUARD>(x, sc)), lo, hi);
}

// INT4 code of a weight: the scale may be stale (Sec. 3.2), so the quotient is guarded and the clamp is live
__device__ __forceinline__ int int4_code(float w, Scale sc) { return code_i<true>(w, sc, -8.0f, 7.0f); }
// INT8 code of a gradient value under a scale the caller supplied
__device__ __forceinline__ int int8_code(float g, Scale sc) { return code_i<true>(g, sc, -128.0f, 127.0f); }
// ... under a scale derived from the maximum of the very values being quantised: |g / s| <= 127 (1 + 2^-23)
__device__ __forceinline__ int int8_code_fresh(float g, Scale sc) { return code_i<false>(g, sc, -128.0f, 127.0f); }

// four codes -> four bytes, element 0 in the low byte
__device__ __forceinline__ unsigned pack_bytes(int q0, int q1, int q2, int q3)
{
    return ((unsigned)q0 & 0xFFu) | (((unsigned)q1 & 0xFFu) << 8) | (((unsigned)q2 & 0xFFu) << 16) | ((unsigned)q3 << 24);
}

// unsigned division of numbers below 2^31 by a fixed divisor (host-side set-up)
struct FastDiv {
    unsigned magic, shift, d;
    __host__ static FastDiv make(unsigned divisor)
    {
        FastDiv f;
        unsigned l = 0;
        while ((1u << l) < divisor) ++l;
        // ceil(2^(31 + l) / d) < 2^32 for d >= 2; exact quotients for every dividend below 2^31
        const unsigned long long p = 1ull << (31 + l);
        f.magic = divisor > 1 ? (unsigned)((p + divisor - 1) / divisor) : 0u;
        f.shift = l > 0 ? l - 1 : 0;
        f.d = divisor;
        return f;
    }
    __device__ __forceinline__ unsigned div(unsigned x) const { return d > 1 ? __umulhi(x, magic) >> shift : x; }
};

// sign-extend the low 4 bits of v
__device__ __forceinline__ int nibble_code(unsigned v) { return (int)((v & 0xFu) ^ 8u) - 8; }

// four codes -> two bytes, element 0 in the low nibble of byte 0
__device__ __forceinline__ unsigned pack4(int q0, int q1, int q2, int q3)
{
    return ((unsigned)q0 & 0xFu) | (((unsigned)q1 & 0xFu) << 4) | (((unsigned)q2 & 0xFu) << 8) | (((unsigned)q3 & 0xFu) << 12);
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

// exclusive prefix sum over the threads of a block of kWaves waves; *total = sum of all
template <int kWaves>
__device__ __forceinline__ int block_excl_scan_add(int v, int lane, int wave, int *s_w, int *total)
{
    const int incl = wave_incl_scan_add(v, lane);
    __syncthreads(); // s_w may still be read from a previous use
    if (lane == kWave - 1) s_w[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const int x = s_w[w];
        if (w < wave) base += x;
        tot += x;
    }
    *total = tot;
    return base + incl - v;
}

// lanes of the wave whose 8-bit digit equals mine (all 64 lanes must be active)
__device__ __forceinline__ unsigned long long match_any8(unsigned d)
{
    // per bit: the lanes whose bit is set (ballot) against my own bit spread over a word (0 or all ones, a signed
    // one-bit field extract): the lanes whose bit equals mine are ~(ballot ^ mine), and gfx950 folds that and the
    // running AND into one three-input bit operation per 32-bit half
    unsigned lo = ~0u, hi = ~0u;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        unsigned mine = (unsigned)(int)__builtin_amdgcn_sbfe(d, b, 1);
        asm volatile("" : "+v"(mine)); // (keeps the compiler from deriving the ballot from d again: a shift more per bit)
        const unsigned long long bal = __ballot(mine != 0u);
        lo &= ~((unsigned)bal ^ mine);
        hi &= ~((unsigned)(bal >> 32) ^ mine);
    }
    return ((unsigned long long)hi << 32) | lo;
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
