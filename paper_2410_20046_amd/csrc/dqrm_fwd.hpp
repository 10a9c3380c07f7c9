// Forward: gather -> INT4 fake-quant -> sum-pool (Sec. 3.1 and Sec. 4.1 of the paper).
//
// A workgroup owns a tile of kFwdTileB consecutive samples x up to kFwdTileT
// consecutive tables.  The index arrays are table-major (bag = t * B + b), the
// output is sample-major (slot = b * T + t): with 16 samples per tile every
// 128-byte line of `offsets` / `indices` is read by one workgroup only, and with
// all tables in the tile (T <= kFwdTileT) the workgroup's output is one
// contiguous piece of `out`.  Three phases, each one memory round trip deep, so
// the dependent chain offsets -> index -> row is paid once per workgroup:
//   A  one thread per bag (sample fastest, so the reads coalesce) reads the
//      bag's extent and first index, checks them, and leaves the row's byte
//      offset, the table scale and the output slot in LDS, filed in output order;
//   B  groups of G = pow2ceil(D/4) lanes walk the tile in output order; lane l
//      of a group owns columns 4l..4l+3 (one 16-byte store per row).  The first
//      rows of a whole batch of slots are requested before any is used;
//   C  `out = 0 + s * q` is stored.  Tiles with a bag of more than one lookup take the
//      general path instead: the tile's index lists are turned into checked row
//      offsets in LDS by all threads (one more round trip for the whole tile), then
//      every bag's rows are requested kFwdBagBatch at a time and added in order.
// The per-column sum is the plain left-to-right sum over the bag, so no
// cross-lane reduction is needed and the result does not depend on the mapping.
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

constexpr int kFwdTileB = 16;                      // samples per tile
constexpr int kFwdTileT = 32;                      // tables per tile, at most
constexpr int kFwdSlots = kFwdTileB * kFwdTileT;   // bags per tile, at most
constexpr int kFwdThreads = 512;
constexpr int kFwdBatch = 16;                      // first rows in flight per lane
constexpr int kFwdLdsLookups = 4096;               // lookups of a tile whose row offsets fit in LDS (general bags)
constexpr int kFwdBagBatch = 8;                    // rows of one bag in flight per lane (general bags)

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
    int T, B, D;
    int tile_t;  // tables per tile: min(T, kFwdTileT); gridDim = (ceil(B / kFwdTileB), ceil(T / tile_t))
    int no_rows; // the tables hold no row at all: nothing may be read from them
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store_codes(int8_t *codes, int64_t i, int D, int col, float4 q)
{
    char4 c = make_char4((signed char)(int)q.x, (signed char)(int)q.y, (signed char)(int)q.z, (signed char)(int)q.w);
    *reinterpret_cast<char4 *>(codes + i * D + col) = c;
}

// The raw bytes of 4 consecutive elements of one row as they come from memory:
// two packed bytes, or four fp32 values.
template <bool PACKED> struct RowPiece;
template <> struct RowPiece<true> {
    unsigned v;
    __device__ __forceinline__ void load(const char *p) { v = *reinterpret_cast<const unsigned short *>(p); }
    __device__ __forceinline__ float4 codes(Scale) const
    {
        // the builtin's result is typed unsigned although the extract sign-extends
        return make_float4((float)(int)__builtin_amdgcn_sbfe((int)v, 0, 4), (float)(int)__builtin_amdgcn_sbfe((int)v, 4, 4),
                           (float)(int)__builtin_amdgcn_sbfe((int)v, 8, 4), (float)(int)__builtin_amdgcn_sbfe((int)v, 12, 4));
    }
};
template <> struct RowPiece<false> {
    float4 w;
    __device__ __forceinline__ void load(const char *p) { w = *reinterpret_cast<const float4 *>(p); }
    __device__ __forceinline__ float4 codes(Scale s) const
    {
        return make_float4((float)int4_code(w.x, s), (float)int4_code(w.y, s), (float)int4_code(w.z, s),
                           (float)int4_code(w.w, s));
    }
};

// The slots of the tile in output order when no bag has more than one lookup (the usual batch):
// out = 0 + s * q, nothing else to add.  A slot without a valid lookup reads row 0 and multiplies by 0;
// the addition turns a -0 product into the +0 of an empty sum.  Slots from `live` on do not exist
// (samples beyond the batch); their LDS entries read as "no lookup".
template <int G, bool PACKED>
__device__ __forceinline__ void fwd_single_lookup_tile(const char *tab, const int64_t *s_off, const Scale *s_scale,
                                                       const float *s_mul, const int *s_slot, int grp, float *out_col,
                                                       int D, int live)
{
    constexpr int kGroups = kFwdThreads / G;
    constexpr int kIters = (kFwdSlots + kGroups - 1) / kGroups;
    constexpr int kBatch = kIters < kFwdBatch ? kIters : kFwdBatch;
    for (int k0 = 0; k0 * kGroups < live; k0 += kBatch) {
        RowPiece<PACKED> piece[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const int i = min((k0 + k) * kGroups + grp, kFwdSlots - 1);
            piece[k].load(tab + s_off[i]);
        }
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const int i = (k0 + k) * kGroups + grp;
            if (i < live) {
                const float m = s_mul[i];
                const float4 q = piece[k].codes(s_scale[i]);
                const f32x4 v = {0.f + m * q.x, 0.f + m * q.y, 0.f + m * q.z, 0.f + m * q.w};
                // (plain stores: the consumer of `out`, the dense part of the model, runs next and finds it in the caches)
                *reinterpret_cast<f32x4 *>(out_col + (size_t)(unsigned)s_slot[i] * D) = v;
            }
        }
    }
}

template <int G, bool PACKED>
__global__ __launch_bounds__(kFwdThreads) void embbag_fwd_kernel(FwdArgs a)
{
    __shared__ int64_t s_off[kFwdSlots]; // byte offset of the first lookup's row in the table (0 if none / invalid)
    __shared__ int64_t s_beg[kFwdSlots]; // position of the bag's first lookup
    __shared__ int s_len[kFwdSlots];     // lookups in the bag
    __shared__ int s_tab[kFwdSlots];
    __shared__ int s_slot[kFwdSlots];    // output slot b * T + t (below 2^31: checked on the host)
    __shared__ Scale s_scale[kFwdSlots]; // table scale (and its reciprocal)
    __shared__ float s_mul[kFwdSlots];   // table scale, or 0 when the first lookup is absent or invalid
    __shared__ unsigned char s_ok[kFwdSlots]; // the first lookup exists and is in range
    __shared__ int s_general;            // some bag of the tile has more than one lookup
    __shared__ int64_t s_loff[kFwdLdsLookups]; // general bags: row byte offset of every lookup of the tile, -1 if bad
    __shared__ int s_pos[kFwdSlots];     // ... where slot i's list starts in s_loff
    __shared__ int s_w[kFwdThreads / kWave];
    static_assert(kFwdSlots == kFwdThreads, "one slot per thread");

    const int tid = threadIdx.x;
    const int b0 = (int)blockIdx.x * kFwdTileB, t0 = (int)blockIdx.y * a.tile_t;
    const int nb = min(kFwdTileB, a.B - b0), nt = min(a.tile_t, a.T - t0); // samples / tables of this tile
    const int live = nb * nt;                                              // its slots, a prefix in output order
    const int row_bytes = PACKED ? (a.D >> 1) : a.D * 4;
    if (tid == 0) s_general = 0;
    __syncthreads();

    // ---- phase A: one bag per thread, sample fastest ---------------------------
    for (int s = tid; s < kFwdSlots; s += kFwdThreads) {
        const int bl = s % kFwdTileB, tl = s / kFwdTileB;
        const bool exists = bl < nb && tl < nt;
        // output-order index inside the tile; the entries past `live` are filled with "no lookup"
        int i = bl * nt + tl;
        if (!exists) i = tl < nt ? live + (bl - nb) * nt + tl : s;
        int64_t off = 0, beg = 0;
        int len = 0;
        const int t = exists ? t0 + tl : 0, b = b0 + bl;
        float sc = 1.0f, mul = 0.0f;
        bool ok = false;
        if (exists) {
            const int64_t bag = (int64_t)t * a.B + b;
            int64_t lo = a.offsets[bag], hi = a.offsets[bag + 1];
            if (lo < 0 || hi > a.num_indices || lo > hi) {
                report(DQRM_ERR_BAD_OFFSETS, t, bag);
                lo = hi = 0;
            }
            if (hi - lo > 0x7fffffff) hi = lo + 0x7fffffff;
            beg = lo;
            len = (int)(hi - lo);
            sc = a.w_scale[t];
            if (len > 0) {
                const int64_t idx = a.indices[lo];
                const int64_t r0 = a.row_offsets[t], r1 = a.row_offsets[t + 1];
                if (idx >= 0 && idx < r1 - r0) {
                    off = (r0 + idx) * row_bytes;
                    mul = sc;
                    ok = true;
                } else {
                    report(DQRM_ERR_INDEX_OUT_OF_RANGE, t, idx);
                }
                if (len > 1) s_general = 1;
            }
        }
        s_off[i] = off;
        s_beg[i] = beg;
        s_len[i] = len;
        s_tab[i] = t;
        s_slot[i] = exists ? b * a.T + t : 0;
        // the packed rows hold codes already: no quotient, no reciprocal
        s_scale[i] = PACKED ? Scale(sc, 0.0f) : Scale(sc);
        s_mul[i] = mul;
        s_ok[i] = ok;
    }
    __syncthreads();

    // ---- general bags: the tile's lookups as checked row offsets in LDS ------------------
    const bool general = s_general != 0 || a.codes != nullptr || a.no_rows != 0;
    bool staged = false;
    if (general && !a.no_rows) {
        // position of every slot's list in s_loff (slots in output order; kFwdThreads == kFwdSlots)
        const int my_len = tid < live ? s_len[tid] : 0;
        int total;
        const int pos = block_excl_scan_add<kFwdThreads / kWave>(my_len, tid & (kWave - 1), tid / kWave, s_w, &total);
        s_pos[tid] = pos;
        staged = total <= kFwdLdsLookups; // block-uniform
        if (staged && my_len > 0) {
            const int t = s_tab[tid];
            const int64_t r0 = a.row_offsets[t], r1 = a.row_offsets[t + 1];
            const int64_t beg = s_beg[tid];
            for (int j0 = 0; j0 < my_len; j0 += kFwdBagBatch) {
                int64_t idx[kFwdBagBatch];
#pragma unroll
                for (int j = 0; j < kFwdBagBatch; ++j) idx[j] = a.indices[beg + min(j0 + j, my_len - 1)];
#pragma unroll
                for (int j = 0; j < kFwdBagBatch; ++j) {
                    if (j0 + j >= my_len) break;
                    int64_t off = -1;
                    if (idx[j] >= 0 && idx[j] < r1 - r0)
                        off = (r0 + idx[j]) * row_bytes;
                    else
                        report(DQRM_ERR_INDEX_OUT_OF_RANGE, t, idx[j]);
                    s_loff[pos + j0 + j] = off;
                }
            }
        }
        __syncthreads();
    }

    // ---- phases B and C ------------------------------------------------------------
    constexpr int kGroups = kFwdThreads / G; // groups per workgroup
    const int lg = tid & (G - 1);
    const int grp = tid / G;
    const int col = lg * 4;
    if (col >= a.D) return; // lanes beyond the row (D / 4 not a power of two) have nothing to do from here on
    const char *tab = PACKED ? reinterpret_cast<const char *>(a.packed) + (col >> 1)
                             : reinterpret_cast<const char *>(a.master + col);
    float *out_col = a.out + col;

    if (!general) {
        fwd_single_lookup_tile<G, PACKED>(tab, s_off, s_scale, s_mul, s_slot, grp, out_col, a.D, live);
        return;
    }

    if (staged) {
        // A bag's rows kFwdBagBatch at a time, none under a branch: a lookup past the bag's end or with a bad
        // index reads row 0 and enters the sum as 0 * q, which leaves the sum as it is.
        for (int i = grp; i < live; i += kGroups) {
            const Scale sq = s_scale[i];
            const int len = s_len[i], pos = s_pos[i];
            const int64_t beg = s_beg[i];
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int j0 = 0; j0 < len; j0 += kFwdBagBatch) {
                RowPiece<PACKED> piece[kFwdBagBatch];
                float m[kFwdBagBatch];
#pragma unroll
                for (int j = 0; j < kFwdBagBatch; ++j) {
                    const int64_t off = s_loff[pos + min(j0 + j, len - 1)];
                    m[j] = (j0 + j < len && off >= 0) ? sq.s : 0.0f;
                    piece[j].load(tab + (off >= 0 ? off : 0));
                }
#pragma unroll
                for (int j = 0; j < kFwdBagBatch; ++j) {
                    const float4 q = piece[j].codes(sq);
                    acc.x = acc.x + m[j] * q.x;
                    acc.y = acc.y + m[j] * q.y;
                    acc.z = acc.z + m[j] * q.z;
                    acc.w = acc.w + m[j] * q.w;
                    if (a.codes && m[j] != 0.0f) store_codes(a.codes, beg + j0 + j, a.D, col, q);
                }
            }
            const f32x4 v = {acc.x, acc.y, acc.z, acc.w};
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(out_col + (size_t)(unsigned)s_slot[i] * a.D));
        }
        return;
    }

    // general bags of a tile with too many lookups for LDS, or tables without rows: one lookup at a time
    for (int i = grp; i < live; i += kGroups) {
        const Scale sq = s_scale[i];
        const float s = sq.s;
        const int len = s_len[i];
        const int64_t beg = s_beg[i];
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (len > 0 && !a.no_rows) {
            const int t = s_tab[i];
            const int64_t r0 = a.row_offsets[t], r1 = a.row_offsets[t + 1];
            for (int64_t p = beg; p < beg + len; ++p) {
                const int64_t idx = a.indices[p];
                if (idx < 0 || idx >= r1 - r0) {
                    if (lg == 0 && p > beg) report(DQRM_ERR_INDEX_OUT_OF_RANGE, t, idx); // (the first one: phase A)
                    continue;
                }
                RowPiece<PACKED> piece;
                piece.load(tab + (r0 + idx) * row_bytes);
                const float4 q = piece.codes(sq);
                acc.x = acc.x + s * q.x;
                acc.y = acc.y + s * q.y;
                acc.z = acc.z + s * q.z;
                acc.w = acc.w + s * q.w;
                if (a.codes) store_codes(a.codes, p, a.D, col, q);
            }
        }
        const f32x4 v = {acc.x, acc.y, acc.z, acc.w};
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(out_col + (size_t)(unsigned)s_slot[i] * a.D));
    }
}

} // namespace dqrm
