// The dense part of the DLRM train step (model-architecture table of the paper):
// bottom MLP -> pairwise-dot interaction with the pooled embeddings -> top MLP ->
// sigmoid + mean binary cross-entropy, its backward, and plain SGD on the MLP
// weights.  FP32 throughout (the paper's "MLP in FP32" variant); the matrix
// products run on the matrix cores (v_mfma_f32_32x32x2_f32).
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// C(i,j) = epilogue( sum_r A(i,r) * B(r,j) ), all operands addressed with
// explicit strides so that one kernel serves X*W^T, dY*W and dY^T*X.
//
// One wave owns a 32x32 tile of C: it keeps the tile in the 16 accumulator
// registers of v_mfma_f32_32x32x2_f32 and walks the reduction in slabs of 32.
// In a slab, lane l = (h, w) with w = l % 32, h = l / 32 holds
// A(i0 + w, r0 + 16 h + s) and B(r0 + 16 h + s, j0 + w) for s = 0..15 and issues
// 16 products, the s-th pairing r0 + s (lanes h = 0) with r0 + 16 + s (lanes
// h = 1): every r of the slab is used once, in an order that is the same for
// both operands.  Two slabs are in flight from memory, and the slab after the
// current one is brought into that register layout while the current one is
// multiplied.
//
// How an operand's slab reaches the register layout depends on its memory layout
// (the kOp* forms below): read along its unit-stride index with 16-byte loads and
// passed through a per-wave piece of LDS, or, when the 32-wide index is the
// unit-stride one, also with 4-byte loads straight into place.  Nothing assumes
// an alignment beyond 4 bytes.  No load sits under a branch: indices past the
// edge are clamped and the value is replaced by 0 (or by 1 for the virtual
// all-ones last column of B).
//
// Several products can share one launch (the weight gradients of all layers):
// the waves are dealt over the tiles of all problems.  With splits > 1 the
// reduction is cut: slice z covers r in [z*k_per_split, ...) and stores its raw
// partial tile to P[z][M][N]; sgd_from_partials_kernel adds the slices in order.
// With kslices > 1 (one product per launch) the waves of a workgroup share tiles
// and add their accumulators through LDS instead.
struct GemmArgs {
    const float *A;
    long long a_si, a_sr;
    const float *B;
    long long b_sr, b_sj;
    float *C;
    long long c_si, c_sj;
    int M, N, K;
    const float *bias; // [N] added per column j, or null
    const float *mask; // same addressing as C: result multiplied by (mask > 0), or null
    int relu;          // max(x, 0) after the bias
    int b_ones_last;   // B's last column (j = N-1) is all ones and is not read from memory
    int splits;        // slices of the reduction (1: the epilogue above; > 1: partial tiles to P)
    int k_per_split;   // reduction length per slice (multiple of 32), K if not split
    float *P;          // [splits][M][N] partial tiles when split
    int tile_begin;    // first wave-tile of this problem in the launch (filled by the launcher)
};

constexpr int kGemmMaxGroup = 16;
struct GemmGroup {
    GemmArgs p[kGemmMaxGroup];
    int count, total_tiles;
};

constexpr int kGemmThreads = 256;
constexpr int kGemmWaves = kGemmThreads / kWave;
constexpr int kGemmBK = 32;      // reduction slab
constexpr int kGemmPitch = 36;   // LDS row pitch of a turned slab (floats): rows stay 16-byte aligned

struct SlabRegs {
    float v[16];
};

// Wide-contiguous operand: element (wide, r) at base[wide * sw + r * sr].  Lane (h, w) reads
// r = r0 + 16 h + s, s = 0..15, of its own wide index.  SAFE: the wide index was clamped by the caller and r
// is clamped / zeroed here (the last partial slab, tiles of operands narrower than 32); otherwise everything
// is known to be inside.
template <bool SAFE>
__device__ __forceinline__ void slab_load_direct(SlabRegs &x, const float *base, long long sw, long long sr, int wide,
                                                 int r0, int r_end, int h, bool ones)
{
    if (!SAFE) {
        const float *p = base + (long long)wide * sw + (long long)(r0 + 16 * h) * sr;
#pragma unroll
        for (int s = 0; s < 16; ++s) x.v[s] = p[(long long)s * sr];
        return;
    }
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const int r = r0 + 16 * h + s;
        const int rc = min(r, r_end - 1);
        const float val = base[(long long)wide * sw + (long long)rc * sr];
        x.v[s] = r < r_end ? (ones ? 1.0f : val) : 0.0f;
    }
}

// Reduction-contiguous operand: element (wide, r) at base[wide * sw + r], clamped form.  Step 1: lane l reads
// r = r0 + l % 32 of the tile's rows 2 it + l / 32, it = 0..15 (first_wide = the tile's first wide index,
// n_wide = the operand's extent in that index).
__device__ __forceinline__ void slab_load_along_r(SlabRegs &x, const float *base, long long sw, int first_wide,
                                                  int n_wide, int r0, int r_end, int lane)
{
    const int r = r0 + (lane & 31);
    const int rc = min(r, r_end - 1);
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int wide = min(first_wide + 2 * it + (lane >> 5), n_wide - 1);
        const float val = base[(long long)wide * sw + rc];
        x.v[it] = r < r_end ? val : 0.0f;
    }
}

// step 2: through the wave's LDS piece into the product layout
__device__ __forceinline__ void slab_turn(SlabRegs &x, const SlabRegs &st, float *lds, int lane)
{
#pragma unroll
    for (int it = 0; it < 16; ++it) lds[(2 * it + (lane >> 5)) * kGemmPitch + (lane & 31)] = st.v[it];
    // (same wave: the LDS operations complete in order, no barrier needed)
    const float4 *row = reinterpret_cast<const float4 *>(lds + (lane & 31) * kGemmPitch + 16 * (lane >> 5));
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
        const float4 q = row[s4];
        x.v[4 * s4 + 0] = q.x, x.v[4 * s4 + 1] = q.y, x.v[4 * s4 + 2] = q.z, x.v[4 * s4 + 3] = q.w;
    }
}

// How the whole slabs of an operand are read (template parameters of the kernel):
//   kOpRC       the reduction index is the unit-stride one: 16-byte loads along it, turned through LDS
//   kOpWide     the 32-wide index is the unit-stride one: 4-byte loads straight into place, each lane from its own
//               (possibly clamped) wide index - the form that can serve a virtual all-ones column
//   kOpWideVec  the same layout read with 16-byte loads along the wide index, through LDS: only for tiles whose
//               32 wide indices all exist
// The last partial slab, and kOpWideVec tiles of operands narrower than 32, take the clamped 4-byte path instead.
enum { kOpRC = 0, kOpWide = 1, kOpWideVec = 2 };

// four floats that are only known to start on a 4-byte boundary (a 16-byte global load needs no more)
typedef float Float4Dw __attribute__((ext_vector_type(4), aligned(4)));

// `first_wide`: the tile's first wide index, `n_wide`: the operand's extent in it (kOpRC reads row n_wide - 1 in
// place of the rows past it; kOpWideVec needs all 32 to exist); `wide`: this lane's own, clamped (kOpWide only)
template <int MODE>
__device__ __forceinline__ void slab_fetch_fast(SlabRegs &st, const float *base, long long sw, long long sr,
                                                int first_wide, int n_wide, int wide, int r0, int lane)
{
    // lane l reads four consecutive floats (l % 8) * 4 .. + 3 of lines l / 8 + 8 it, it = 0..3; a line is a
    // row of the operand (kOpRC: along r) or one reduction index (kOpWideVec: along the wide index)
    const int line = lane >> 3, c4 = (lane & 7) * 4;
    if (MODE == kOpWide) {
        slab_load_direct<false>(st, base, sw, sr, wide, r0, 0, lane >> 5, false);
    } else if (MODE == kOpRC) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int row = min(first_wide + line + 8 * it, n_wide - 1);
            const Float4Dw q = *reinterpret_cast<const Float4Dw *>(base + (long long)row * sw + (r0 + c4));
            st.v[4 * it + 0] = q.x, st.v[4 * it + 1] = q.y, st.v[4 * it + 2] = q.z, st.v[4 * it + 3] = q.w;
        }
    } else {
        const float *p = base + (long long)(r0 + line) * sr + (first_wide + c4);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const Float4Dw q = *reinterpret_cast<const Float4Dw *>(p + (long long)(8 * it) * sr);
            st.v[4 * it + 0] = q.x, st.v[4 * it + 1] = q.y, st.v[4 * it + 2] = q.z, st.v[4 * it + 3] = q.w;
        }
    }
}

// staging registers of a whole slab -> product layout (`ones`: this lane's column is the virtual one)
template <int MODE>
__device__ __forceinline__ void slab_settle_fast(SlabRegs &x, const SlabRegs &st, float *lds, int lane, bool ones)
{
    if (MODE == kOpWide) {
#pragma unroll
        for (int s = 0; s < 16; ++s) x.v[s] = ones ? 1.0f : st.v[s];
    } else {
        const int line = lane >> 3, c4 = (lane & 7) * 4;
#pragma unroll
        for (int it = 0; it < 4; ++it)
            *reinterpret_cast<float4 *>(lds + (line + 8 * it) * kGemmPitch + c4) =
                make_float4(st.v[4 * it + 0], st.v[4 * it + 1], st.v[4 * it + 2], st.v[4 * it + 3]);
        // (same wave: the LDS operations complete in order, no barrier needed)
        const int w = lane & 31, h = lane >> 5;
        if (MODE == kOpRC) { // LDS holds [wide][r]: 16 consecutive r of my wide index
            const float4 *row = reinterpret_cast<const float4 *>(lds + w * kGemmPitch + 16 * h);
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const float4 q = row[s4];
                x.v[4 * s4 + 0] = q.x, x.v[4 * s4 + 1] = q.y, x.v[4 * s4 + 2] = q.z, x.v[4 * s4 + 3] = q.w;
            }
        } else { // LDS holds [r][wide]: my wide index of 16 consecutive r
#pragma unroll
            for (int s = 0; s < 16; ++s) x.v[s] = lds[(16 * h + s) * kGemmPitch + w];
        }
    }
}

// the tile `tile` (and, with ks > 1, the slice wave % ks of its reduction) of problem g, by one wave
template <int A_MODE, int B_MODE>
__device__ __forceinline__ void gemm_wave_tile(const GemmArgs &g, int tile, bool live, int ks, int wave, int lane)
{
    constexpr bool A_RC = A_MODE == kOpRC, B_RC = B_MODE == kOpRC;
    __shared__ __align__(16) float turn[kGemmWaves][2][32 * kGemmPitch]; // per wave: LDS pieces of A and B
    const int kz = wave & (ks - 1);
    const int tiles_j = (g.N + 31) / 32, tiles_i = (g.M + 31) / 32;
    int local = tile - g.tile_begin;
    const int z = local / (tiles_i * tiles_j);
    local -= z * tiles_i * tiles_j;
    const int i_first = (local / tiles_j) * 32, j_first = (local % tiles_j) * 32; // first row / column this tile stores
    // this wave's part of the reduction: slice z of a split product, or slice kz of the workgroup's
    const int k_per_wave = ks > 1 ? ((g.K + 2 * kGemmBK * ks - 1) / (2 * kGemmBK * ks)) * (2 * kGemmBK) : g.k_per_split;
    const int r_begin = ks > 1 ? kz * k_per_wave : z * g.k_per_split;
    const int r_end = live ? min(g.K, r_begin + k_per_wave) : r_begin;
    const int w = lane & 31, h = lane >> 5;

    // The last tile of a dimension that is not a multiple of 32 is moved back so that it ends at the edge: it
    // recomputes a few rows / columns of its neighbour, stores only its own, and reads whole slabs like any
    // other.  Operands narrower than 32 cannot: their tiles re-read the last row / column (clamped indices)
    // and those results are not stored.  The all-ones last column of B is virtual (kOpWide only: host): its lane
    // reads the column before it and the value is replaced.
    const int n_mem = g.b_ones_last ? g.N - 1 : g.N; // columns of B that exist in memory (>= 1: host)
    const int i0 = (i_first + 32 > g.M && g.M >= 32) ? g.M - 32 : i_first;
    const int j0 = (j_first + 32 > g.N && g.N >= 32) ? g.N - 32 : j_first;
    // whole slabs can be read the fast way (kOpWideVec: only if the tile's 32 rows / columns all exist)
    const bool whole = (A_MODE != kOpWideVec || i0 + 32 <= g.M) && (B_MODE != kOpWideVec || j0 + 32 <= g.N);
    const int ia = min(i0 + w, g.M - 1), jb = min(j0 + w, n_mem - 1);
    const bool ones = g.b_ones_last && j0 + w == g.N - 1;
    float *lds_a = turn[wave][0], *lds_b = turn[wave][1];
    // (requested now, used in the epilogue)
    const float bias_j = (g.bias && g.splits <= 1) ? g.bias[min(j0 + w, g.N - 1)] : 0.0f;
    // ... and so is the mask of this lane's 16 outputs (rows and columns past the edge re-read the last ones)
    float mask_v[16];
    if (g.mask && g.splits <= 1) {
        const long long mj = (long long)min(j0 + w, g.N - 1) * g.c_sj;
#pragma unroll
        for (int v = 0; v < 16; ++v)
            mask_v[v] = g.mask[(long long)min(i0 + 8 * (v >> 2) + 4 * h + (v & 3), g.M - 1) * g.c_si + mj];
    } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) mask_v[v] = 1.0f;
    }

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    // Two slabs are in flight while a third is multiplied: sa[q] / sb[q] receive slab n with n % 2 == q as it
    // comes from memory, a / b hold the current slab in product layout.
    SlabRegs a, b, sa[2], sb[2];
    auto fetch_safe = [&](int q, int r0) {
        if (A_RC)
            slab_load_along_r(sa[q], g.A, g.a_si, i0, g.M, r0, r_end, lane);
        else
            slab_load_direct<true>(sa[q], g.A, g.a_si, g.a_sr, ia, r0, r_end, h, false);
        if (B_RC)
            slab_load_along_r(sb[q], g.B, g.b_sj, j0, n_mem, r0, r_end, lane);
        else
            slab_load_direct<true>(sb[q], g.B, g.b_sj, g.b_sr, jb, r0, r_end, h, ones);
    };
    auto fetch_fast = [&](int q, int r0) { // whole tile, whole slab
        slab_fetch_fast<A_MODE>(sa[q], g.A, g.a_si, g.a_sr, i0, g.M, ia, r0, lane);
        slab_fetch_fast<B_MODE>(sb[q], g.B, g.b_sj, g.b_sr, j0, n_mem, jb, r0, lane);
    };
    auto settle_fast = [&](int q) {
        slab_settle_fast<A_MODE>(a, sa[q], lds_a, lane, false);
        slab_settle_fast<B_MODE>(b, sb[q], lds_b, lane, ones);
    };
    auto settle = [&](int q) { // staging registers of the clamped path -> product layout
        if (A_RC)
            slab_turn(a, sa[q], lds_a, lane);
        else
            a = sa[q];
        if (B_RC)
            slab_turn(b, sb[q], lds_b, lane);
        else
            b = sb[q];
    };
    auto products = [&]() {
#pragma unroll
        for (int s = 0; s < 16; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[s], b.v[s], acc, 0, 0, 0);
    };

    // Pairs of whole slabs of a whole tile.  The loop bodies below have no branch and every fetch is
    // unconditional, so that the loads in flight are the same, in number and order, on entry and on the way
    // round: only then does the compiler wait for exactly the slab it needs.  (A fetch past the fast part
    // re-reads its last pair of slabs: harmless.)
    int r0 = r_begin;
    const int r_pairs = whole ? r_begin + (r_end - r_begin) / (2 * kGemmBK) * (2 * kGemmBK) : r_begin;
    if (r0 < r_pairs) {
        const int r_last = r_pairs - 2 * kGemmBK;
        // a2 / b2: the slab after the current one is brought into product layout while the current one is
        // multiplied (the matrix core runs on its own once a product is issued; the LDS traffic of the turn
        // goes out in its shadow)
        SlabRegs a2, b2;
        fetch_fast(0, r0);
        __builtin_amdgcn_sched_barrier(0);
        fetch_fast(1, r0 + kGemmBK);
        __builtin_amdgcn_sched_barrier(0);
        settle_fast(0);
        __builtin_amdgcn_sched_barrier(0);
        for (; r0 < r_pairs; r0 += 2 * kGemmBK) {
            const int rn = min(r0 + 2 * kGemmBK, r_last);
            fetch_fast(0, rn);
            __builtin_amdgcn_sched_barrier(0);
            slab_settle_fast<A_MODE>(a2, sa[1], lds_a, lane, false);
            slab_settle_fast<B_MODE>(b2, sb[1], lds_b, lane, ones);
            products();
            __builtin_amdgcn_sched_barrier(0);
            fetch_fast(1, rn + kGemmBK);
            __builtin_amdgcn_sched_barrier(0);
            slab_settle_fast<A_MODE>(a, sa[0], lds_a, lane, false);
            slab_settle_fast<B_MODE>(b, sb[0], lds_b, lane, ones);
#pragma unroll
            for (int s = 0; s < 16; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a2.v[s], b2.v[s], acc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // what is left: at most one whole and one partial slab of a whole tile, or everything of a clamped tile
    // (past the end: clamped addresses, zeros, and a product that adds nothing)
    if (r0 < r_end) {
        fetch_safe(0, r0);
        fetch_safe(1, r0 + kGemmBK);
        for (; r0 < r_end; r0 += 2 * kGemmBK) {
            settle(0);
            fetch_safe(0, r0 + 2 * kGemmBK);
            products();
            settle(1);
            fetch_safe(1, r0 + 3 * kGemmBK);
            products();
        }
    }

    // the slices of a tile meet: slice 0 adds the others' accumulators in order and goes on alone
    if (ks > 1) {
        float *mine = &turn[wave][0][0];
        if (kz > 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) mine[v * kWave + lane] = acc[v];
        }
        __syncthreads();
        if (kz > 0 || !live) return;
        for (int k = 1; k < ks; ++k) {
            const float *other = &turn[wave + k][0][0];
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] += other[v * kWave + lane];
        }
    }

    // accumulator layout: lane l holds column j = l % 32 and rows 8*(v/4) + 4*(l/32) + v%4, v = 0..15
    const int j = j0 + w;
    if (j < j_first || j >= g.N) return; // (a moved tile stores only its own columns and rows)
    if (g.splits > 1) {
        float *p = g.P + (long long)z * g.M * g.N;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (i >= i_first && i < g.M) p[(long long)i * g.N + j] = acc[v];
        }
        return;
    }
    const float bj = bias_j;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = i0 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (i < i_first || i >= g.M) continue;
        float x = acc[v] + bj;
        if (g.relu) x = fmaxf(x, 0.0f);
        const long long off = (long long)i * g.c_si + (long long)j * g.c_sj;
        x = mask_v[v] > 0.0f ? x : 0.0f;
        g.C[off] = x;
    }
}

// With kslices > 1 the waves of a workgroup meet at a barrier inside: a wave past the last tile stays, takes the
// last tile with an empty reduction and stores nothing.
struct GemmOne {
    GemmArgs p;
    int total_tiles, kslices;
};

// one product per launch
template <int A_MODE, int B_MODE>
__global__ __launch_bounds__(kGemmThreads) void gemm_wave_kernel(GemmOne one)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave); // wave-uniform, and known to be
    const int ks = one.kslices;
    int tile = ((int)blockIdx.x * kGemmWaves + wave) / ks;
    const bool live = tile < one.total_tiles;
    if (!live && ks == 1) return;
    gemm_wave_tile<A_MODE, B_MODE>(one.p, min(tile, one.total_tiles - 1), live, ks, wave, lane);
}

// several products in one launch (kslices == 1)
template <int A_MODE, int B_MODE>
__global__ __launch_bounds__(kGemmThreads) void gemm_wave_group_kernel(GemmGroup grp)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / kWave);
    const int tile = (int)blockIdx.x * kGemmWaves + wave;
    if (tile >= grp.total_tiles) return; // whole waves leave; no barrier inside with one slice
    int pi = 0;
#pragma unroll 1
    for (int q = 1; q < grp.count; ++q)
        if (tile >= grp.p[q].tile_begin) pi = q;
    gemm_wave_tile<A_MODE, B_MODE>(grp.p[pi], tile, true, 1, wave, lane);
}

// ---- a layer with a short input (the bottom MLP's first: 13 dense features) -------------------------------
// Y[b][o] = act(sum_k X[b][k] * W[o][k] + bias[o]) for K <= kSmallKMax: a product with a reduction this short is
// all launch and edge handling on the matrix cores.  A thread owns four consecutive outputs: their 4 K weights stay
// in registers while the thread walks the workgroup's kSmallKSamples samples, whose inputs sit in LDS.
constexpr int kSmallKMax = 16;
constexpr int kSmallKThreads = 128;
constexpr int kSmallKSamples = 4; // samples per workgroup
struct SmallKArgs {
    const float *X, *W, *bias;
    float *Y;
    int B, N, K, relu; // N a multiple of 4, bias and Y 16-byte aligned (host)
};

__global__ __launch_bounds__(kSmallKThreads) void linear_small_k_kernel(SmallKArgs a)
{
    __shared__ float xs[kSmallKSamples * kSmallKMax];
    const int N = a.N, K = a.K;
    const int b0 = (int)blockIdx.x * kSmallKSamples, nb = min(kSmallKSamples, a.B - b0);
    for (int e = threadIdx.x; e < kSmallKSamples * kSmallKMax; e += kSmallKThreads) {
        const int bl = e / kSmallKMax, k = e % kSmallKMax;
        xs[e] = (bl < nb && k < K) ? a.X[(long long)(b0 + bl) * K + k] : 0.0f;
    }
    __syncthreads();
    for (int o = (int)threadIdx.x * 4; o < N; o += kSmallKThreads * 4) {
        // (4-byte loads: a row of an odd number of floats starts on no wider boundary; all 4 K are requested at once,
        // past K the last weight is read again and meets a zero input)
        float wr[4][kSmallKMax];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int k = 0; k < kSmallKMax; ++k) wr[r][k] = a.W[(long long)(o + r) * K + min(k, K - 1)];
        const float4 bias = *reinterpret_cast<const float4 *>(a.bias + o);
        for (int bl = 0; bl < nb; ++bl) {
            float acc[4] = {bias.x, bias.y, bias.z, bias.w};
#pragma unroll
            for (int k = 0; k < kSmallKMax; ++k) {
                const float xv = xs[bl * kSmallKMax + k]; // zero past K
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = __builtin_fmaf(xv, wr[r][k], acc[r]);
            }
            if (a.relu) {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = fmaxf(acc[r], 0.0f);
            }
            *reinterpret_cast<float4 *>(a.Y + (long long)(b0 + bl) * N + o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        }
    }
}

// ---- the head: last linear layer (one output), sigmoid, binary cross-entropy, gradient w.r.t. its input ----
// z = X[b] . w + bias;  p = 1 / (1 + exp(-z));  term_b = -(y log max(p, 1e-12) + (1-y) log max(1-p, 1e-12));
// dz = (p - y) / B;  dX[b][k] = dz * w[k], masked by X[b][k] > 0 when X is a ReLU output.
// One wave per sample.  The mean of the terms is taken by loss_sum_block in the step's last kernel.
// (Block 0 also clears the `nzero` words at `zero`: the per-tensor gradient maxima of the INT8-gradient path,
// which are accumulated later in the same step.)
struct HeadArgs {
    const float *X;    // [B][in] input of the last top layer
    const float *w;    // [in] its weights (the ones the forward uses)
    const float *bias; // [1]
    const float *y;    // [B] labels
    float *z;          // [B] logits
    float *dz;         // [B]
    float *terms;      // [B] per-sample loss
    float *dX;         // [B][in]
    int relu_input;
    int B, in;
    unsigned *zero; // nzero words, zstride apart
    int nzero, zstride;
};

__global__ __launch_bounds__(256) void head_kernel(HeadArgs a)
{
    if (blockIdx.x == 0)
        for (int k = threadIdx.x; k < a.nzero; k += 256) a.zero[(long long)k * a.zstride] = 0u;
    const int lane = threadIdx.x & (kWave - 1);
    const int b = (int)blockIdx.x * (256 / kWave) + (int)threadIdx.x / kWave;
    if (b >= a.B) return;
    const float *x = a.X + (long long)b * a.in;
    float s = 0.0f;
    for (int k = lane; k < a.in; k += kWave) s += x[k] * a.w[k];
#pragma unroll
    for (int d = kWave / 2; d >= 1; d >>= 1) s += __shfl_xor(s, d, kWave); // (every lane ends with the same sum)
    const float z = s + a.bias[0];
    const float p = 1.0f / (1.0f + expf(-z));
    const float yy = a.y[b];
    const float dz = (p - yy) / (float)a.B;
    if (lane == 0) {
        a.z[b] = z;
        a.dz[b] = dz;
        a.terms[b] = -(yy * logf(fmaxf(p, 1e-12f)) + (1.0f - yy) * logf(fmaxf(1.0f - p, 1e-12f)));
    }
    float *dx = a.dX + (long long)b * a.in;
    for (int k = lane; k < a.in; k += kWave) {
        const float g = dz * a.w[k];
        dx[k] = (!a.relu_input || x[k] > 0.0f) ? g : 0.0f;
    }
}

// loss = mean of the per-sample terms, by one block of 256 threads (fixed order: strided partial sums, then a tree)
__device__ __forceinline__ void loss_sum_block(const float *terms, int B, float *loss)
{
    __shared__ float part[256];
    float s = 0.0f;
    for (int b = threadIdx.x; b < B; b += 256) s += terms[b];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = part[0] / (float)B;
}

// SGD step from the split products of [dZ^T * X | dZ^T * 1], all layers in one launch:
// layer q's P is [S][out][in + 1];  W[o][i] -= lr * sum_s P[s][o][i],  b[o] -= lr * sum_s P[s][o][in]
// (slices added in order).  elem_begin[q] = first element of layer q in the launch's flat index space.
struct SgdLayer {
    const float *P;
    float *W, *b;
    int S, out, in;
    long long elem_begin; // first element of the layer in this launch's index space
    long long flat_begin; // ... in the model's flat parameter order (see dqrm_dense_quant_t)
    int tensor0;          // index of the layer's weight tensor in that order (its bias is tensor0 + 1)
};
struct SgdGroup {
    SgdLayer l[kGemmMaxGroup];
    int count;
    long long total;
    float lr;
    // INT8 gradients with error compensation (distributed-training section): flat arrays over the model
    float *grads;        // [P] this step's FP32 gradients (before the residual is added)
    float *err;          // [P] residuals carried between steps, or null
    int8_t *codes;       // [P] INT8 codes out, or null
    unsigned *gmax_bits; // [tensors][kGradMaxSlots][kGradMaxStride] running max |g + e| per tensor (word 0 of each line), as bit
                         // patterns, zeroed before the step
    float *grad_scale;   // [tensors] out
    // Simulated data parallelism (FP32 gradients): the gradient is added to (or starts) the caller's buffer, flat
    // over the model like `grads`, and the parameters take the step from the buffer, or none at all
    float *buffer;     // [P], or null
    int buffer_add;    // the buffer already holds earlier micro-batches
    int buffer_update; // this micro-batch ends its group: parameter <- parameter - lr * buffer
    // The launch that ends the step has one more block than the parameters need: it turns the per-sample loss
    // terms into the mean (null otherwise).
    const float *loss_terms; // [batch]
    float *loss;
    int batch;
};

// blocks that work on the parameters; the extra one, if any, does its job here and the caller returns
__device__ __forceinline__ bool sgd_extra_block(const SgdGroup &grp, int &blocks)
{
    blocks = gridDim.x;
    if (!grp.loss_terms) return false;
    blocks -= 1;
    if ((int)blockIdx.x < blocks) return false;
    loss_sum_block(grp.loss_terms, grp.batch, grp.loss);
    return true;
}

// which layer of the group element e belongs to, and where inside it
struct SgdElem {
    int q, o, i; // layer, output row, input column (i == in: the bias)
    long long le;
};
__device__ __forceinline__ SgdElem sgd_elem(const SgdGroup &grp, long long e)
{
    SgdElem r;
    r.q = 0;
#pragma unroll 1
    for (int k = 1; k < grp.count; ++k)
        if (e >= grp.l[k].elem_begin) r.q = k;
    const SgdLayer &L = grp.l[r.q];
    r.le = e - L.elem_begin;
    r.o = (int)(r.le / (L.in + 1));
    r.i = (int)(r.le - (long long)r.o * (L.in + 1));
    return r;
}

constexpr int kSgdMaxSlices = 16; // slices of a split product, at most (the host's limit)

// the slices of one element, added in order; all of them are requested before the first is used (a slice
// index past the last re-reads the last slice and is left out)
__device__ __forceinline__ float sum_partials(const SgdLayer &L, long long le)
{
    const long long per = (long long)L.out * (L.in + 1);
    float p[kSgdMaxSlices];
#pragma unroll
    for (int z = 0; z < kSgdMaxSlices; ++z) p[z] = L.P[(long long)min(z, L.S - 1) * per + le];
    float s = 0.0f;
#pragma unroll
    for (int z = 0; z < kSgdMaxSlices; ++z)
        if (z < L.S) s += p[z];
    return s;
}

__global__ __launch_bounds__(256) void sgd_from_partials_kernel(SgdGroup grp)
{
    int blocks;
    if (sgd_extra_block(grp, blocks)) return;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < grp.total; e += (long long)blocks * 256) {
        const SgdElem x = sgd_elem(grp, e);
        const SgdLayer &L = grp.l[x.q];
        float s = sum_partials(L, x.le);
        if (grp.buffer) {
            float *slot = grp.buffer + L.flat_begin + x.le;
            if (grp.buffer_add) s = *slot + s;
            *slot = s;
            if (!grp.buffer_update) continue;
        }
        if (x.i < L.in)
            L.W[(long long)x.o * L.in + x.i] = L.W[(long long)x.o * L.in + x.i] - grp.lr * s;
        else
            L.b[x.o] = L.b[x.o] - grp.lr * s;
    }
}

// INT8 gradients, pass 1: the FP32 gradient of every parameter (slices added in order) goes to `grads`,
// and the maximum of |gradient + residual| of every tensor to gmax_bits (per-block maxima in LDS first).
constexpr int kMaxGradTensors = 2 * 2 * 16; // weights and bias of at most 16 + 16 layers
constexpr int kGradMaxSlots = 16;           // lines per tensor, a workgroup uses line blockIdx % 16: a large tensor's
                                            // ~700 workgroups would otherwise queue up at one line
constexpr int kGradMaxStride = 32;          // words between two maxima: one 128-byte line each (same-line
                                            // atomics from many workgroups serialise at the memory side)
__global__ __launch_bounds__(256) void grad_sum_absmax_kernel(SgdGroup grp)
{
    __shared__ unsigned s_max[kMaxGradTensors];
    for (int k = threadIdx.x; k < kMaxGradTensors; k += 256) s_max[k] = 0u;
    __syncthreads();
    // a thread keeps the running maximum of the tensor it is in and hands it over when the tensor changes
    int cur_t = -1;
    float cur_max = 0.0f;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < grp.total; e += (long long)gridDim.x * 256) {
        const SgdElem x = sgd_elem(grp, e);
        const SgdLayer &L = grp.l[x.q];
        const float s = sum_partials(L, x.le);
        const long long f = L.flat_begin + x.le;
        grp.grads[f] = s;
        const float gp = grp.err ? s + grp.err[f] : s;
        const int t = L.tensor0 + (x.i < L.in ? 0 : 1);
        if (t != cur_t) {
            if (cur_t >= 0 && cur_max > 0.0f) atomicMax(s_max + cur_t, __float_as_uint(cur_max));
            cur_t = t;
            cur_max = 0.0f;
        }
        cur_max = fmaxf(cur_max, fabsf(gp));
    }
    // usually the whole wave ends in one tensor: one LDS atomic per wave
    const int tt = wave_max_int(cur_t);
    if (__all(cur_t < 0 || cur_t == tt)) {
        const float m = wave_max(cur_max);
        if ((threadIdx.x & (kWave - 1)) == 0 && tt >= 0 && m > 0.0f) atomicMax(s_max + tt, __float_as_uint(m));
    } else if (cur_t >= 0 && cur_max > 0.0f) {
        atomicMax(s_max + cur_t, __float_as_uint(cur_max));
    }
    __syncthreads();
    for (int k = threadIdx.x; k < kMaxGradTensors; k += 256)
        if (s_max[k] != 0u)
            atomicMax(grp.gmax_bits + (k * kGradMaxSlots + (int)(blockIdx.x % kGradMaxSlots)) * kGradMaxStride, s_max[k]);
}

// pass 2: g' = g + e;  s = max(max|g'| / 127, 1e-8);  code = clamp(rint(g' / s), -128, 127);
// e <- g' - s * code;  parameter <- parameter - lr * (s * code)   (every operation rounded on its own)
__global__ __launch_bounds__(256) void grad_quant_ec_kernel(SgdGroup grp)
{
    __shared__ Scale s_scale[kMaxGradTensors];
    int blocks;
    if (sgd_extra_block(grp, blocks)) return;
    // the tensors of this launch's layers
    for (int k = threadIdx.x; k < 2 * grp.count; k += 256) {
        const int t = grp.l[k >> 1].tensor0 + (k & 1);
        unsigned m[kGradMaxSlots], mx = 0u;
#pragma unroll
        for (int q = 0; q < kGradMaxSlots; ++q) m[q] = grp.gmax_bits[(t * kGradMaxSlots + q) * kGradMaxStride];
#pragma unroll
        for (int q = 0; q < kGradMaxSlots; ++q) mx = max(mx, m[q]); // (non-negative floats order like their bits)
        const float gs = scale_from_absmax(__uint_as_float(mx), 127.0f);
        s_scale[t] = Scale(gs);
        if (blockIdx.x == 0) grp.grad_scale[t] = gs;
    }
    __syncthreads();
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < grp.total; e += (long long)blocks * 256) {
        const SgdElem x = sgd_elem(grp, e);
        const SgdLayer &L = grp.l[x.q];
        const long long f = L.flat_begin + x.le;
        const Scale sc = s_scale[L.tensor0 + (x.i < L.in ? 0 : 1)];
        const float g = grp.grads[f];
        const float gp = grp.err ? g + grp.err[f] : g;
        const int c = int8_code_fresh(gp, sc); // the scale comes from the maximum of these very values
        if (grp.codes) grp.codes[f] = (int8_t)c;
        const float deq = sc.s * (float)c;
        if (grp.err) grp.err[f] = gp - deq;
        const float step = grp.lr * deq;
        float *p = x.i < L.in ? L.W + (long long)x.o * L.in + x.i : L.b + x.o;
        *p = *p - step;
    }
}

// ---- channel-wise fake quantisation of the linear layers' weights (model-quantisation appendix) ------
// One scale per output row: s_o = max(max_i |W[o][i]| / qmax, 1e-8), Wq[o][i] = s_o * clamp(rint(W[o][i] / s_o)).
// One wave per row, all layers in one launch.
struct FqLayer {
    const float *W;
    float *Wq;
    int out, in, row_begin;
};
struct FqGroup {
    FqLayer l[kGemmMaxGroup];
    int count, total_rows;
    float qmax; // 7 or 127; the lowest code is -qmax - 1
};

__global__ __launch_bounds__(256) void mlp_fake_quant_kernel(FqGroup grp)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int row = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (256 / kWave) + threadIdx.x / kWave));
    if (row >= grp.total_rows) return;
    int q = 0;
#pragma unroll 1
    for (int k = 1; k < grp.count; ++k)
        if (row >= grp.l[k].row_begin) q = k;
    const FqLayer &L = grp.l[q];
    const float *w = L.W + (long long)(row - L.row_begin) * L.in;
    float *wq = L.Wq + (long long)(row - L.row_begin) * L.in;
    float m = 0.0f;
    for (int i = lane; i < L.in; i += kWave) m = fmaxf(m, fabsf(w[i]));
    m = wave_max(m);
    const Scale sc(scale_from_absmax(m, grp.qmax));
    for (int i = lane; i < L.in; i += kWave) {
        // a fresh scale: no quotient beyond qmax (1 + 2^-23)
        const int c = code_i<false>(w[i], sc, -grp.qmax - 1.0f, grp.qmax);
        wq[i] = sc.s * (float)c;
    }
}

// ---- pairwise-dot interaction ---------------------------------------------------
// Z[b] = [bottom-MLP output, table 0 .. table T-1], V = T + 1 vectors of width D.
// R[b] = [Z[b][0] (D values), dot(Z[b][i], Z[b][j]) for i = 1..V-1, j = 0..i-1, row-major].
struct InteractArgs {
    const float *bot; // [B][D]
    const float *emb; // [B][T][D]
    float *R;         // [B][D + V(V-1)/2]
    const float *dR;  // backward: gradient w.r.t. R
    float *dbot;      // [B][D]
    float *demb;      // [B][T][D]
    const float *bot_mask; // the bottom MLP's last activation (ReLU mask for dbot), or null
    int B, T, D;
    // The bottom MLP's last layer, when it is small enough to ride along (lin_w != null): the forward kernel computes
    // bot[b] = relu(lin_x[b] * lin_w^T + lin_b) itself (and stores it to lin_y for the backward pass); the backward
    // kernel goes on from dbot to that layer's input gradient, lin_dx[b] = (dbot[b] * lin_w) masked by lin_mask > 0.
    const float *lin_x;    // [B][lin_k] input of that layer
    const float *lin_w;    // [D][lin_k]
    const float *lin_b;    // [D]
    float *lin_y;          // [B][D] its output
    const float *lin_mask; // [B][lin_k] backward: the layer's input if that is a ReLU output, or null
    float *lin_dx;         // [B][lin_k] backward: gradient w.r.t. the pre-activation of the layer before, or null
    int lin_k;
};

constexpr int kInterThreads = 128;
constexpr int kInterMaxV = 64;      // vectors per sample, at most (host)
constexpr int kInterMaxZ = 64 * 64; // V * D floats, at most (host)

// dynamic LDS of the two kernels below (at most ~33 KB: V <= 64, V * D <= 4096)
constexpr int kInterMaxLinK = 1024; // widest input of a bottom layer that rides along (host)
inline size_t interact_lds_bytes(int T, int D, bool backward, int lin_k = 0)
{
    const int V = T + 1;
    return sizeof(float) * ((backward ? (size_t)V * D + (size_t)V * (V | 1) + (size_t)D : (size_t)V * (D + 1)) + (size_t)lin_k);
}

// pair index p -> (i, j), i > j, p = i(i-1)/2 + j
__device__ __forceinline__ void pair_of(int p, int &i, int &j)
{
    i = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)p)) * 0.5f);
    while (i * (i - 1) / 2 > p) --i;
    while ((i + 1) * i / 2 <= p) ++i;
    j = p - i * (i - 1) / 2;
}

__global__ __launch_bounds__(kInterThreads) void interact_fwd_kernel(InteractArgs a)
{
    // rows one float apart from a multiple of the bank count: the lanes of a wave read different rows at the
    // same d, and with a pitch of D = 16 all of them would fall into two banks
    extern __shared__ float inter_lds[]; // V * (D + 1) (+ lin_k) floats (interact_lds_bytes)
    float *z = inter_lds;
    const int b = blockIdx.x, V = a.T + 1, D = a.D, pitch = D + 1;
    if (a.lin_w) {
        // the embeddings travel while the layer is computed: 8 threads per output, each a strided eighth of the sum
        for (int e = D + (int)threadIdx.x; e < V * D; e += kInterThreads) {
            const int i = e / D, d = e - i * D;
            z[i * pitch + d] = a.emb[(long long)b * a.T * D + (e - D)];
        }
        float *xin = inter_lds + V * pitch; // lin_k floats
        const int K = a.lin_k;
        for (int k = threadIdx.x; k < K; k += kInterThreads) xin[k] = a.lin_x[(long long)b * K + k];
        __syncthreads();
        for (int e0 = 0; e0 < D * 8; e0 += kInterThreads) { // (kInterThreads is a multiple of 8: teams stay whole)
            const int e = e0 + (int)threadIdx.x;
            const int d = min(e >> 3, D - 1), part = e & 7;
            const float *w = a.lin_w + (long long)d * K;
            float s = 0.0f;
            for (int k = part; k < K; k += 8) s = __builtin_fmaf(xin[k], w[k], s);
            s += __shfl_xor(s, 1, kWave);
            s += __shfl_xor(s, 2, kWave);
            s += __shfl_xor(s, 4, kWave);
            if (part == 0 && e < D * 8) {
                const float y = fmaxf(s + a.lin_b[d], 0.0f);
                z[d] = y;
                a.lin_y[(long long)b * D + d] = y;
            }
        }
    } else {
        for (int e = threadIdx.x; e < V * D; e += kInterThreads) {
            const int i = e / D, d = e - i * D;
            z[i * pitch + d] = e < D ? a.bot[(long long)b * D + e] : a.emb[(long long)b * a.T * D + (e - D)];
        }
    }
    __syncthreads();
    const int P = V * (V - 1) / 2, W = D + P;
    float *r = a.R + (long long)b * W;
    for (int e = threadIdx.x; e < W; e += kInterThreads) {
        if (e < D) {
            r[e] = z[e];
        } else {
            int i, j;
            pair_of(e - D, i, j);
            const float *zi = z + i * pitch, *zj = z + j * pitch;
            float s = 0.0f;
            for (int d = 0; d < D; ++d) s += zi[d] * zj[d];
            r[e] = s;
        }
    }
}

// dZ[i] = sum over j != i of dP(i, j) * Z[j]  (+ dR[0..D) for i = 0): the pair gradients are spread into a
// symmetric V x V matrix with a zero diagonal first, so that the sum runs over all j without a case distinction
// (terms in the order j = 0 .. V-1).
__global__ __launch_bounds__(kInterThreads) void interact_bwd_kernel(InteractArgs a)
{
    extern __shared__ float inter_lds[]; // V * D + V * (V | 1) + D floats (interact_lds_bytes)
    const int b = blockIdx.x, V = a.T + 1, D = a.D, vp = V | 1; // odd pitch
    float *z = inter_lds, *dpf = inter_lds + V * D, *dzl = dpf + V * vp; // dzl: D floats, the gradient w.r.t. bot
    const int P = V * (V - 1) / 2, W = D + P;
    for (int e = threadIdx.x; e < V * D; e += kInterThreads)
        z[e] = e < D ? a.bot[(long long)b * D + e] : a.emb[(long long)b * a.T * D + (e - D)];
    const float *dr = a.dR + (long long)b * W;
    for (int p = threadIdx.x; p < P; p += kInterThreads) {
        int i, j;
        pair_of(p, i, j);
        const float g = dr[D + p];
        dpf[i * vp + j] = g;
        dpf[j * vp + i] = g;
    }
    for (int i = threadIdx.x; i < V; i += kInterThreads) dpf[i * vp + i] = 0.0f;
    __syncthreads();
    for (int e = threadIdx.x; e < V * D; e += kInterThreads) {
        const int i = e / D, d = e - i * D;
        float s = (i == 0) ? dr[d] : 0.0f;
        const float *row = dpf + i * vp, *col = z + d;
        for (int j = 0; j < V; ++j) s += row[j] * col[j * D];
        if (i == 0) {
            const long long off = (long long)b * D + d;
            if (a.bot_mask) s = a.bot_mask[off] > 0.0f ? s : 0.0f;
            a.dbot[off] = s;
            dzl[d] = s;
        } else {
            a.demb[(long long)b * a.T * D + (e - D)] = s;
        }
    }
    if (a.lin_w && a.lin_dx) { // on to the input gradient of the bottom MLP's last layer
        __syncthreads();
        const int K = a.lin_k;
        for (int k = threadIdx.x; k < K; k += kInterThreads) {
            float s = 0.0f;
            for (int d = 0; d < D; ++d) s = __builtin_fmaf(dzl[d], a.lin_w[(long long)d * K + k], s);
            if (a.lin_mask) s = a.lin_mask[(long long)b * K + k] > 0.0f ? s : 0.0f;
            a.lin_dx[(long long)b * K + k] = s;
        }
    }
}

} // namespace dqrm
