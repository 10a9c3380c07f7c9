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
// Workgroup = 4 waves, each owns a 32x32 block of a 64x64 tile of C and feeds
// v_mfma_f32_32x32x2_f32 from LDS.  The reduction runs in slabs of 64: while the
// matrix cores work on one slab, the next one is already on its way from HBM
// into registers (these products are small -- a few hundred workgroups -- so
// latency, not bandwidth, is what has to be hidden).  With gridDim.z > 1 the
// reduction is split: slice z covers r in [z*k_per_split, ...) and stores its raw
// partial tile to P[z][M][N]; a second kernel adds the slices in order.
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
    int k_per_split;   // reduction length per z slice (multiple of kGemmBK), K if not split
    float *P;          // [gridDim.z][M][N] partial tiles when split
};

constexpr int kGemmThreads = 256;
constexpr int kGemmBM = 64, kGemmBN = 64, kGemmBK = 32;
constexpr int kGemmLd = kGemmBM + 1;                             // LDS row pitch (floats)
constexpr int kGemmPerThread = kGemmBM * kGemmBK / kGemmThreads; // 8 elements of each operand per slab

// A thread's q-th element (q = 0..7) of a 64 (i or j) x 32 (r) operand slab.  CONTIG
// says whether the 64-wide index is the one that is contiguous in memory; either
// way consecutive threads walk along the contiguous direction, four elements each.
template <bool WIDE_CONTIG>
__device__ __forceinline__ void gemm_slot(int tid, int q, int *wide, int *r)
{
    if (WIDE_CONTIG) {
        *wide = (tid & 15) * 4 + (q & 3);
        *r = (tid >> 4) + 16 * (q >> 2);
    } else {
        *r = (tid & 7) * 4 + (q & 3);
        *wide = (tid >> 3) + 32 * (q >> 2);
    }
}

template <bool A_I_CONTIG, bool B_J_CONTIG>
__global__ __launch_bounds__(kGemmThreads) void gemm_mfma_kernel(GemmArgs g)
{
    __shared__ float As[kGemmBK][kGemmLd]; // As[r][i]
    __shared__ float Bs[kGemmBK][kGemmLd]; // Bs[r][j]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i0 = blockIdx.y * kGemmBM, j0 = blockIdx.x * kGemmBN;
    const int r_begin = blockIdx.z * g.k_per_split;
    const int r_end = min(g.K, r_begin + g.k_per_split);

    // per-thread element offsets of the first slab (the host checks that every matrix has < 2^31 elements)
    int off_a[kGemmPerThread], off_b[kGemmPerThread];
    unsigned ok_a = 0, ok_b = 0, ones_b = 0;
#pragma unroll
    for (int q = 0; q < kGemmPerThread; ++q) {
        int ai, ar, bj, br;
        gemm_slot<A_I_CONTIG>(tid, q, &ai, &ar);
        gemm_slot<B_J_CONTIG>(tid, q, &bj, &br);
        off_a[q] = (int)((long long)(i0 + ai) * g.a_si + (long long)(r_begin + ar) * g.a_sr);
        off_b[q] = (int)((long long)(r_begin + br) * g.b_sr + (long long)(j0 + bj) * g.b_sj);
        if (i0 + ai < g.M) ok_a |= 1u << q;
        if (j0 + bj < g.N) ok_b |= 1u << q;
        if (g.b_ones_last && j0 + bj == g.N - 1) ones_b |= 1u << q;
    }
    const int step_a = (int)(kGemmBK * g.a_sr), step_b = (int)(kGemmBK * g.b_sr);

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    float av[kGemmPerThread], bv[kGemmPerThread];
    auto load_slab = [&](int r0) {
#pragma unroll
        for (int q = 0; q < kGemmPerThread; ++q) {
            int ai, ar, bj, br;
            gemm_slot<A_I_CONTIG>(tid, q, &ai, &ar);
            gemm_slot<B_J_CONTIG>(tid, q, &bj, &br);
            const bool in_a = ((ok_a >> q) & 1u) && (r0 + ar < r_end);
            const bool in_b = ((ok_b >> q) & 1u) && (r0 + br < r_end);
            av[q] = in_a ? g.A[off_a[q]] : 0.0f;
            bv[q] = in_b ? (((ones_b >> q) & 1u) ? 1.0f : g.B[off_b[q]]) : 0.0f;
            off_a[q] += step_a;
            off_b[q] += step_b;
        }
    };
    if (r_begin < r_end) load_slab(r_begin);
    for (int r0 = r_begin; r0 < r_end; r0 += kGemmBK) {
        // registers -> LDS
#pragma unroll
        for (int q = 0; q < kGemmPerThread; ++q) {
            int ai, ar, bj, br;
            gemm_slot<A_I_CONTIG>(tid, q, &ai, &ar);
            gemm_slot<B_J_CONTIG>(tid, q, &bj, &br);
            As[ar][ai] = av[q];
            Bs[br][bj] = bv[q];
        }
        __syncthreads();
        // next slab: on its way while the matrix cores run
        if (r0 + kGemmBK < r_end) load_slab(r0 + kGemmBK);
        // one 32x32x2 product per step: lane l feeds A(i = l % 32, r = l / 32) and B(r = l / 32, j = l % 32)
#pragma unroll
        for (int rr = 0; rr < kGemmBK; rr += 2) {
            const float a = As[rr + (lane >> 5)][wm * 32 + (lane & 31)];
            const float b = Bs[rr + (lane >> 5)][wn * 32 + (lane & 31)];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        __syncthreads();
    }

    // accumulator layout: lane l holds column j = l % 32 and rows 8*(v/4) + 4*(l/32) + v%4, v = 0..15
    const int j = j0 + wn * 32 + (lane & 31);
    if (j >= g.N) return;
    if (gridDim.z > 1) {
        float *p = g.P + (long long)blockIdx.z * g.M * g.N;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = i0 + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
            if (i < g.M) p[(long long)i * g.N + j] = acc[v];
        }
        return;
    }
    const float bj = g.bias ? g.bias[j] : 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = i0 + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (i >= g.M) continue;
        float x = acc[v] + bj;
        if (g.relu) x = fmaxf(x, 0.0f);
        const long long off = (long long)i * g.c_si + (long long)j * g.c_sj;
        if (g.mask) x = g.mask[off] > 0.0f ? x : 0.0f;
        g.C[off] = x;
    }
}

// SGD step from the split products of [dZ^T * X | dZ^T * 1]: P is [S][out][in + 1];
// W[o][i] -= lr * sum_s P[s][o][i],  b[o] -= lr * sum_s P[s][o][in]  (slices added in order)
__global__ __launch_bounds__(256) void sgd_from_partials_kernel(const float *__restrict__ P, int S, int out, int in,
                                                                float lr, float *__restrict__ W, float *__restrict__ b)
{
    const long long total = (long long)out * (in + 1);
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        float s = 0.0f;
        for (int z = 0; z < S; ++z) s += P[(long long)z * total + e];
        const int o = (int)(e / (in + 1)), i = (int)(e - (long long)o * (in + 1));
        if (i < in)
            W[(long long)o * in + i] = W[(long long)o * in + i] - lr * s;
        else
            b[o] = b[o] - lr * s;
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
};

constexpr int kInterThreads = 128;
constexpr int kInterMaxZ = 64 * 64; // V * D floats held in LDS

__global__ __launch_bounds__(kInterThreads) void interact_fwd_kernel(InteractArgs a)
{
    __shared__ float z[kInterMaxZ];
    const int b = blockIdx.x, V = a.T + 1, D = a.D;
    for (int e = threadIdx.x; e < V * D; e += kInterThreads)
        z[e] = e < D ? a.bot[(long long)b * D + e] : a.emb[(long long)b * a.T * D + (e - D)];
    __syncthreads();
    const int P = V * (V - 1) / 2, W = D + P;
    float *r = a.R + (long long)b * W;
    for (int e = threadIdx.x; e < W; e += kInterThreads) {
        if (e < D) {
            r[e] = z[e];
        } else {
            // pair index p -> (i, j), i > j: i = largest with i(i-1)/2 <= p
            const int p = e - D;
            int i = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)p)) * 0.5f);
            while (i * (i - 1) / 2 > p) --i;
            while ((i + 1) * i / 2 <= p) ++i;
            const int j = p - i * (i - 1) / 2;
            float s = 0.0f;
            for (int d = 0; d < D; ++d) s += z[i * D + d] * z[j * D + d];
            r[e] = s;
        }
    }
}

__global__ __launch_bounds__(kInterThreads) void interact_bwd_kernel(InteractArgs a)
{
    __shared__ float z[kInterMaxZ];
    __shared__ float dp[64 * 63 / 2];
    const int b = blockIdx.x, V = a.T + 1, D = a.D;
    const int P = V * (V - 1) / 2, W = D + P;
    for (int e = threadIdx.x; e < V * D; e += kInterThreads)
        z[e] = e < D ? a.bot[(long long)b * D + e] : a.emb[(long long)b * a.T * D + (e - D)];
    const float *dr = a.dR + (long long)b * W;
    for (int e = threadIdx.x; e < P; e += kInterThreads) dp[e] = dr[D + e];
    __syncthreads();
    for (int e = threadIdx.x; e < V * D; e += kInterThreads) {
        const int i = e / D, d = e - i * D;
        float s = (i == 0) ? dr[d] : 0.0f;
        for (int j = 0; j < V; ++j) {
            if (j == i) continue;
            const int p = j < i ? i * (i - 1) / 2 + j : j * (j - 1) / 2 + i;
            s += dp[p] * z[j * D + d];
        }
        if (i == 0) {
            const long long off = (long long)b * D + d;
            if (a.bot_mask) s = a.bot_mask[off] > 0.0f ? s : 0.0f;
            a.dbot[off] = s;
        } else {
            a.demb[(long long)b * a.T * D + (e - D)] = s;
        }
    }
}

// ---- sigmoid + mean binary cross-entropy -------------------------------------------
// p = 1 / (1 + exp(-z)); loss = -mean(y log max(p, 1e-12) + (1-y) log max(1-p, 1e-12));
// dz = (p - y) / B.  One block; B is a few thousand.
__global__ __launch_bounds__(256) void bce_kernel(const float *__restrict__ z, const float *__restrict__ y, int B,
                                                  float *__restrict__ dz, float *__restrict__ loss)
{
    __shared__ float part[256];
    float s = 0.0f;
    for (int b = threadIdx.x; b < B; b += 256) {
        const float p = 1.0f / (1.0f + expf(-z[b]));
        const float yy = y[b];
        s += -(yy * logf(fmaxf(p, 1e-12f)) + (1.0f - yy) * logf(fmaxf(1.0f - p, 1e-12f)));
        dz[b] = (p - yy) / (float)B;
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = part[0] / (float)B;
}

} // namespace dqrm
