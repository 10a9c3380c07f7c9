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
    int update;        // 0: C = acc';  1: C = C + alpha * acc' (in place, e.g. W -= lr * dW)
    float alpha;
    int a_i_contig;    // which index of A is contiguous in memory (only steers the load pattern)
    int b_j_contig;
};

constexpr int kGemmThreads = 256;
constexpr int kGemmBM = 64, kGemmBN = 64, kGemmBK = 16;
constexpr int kGemmLd = kGemmBM + 4; // LDS row pitch (floats)

__global__ __launch_bounds__(kGemmThreads) void gemm_mfma_kernel(GemmArgs g)
{
    __shared__ float As[kGemmBK][kGemmLd]; // As[r][i]
    __shared__ float Bs[kGemmBK][kGemmLd]; // Bs[r][j]
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int i0 = blockIdx.y * kGemmBM, j0 = blockIdx.x * kGemmBN;

    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    for (int r0 = 0; r0 < g.K; r0 += kGemmBK) {
        // global -> LDS, 4 elements of each operand per thread, zero-filled outside the matrices
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + q * kGemmThreads; // 0..1023
            int ai, ar, bj, br;
            if (g.a_i_contig) {
                ai = e & 63;
                ar = e >> 6;
            } else {
                ar = e & 15;
                ai = e >> 4;
            }
            if (g.b_j_contig) {
                bj = e & 63;
                br = e >> 6;
            } else {
                br = e & 15;
                bj = e >> 4;
            }
            float av = 0.0f, bv = 0.0f;
            if (i0 + ai < g.M && r0 + ar < g.K) av = g.A[(long long)(i0 + ai) * g.a_si + (long long)(r0 + ar) * g.a_sr];
            if (j0 + bj < g.N && r0 + br < g.K) bv = g.B[(long long)(r0 + br) * g.b_sr + (long long)(j0 + bj) * g.b_sj];
            As[ar][ai] = av;
            Bs[br][bj] = bv;
        }
        __syncthreads();
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
    const float bj = g.bias ? g.bias[j] : 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int i = i0 + wm * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (i >= g.M) continue;
        float x = acc[v] + bj;
        if (g.relu) x = fmaxf(x, 0.0f);
        const long long off = (long long)i * g.c_si + (long long)j * g.c_sj;
        if (g.mask) x = g.mask[off] > 0.0f ? x : 0.0f;
        if (g.update)
            g.C[off] = g.C[off] + g.alpha * x;
        else
            g.C[off] = x;
    }
}

// b[n] += alpha * sum_m dZ[m][n]   (bias gradient + SGD step); one block per 64 columns
__global__ __launch_bounds__(256) void bias_update_kernel(const float *__restrict__ dZ, int M, int N, float alpha,
                                                          float *__restrict__ b)
{
    __shared__ float part[4][64];
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + c;
    float s = 0.0f;
    if (n < N)
        for (int m = q; m < M; m += 4) s += dZ[(long long)m * N + n];
    part[q][c] = s;
    __syncthreads();
    if (q == 0 && n < N) b[n] = b[n] + alpha * (((part[0][c] + part[1][c]) + part[2][c]) + part[3][c]);
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
