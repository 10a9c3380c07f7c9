// Backward: dedupe (sort by table,row,position) -> segment-sum = the sparse
// "specified sparsity" gradient of Sec. 4.3 / the gradient-quantisation appendix.
//
// Kernel 1 (dedupe_kernel): one 1024-thread workgroup per table sorts the
//   table's lookups in LDS with a stable 8-bit LSD radix sort (keys stay in
//   registers between passes; ranks come from per-wave digit counters and a
//   wave-wide match of equal digits), marks segment heads and chunk heads,
//   and writes table-local segment / chunk lists.  The last workgroup to
//   finish turns the per-table counts into global offsets.
// Kernel 2 (segsum_kernel): one lane group per chunk (<= DQRM_SEG_CHUNK
//   consecutive contributions of one segment) sums its gradient rows left to
//   right.  Segments of one chunk are final at once; for longer segments every
//   chunk stores its partial and the group that arrives last adds the partials
//   in chunk order, so the result does not depend on scheduling.
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

constexpr int kDdThreads = 1024;
constexpr int kDdWaves = kDdThreads / kWave;            // 16
constexpr int kDdMaxRounds = DQRM_MAX_TABLE_LOOKUPS / kDdThreads; // 16 items per thread at most
constexpr int kDdCap = DQRM_MAX_TABLE_LOOKUPS;
constexpr int kSegThreads = 256;

// Views into the caller's workspace (all device pointers).
struct BwdWs {
    unsigned *ticket;          // [1]   workgroups of kernel 1 that have finished
    unsigned *seg_counter;     // [N/32 + 2] chunks of a long segment that have arrived (self-resetting)
    int *table_base;           // [T]   first lookup position of the table
    int *table_nuniq;          // [T]
    int *table_nchunk;         // [T]
    int *table_chunk_offsets;  // [T+1]
    int *bag_of_pos;           // [N]   bag (within its table) of every lookup position
    int *sorted_bag;           // [N]   bag of every sorted lookup
    unsigned *seg_row;         // [N+T+1] table-local: row of segment
    int *seg_start;            // [N+T+1] table-local: first sorted index of segment (+ end sentinel)
    int *chunk_start;          // [N]   table-local: first sorted index of chunk
    int *chunk_seg;            // [N]   table-local: segment of chunk
    float *partial_full;       // [(N/32 + 2) * D] partial of a full chunk of a long segment
    float *partial_last;       // [(N/32 + 2) * D] partial of the last chunk of a long segment
};

// exclusive prefix sum over the 1024 threads of the block; *total = sum of all
__device__ __forceinline__ int block_excl_scan_add(int v, int lane, int wave, int *s_w, int *total)
{
    int incl = wave_incl_scan_add(v, lane);
    __syncthreads(); // s_w may still be read from a previous use
    if (lane == kWave - 1) s_w[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kDdWaves; ++w) {
        int x = s_w[w];
        if (w < wave) base += x;
        tot += x;
    }
    *total = tot;
    return base + incl - v;
}

__global__ __launch_bounds__(kDdThreads) void dedupe_kernel(const int64_t *__restrict__ indices,
                                                            const int64_t *__restrict__ offsets,
                                                            const int64_t *__restrict__ row_offsets, int T, int B,
                                                            int64_t N, BwdWs ws, int32_t *__restrict__ sorted_pos,
                                                            int32_t *__restrict__ seg_offsets,
                                                            int32_t *__restrict__ tuo, int32_t *__restrict__ num_unique,
                                                            float *__restrict__ g_absmax)
{
    __shared__ unsigned skey[kDdCap];             // 64 KB
    __shared__ unsigned short spos[kDdCap];       // 32 KB
    __shared__ unsigned cnt[kDdWaves * 256];      // 16 KB, cnt[wave * 256 + digit]
    __shared__ int s_w[kDdWaves];
    __shared__ int s_w2[kDdWaves];
    __shared__ int s_last;

    const int t = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    const long long rows_ll = row_offsets[t + 1] - row_offsets[t];
    const unsigned rows_t = (unsigned)rows_ll; // host checked: 0 <= rows <= DQRM_MAX_TABLE_ROWS

    // ---- table extent in the lookup list --------------------------------
    long long lo = offsets[(long long)t * B], hi = offsets[(long long)(t + 1) * B];
    bool disabled = false; // a table with unusable extents contributes nothing
    if (lo < 0 || hi > N || lo > hi) {
        if (tid == 0) report(DQRM_ERR_BAD_OFFSETS, t, lo);
        lo = lo < 0 ? 0 : (lo > N ? N : lo);
        disabled = true;
    } else if (hi - lo > kDdCap) {
        if (tid == 0) report(DQRM_ERR_CAPACITY, t, hi - lo);
        disabled = true;
    }
    if (disabled) hi = lo;
    const int n = (int)(hi - lo);
    const int base = (int)lo;

    // ---- phase 0: bag of every lookup position ---------------------------
    if (!disabled) {
        for (int b = tid; b < B; b += kDdThreads) {
            long long s = offsets[(long long)t * B + b], e = offsets[(long long)t * B + b + 1];
            if (s < lo || e > hi || s > e) {
                report(DQRM_ERR_BAD_OFFSETS, t, (long long)t * B + b);
                s = s < lo ? lo : (s > hi ? hi : s);
                e = e < s ? s : (e > hi ? hi : e);
            }
            for (long long p = s; p < e; ++p) ws.bag_of_pos[p] = b;
        }
    }

    // ---- phase 1: keys into registers, wave-striped ----------------------
    const int rounds = (n + kDdThreads - 1) / kDdThreads; // 0..16, same for the whole block
    const int per_wave = rounds * kWave;
    unsigned key[kDdMaxRounds];
    unsigned pos[kDdMaxRounds];
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        key[r] = rows_t; // sentinel: sorts after every valid row
        pos[r] = 0;
        if (r < rounds) {
            const int i = wave * per_wave + r * kWave + lane;
            pos[r] = (unsigned)i;
            if (i < n) {
                long long v = indices[lo + i];
                if (v < 0 || v >= rows_ll)
                    report(DQRM_ERR_INDEX_OUT_OF_RANGE, t, v);
                else
                    key[r] = (unsigned)v;
            }
        }
    }

    // ---- phase 2: stable LSD radix sort, 8 bits per pass -----------------
    const int nbits = 32 - __clz(rows_t | 1u); // bit width of the sentinel (>= 1)
    const int passes = (nbits + 7) / 8;
    for (int p = 0; p < passes; ++p) {
        const int shift = 8 * p;
        for (int k = tid; k < kDdWaves * 256; k += kDdThreads) cnt[k] = 0;
        __syncthreads();
        unsigned lrank[kDdMaxRounds];
#pragma unroll
        for (int r = 0; r < kDdMaxRounds; ++r) {
            lrank[r] = 0;
            if (r < rounds) {
                const unsigned d = (key[r] >> shift) & 255u;
                const unsigned long long peers = match_any8(d);
                const unsigned prev = cnt[wave * 256 + d];
                lrank[r] = prev + (unsigned)__popcll(peers & lt_mask);
                if ((peers & lt_mask) == 0ull) cnt[wave * 256 + d] = prev + (unsigned)__popcll(peers);
            }
        }
        __syncthreads();
        // exclusive scan of the counters in (digit, wave) order: thread k owns
        // digit k/4, waves 4*(k%4) .. 4*(k%4)+3
        {
            const int d = tid >> 2, w0 = (tid & 3) * 4;
            unsigned c0 = cnt[(w0 + 0) * 256 + d], c1 = cnt[(w0 + 1) * 256 + d], c2 = cnt[(w0 + 2) * 256 + d],
                     c3 = cnt[(w0 + 3) * 256 + d];
            int total;
            int ex = block_excl_scan_add((int)(c0 + c1 + c2 + c3), lane, wave, s_w, &total);
            cnt[(w0 + 0) * 256 + d] = (unsigned)ex;
            cnt[(w0 + 1) * 256 + d] = (unsigned)ex + c0;
            cnt[(w0 + 2) * 256 + d] = (unsigned)ex + c0 + c1;
            cnt[(w0 + 3) * 256 + d] = (unsigned)ex + c0 + c1 + c2;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kDdMaxRounds; ++r) {
            if (r < rounds) {
                const unsigned d = (key[r] >> shift) & 255u;
                const unsigned rank = cnt[wave * 256 + d] + lrank[r];
                skey[rank] = key[r];
                spos[rank] = (unsigned short)pos[r];
            }
        }
        __syncthreads();
        if (p + 1 < passes) {
#pragma unroll
            for (int r = 0; r < kDdMaxRounds; ++r) {
                if (r < rounds) {
                    const int i = wave * per_wave + r * kWave + lane;
                    key[r] = skey[i];
                    pos[r] = spos[i];
                }
            }
        }
        // the next pass clears cnt and synchronises before anything is overwritten
    }

    // ---- phase 3: segment heads and chunk heads ---------------------------
    // (skey / spos now hold the table's rounds*1024 items in sorted order;
    //  entries that are padding or had a bad index carry the sentinel key.)
    int seg_of[kDdMaxRounds];   // inclusive head count up to the item, minus one
    int start_of[kDdMaxRounds]; // sorted index of the head of the item's segment
    unsigned char flags[kDdMaxRounds];
    int carry_heads = 0, carry_start = -1, carry_valid = 0;
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        seg_of[r] = 0;
        start_of[r] = 0;
        flags[r] = 0;
        if (r < rounds) {
            const int i = wave * per_wave + r * kWave + lane;
            const unsigned k = skey[i];
            const bool valid = k < rows_t;
            const bool head = valid && (i == 0 || skey[i - 1] != k);
            const int h = wave_incl_scan_add(head ? 1 : 0, lane) + carry_heads;
            const int st = max(wave_incl_scan_max(head ? i : -1, lane), carry_start);
            carry_heads = __shfl(h, kWave - 1, kWave);
            carry_start = __shfl(st, kWave - 1, kWave);
            carry_valid += __popcll(__ballot(valid));
            seg_of[r] = h;
            start_of[r] = st;
            flags[r] = (unsigned char)((valid ? 1 : 0) | (head ? 2 : 0));
        }
    }
    // across waves: exclusive head count, running maximum of head positions
    __syncthreads();
    if (lane == 0) {
        s_w[wave] = carry_heads;
        s_w2[wave] = carry_start;
    }
    __syncthreads();
    int heads_before = 0, start_before = -1, n_uniq = 0;
#pragma unroll
    for (int w = 0; w < kDdWaves; ++w) {
        if (w < wave) {
            heads_before += s_w[w];
            start_before = max(start_before, s_w2[w]);
        }
        n_uniq += s_w[w];
    }
    __syncthreads();
    if (lane == 0) s_w[wave] = carry_valid;
    __syncthreads();
    int n_valid = 0;
#pragma unroll
    for (int w = 0; w < kDdWaves; ++w) n_valid += s_w[w];

    // chunk heads: every DQRM_SEG_CHUNK-th item of a segment, counted from its head
    int chunk_of[kDdMaxRounds];
    int carry_chunks = 0;
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        chunk_of[r] = 0;
        if (r < rounds) {
            const int i = wave * per_wave + r * kWave + lane;
            seg_of[r] = seg_of[r] + heads_before - 1;
            start_of[r] = max(start_of[r], start_before);
            const bool valid = flags[r] & 1;
            const bool chead = valid && (((i - start_of[r]) % DQRM_SEG_CHUNK) == 0);
            const int c = wave_incl_scan_add(chead ? 1 : 0, lane) + carry_chunks;
            carry_chunks = __shfl(c, kWave - 1, kWave);
            chunk_of[r] = c;
            if (chead) flags[r] |= 4;
        }
    }
    __syncthreads();
    if (lane == 0) s_w[wave] = carry_chunks;
    __syncthreads();
    int chunks_before = 0, n_chunk = 0;
#pragma unroll
    for (int w = 0; w < kDdWaves; ++w) {
        if (w < wave) chunks_before += s_w[w];
        n_chunk += s_w[w];
    }

    // ---- phase 4: write the table-local lists -------------------------------
    const int sb = base + t; // the table's slice of seg_row / seg_start has n + 1 slots
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        if (r < rounds) {
            const int i = wave * per_wave + r * kWave + lane;
            const int p = spos[i];
            if (i < n) sorted_pos[base + i] = base + p;
            if (flags[r] & 1) {
                int b = ws.bag_of_pos[base + p];
                b = b < 0 ? 0 : (b >= B ? B - 1 : b);
                ws.sorted_bag[base + i] = b;
            }
            if (flags[r] & 2) {
                ws.seg_row[sb + seg_of[r]] = skey[i];
                ws.seg_start[sb + seg_of[r]] = i;
            }
            if (flags[r] & 4) {
                const int c = chunk_of[r] + chunks_before - 1;
                ws.chunk_start[base + c] = i;
                ws.chunk_seg[base + c] = seg_of[r];
            }
        }
    }
    if (tid == 0) {
        ws.seg_start[sb + n_uniq] = n_valid; // end sentinel
        ws.table_base[t] = base;
        ws.table_nuniq[t] = n_uniq;
        ws.table_nchunk[t] = n_chunk;
        g_absmax[t] = 0.0f;
    }

    // ---- phase 5: the last workgroup turns counts into offsets --------------
    __threadfence();
    __syncthreads();
    if (tid == 0) s_last = (atomicAdd(ws.ticket, 1u) == (unsigned)(T - 1)) ? 1 : 0;
    __syncthreads();
    if (s_last) {
        __threadfence();
        int u = 0, c = 0;
        if (tid < T) {
            u = __hip_atomic_load(ws.table_nuniq + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c = __hip_atomic_load(ws.table_nchunk + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        int tot_u, tot_c;
        const int eu = block_excl_scan_add(u, lane, wave, s_w, &tot_u);
        const int ec = block_excl_scan_add(c, lane, wave, s_w2, &tot_c);
        if (tid < T) {
            tuo[tid] = eu;
            ws.table_chunk_offsets[tid] = ec;
        }
        if (tid == 0) {
            tuo[T] = tot_u;
            ws.table_chunk_offsets[T] = tot_c;
            *num_unique = tot_u;
            seg_offsets[tot_u] = (int32_t)N;
            *ws.ticket = 0u;
        }
    }
}

// ---------------------------------------------------------------------------

struct SegArgs {
    const float *grad_out;
    BwdWs ws;
    const int32_t *tuo;
    int64_t *uniq_rows;
    int32_t *seg_offsets;
    float *values;
    float *g_absmax;
    int T, B, D;
};

__device__ __forceinline__ float4 f4_add(float4 a, float4 b)
{
    return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
}

__device__ __forceinline__ float4 load_coherent_f4(const float *p)
{
    float4 v;
    v.x = __hip_atomic_load(p + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.y = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.z = __hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    v.w = __hip_atomic_load(p + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return v;
}

template <int G>
__global__ __launch_bounds__(kSegThreads) void segsum_kernel(SegArgs a)
{
    __shared__ int s_tco[DQRM_MAX_TABLES + 1];
    __shared__ int s_tuo[DQRM_MAX_TABLES + 1];
    __shared__ int s_base[DQRM_MAX_TABLES];
    const int T = a.T, D = a.D;
    for (int k = threadIdx.x; k <= T; k += kSegThreads) {
        s_tco[k] = a.ws.table_chunk_offsets[k];
        s_tuo[k] = a.tuo[k];
        if (k < T) s_base[k] = a.ws.table_base[k];
    }
    __syncthreads();

    const int lg = threadIdx.x & (G - 1);
    const int grp = threadIdx.x / G;
    constexpr int kGroups = kSegThreads / G;
    const int col = lg * 4;
    const bool col_ok = col < D;
    const int C = s_tco[T];
    const int per_block = (C + (int)gridDim.x - 1) / (int)gridDim.x;
    const int c_begin = (int)blockIdx.x * per_block;
    const int c_end = min(C, c_begin + per_block);

    int cur_t = -1;
    float cur_max = 0.0f;

    for (int c = c_begin + grp; c < c_end; c += kGroups) {
        const int t = table_of(s_tco, T, c);
        const int base = s_base[t];
        const int sb = base + t;
        const int lc = c - s_tco[t];
        const int start = a.ws.chunk_start[base + lc];
        const int seg = a.ws.chunk_seg[base + lc];
        const int s0 = a.ws.seg_start[sb + seg];
        const int s1 = a.ws.seg_start[sb + seg + 1];
        int len = s1 - start;
        len = len > DQRM_SEG_CHUNK ? DQRM_SEG_CHUNK : len;
        const int nchunks = (s1 - s0 + DQRM_SEG_CHUNK - 1) / DQRM_SEG_CHUNK;
        const int kchunk = (start - s0) / DQRM_SEG_CHUNK;
        const int *bags = a.ws.sorted_bag + base + start;
        const int64_t tD = (int64_t)T * D;
        const float *g0 = a.grad_out + (int64_t)t * D + col;

        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col_ok && len > 0) {
            acc = *reinterpret_cast<const float4 *>(g0 + (int64_t)bags[0] * tD);
#pragma unroll 4
            for (int i = 1; i < len; ++i) {
                float4 g = *reinterpret_cast<const float4 *>(g0 + (int64_t)bags[i] * tD);
                acc = f4_add(acc, g);
            }
        }

        const int j = s_tuo[t] + seg; // global segment
        bool final_here = true;
        if (nchunks > 1) {
            // long segment: publish this chunk's partial, the last arrival combines
            const int gpos = base + s0; // global sorted position of the segment's head
            const int slot_seg = gpos / DQRM_SEG_CHUNK;
            const bool is_last_chunk = (kchunk == nchunks - 1);
            float *pslot = is_last_chunk ? a.ws.partial_last + (int64_t)slot_seg * D
                                         : a.ws.partial_full + (int64_t)((base + start) / DQRM_SEG_CHUNK) * D;
            if (col_ok) *reinterpret_cast<float4 *>(pslot + col) = acc;
            __threadfence();
            unsigned arrived = 0;
            if (lg == 0) arrived = atomicAdd(a.ws.seg_counter + slot_seg, 1u);
            arrived = __shfl(arrived, (threadIdx.x & (kWave - 1)) & ~(G - 1), kWave);
            final_here = (arrived == (unsigned)(nchunks - 1));
            if (final_here) {
                __threadfence();
                if (col_ok) {
                    for (int k = 0; k < nchunks; ++k) {
                        const float *ps = (k == nchunks - 1)
                                              ? a.ws.partial_last + (int64_t)slot_seg * D
                                              : a.ws.partial_full + (int64_t)((gpos + k * DQRM_SEG_CHUNK) / DQRM_SEG_CHUNK) * D;
                        float4 pv = load_coherent_f4(ps + col);
                        acc = (k == 0) ? pv : f4_add(acc, pv);
                    }
                }
                if (lg == 0) a.ws.seg_counter[slot_seg] = 0u; // ready for the next call
            }
        }
        if (final_here) {
            if (col_ok) *reinterpret_cast<float4 *>(a.values + (int64_t)j * D + col) = acc;
            if (lg == 0) {
                a.uniq_rows[j] = (int64_t)a.ws.seg_row[sb + seg];
                a.seg_offsets[j] = base + s0;
            }
            float m = fmaxf(fmaxf(fabsf(acc.x), fabsf(acc.y)), fmaxf(fabsf(acc.z), fabsf(acc.w)));
            if (t != cur_t) {
                if (cur_t >= 0 && cur_max > 0.0f) atomic_max_nonneg(a.g_absmax + cur_t, cur_max);
                cur_t = t;
                cur_max = 0.0f;
            }
            cur_max = fmaxf(cur_max, m);
        }
    }

    // flush the running maxima: one atomic per wave when the wave saw one table
    const int tt = wave_max_int(cur_t);
    if (__all(cur_t < 0 || cur_t == tt)) {
        const float m = wave_max(cur_max);
        if ((threadIdx.x & (kWave - 1)) == 0 && tt >= 0 && m > 0.0f) atomic_max_nonneg(a.g_absmax + tt, m);
    } else if (cur_t >= 0 && cur_max > 0.0f) {
        atomic_max_nonneg(a.g_absmax + cur_t, cur_max);
    }
}

} // namespace dqrm
