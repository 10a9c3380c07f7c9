// Backward: dedupe (sort by table,row,position) -> segment-sum = the sparse
// "specified sparsity" gradient of Sec. 4.3 / the gradient-quantisation appendix.
//
// Kernel 1 (dedupe_kernel): one 1024-thread workgroup per table sorts the
//   table's lookups in LDS with a stable 8-bit LSD radix sort (keys stay in
//   registers between passes; ranks come from per-wave digit counters and a
//   wave-wide match of equal digits), marks segment heads and chunk heads,
//   and writes table-local segment / chunk lists plus the table's counts.
//   A table of more than kDdCap lookups is sorted in tiles by several workgroups;
//   dedupe_merge_kernel merges the sorted tiles and dedupe_large_kernel builds the
//   same lists from the merged order.
// Kernel 2 (dedupe_finish_kernel): turns the per-table counts into offsets (T is
//   small, every workgroup repeats the scan), writes the index-only outputs
//   (unique rows, segment offsets, table offsets, count) and one dense list of
//   16-byte chunk descriptors over all tables.
// Kernels 1-2 need only the batch's indices; they form dqrm_dedupe.
// Kernel 3 (segment_sum_kernel): one lane group per chunk (<= DQRM_SEG_CHUNK
//   consecutive contributions of one segment) adds its gradient rows left to
//   right.  A segment of one chunk is final.  The chunks of a longer segment park
//   their sums and count themselves in on the segment's counter; the wave of the
//   chunk that arrives last adds the segment's chunk sums in chunk order.  Which
//   wave that is depends on scheduling; what it computes does not.
// Kernel 4 (absmax_finalize_kernel): folds the per-table maxima.
// segment_sum_multi_kernel / absmax_finalize_multi_kernel: kernels 3 and 4 for several batches in one launch.
#pragma once

#include "dqrm_device.hpp"

namespace dqrm {

constexpr int kDdThreads = 1024;
constexpr int kDdWaves = kDdThreads / kWave;                      // 16
constexpr int kDdCap = 16384;                     // lookups one workgroup sorts in LDS
constexpr int kDdMaxRounds = kDdCap / kDdThreads; // 16 items per thread at most
static_assert(DQRM_MAX_TABLE_LOOKUPS % kDdCap == 0 && DQRM_MAX_TABLE_LOOKUPS / DQRM_SEG_CHUNK < 4096,
              "tiles of the large-table path; the chunk descriptor holds 12 bits of chunk count");
constexpr int kSegThreads = 256;   // dedupe_finish_kernel
constexpr int kSumThreads = 256;   // segment_sum_kernel
constexpr int kSegBatch = 16;      // gradient rows requested before the first is added
constexpr int kSumBlocksPerCu = 4; // grid of segment_sum_kernel, in workgroups per CU (128 registers per lane)

// Views into the caller's workspace (all device pointers).
struct BwdWs {
    int *table_base;          // [T]   first lookup position of the table
    int *table_nuniq;         // [T]
    int *table_nchunk;        // [T]   chunks other than singles
    int *table_nsingle;       // [T]   rows looked up exactly once
    int *bag_of_pos;          // [N]   bag (within its table) of every lookup position
    int *sorted_bag;          // [N]   bag of every sorted lookup
    int4 *chunk_local;        // [N]   table-local chunk lists (table t's start at its first lookup position)
    int4 *single_local;       // [N]   table-local lists of singles: {sorted position, bag, segment, row}
    int4 *chunk_desc;         // [N]   dense chunk list over all tables, as the summing kernels read it
    int *chunk_bags;          // [N/2 + 1][32] bags of chunk c's lookups, so that they can be read before its descriptor
    int4 *single_desc;        // [N]   dense list of singles: {bag, global segment, table, -}
    int *totals;              // [3]   chunks, segments, singles
    // tables with more than kDdCap lookups (present only if N > kDdCap): the sorted tiles, then, in the same two
    // arrays, segment index and segment start of every merged position; the merged order; the segments' heads
    unsigned *run_key;        // [N]   / int seg_idx[N]
    int *run_pos;             // [N]   / int seg_start[N]
    unsigned *merged_key;     // [N]
    int *merged_pos;          // [N]   position inside the table of every merged item
    int *head_of_seg;         // [N + T + 1] sorted index of each segment's head; table t's list starts at (first lookup position + t)
    int *seg_count;           // [N/32 + 2] chunks of a segment of more than one chunk that have parked their sum, filed
                              //       under (sorted position of the segment's head / 32); zero between uses
    float *partial_full;      // [(N/32 + 2) * D] sum of a full chunk of a segment of more than one chunk
    float *partial_last;      // [(N/32 + 2) * D] sum of the last chunk of such a segment
    float *absmax_slots;      // [T][kAbsmaxSlots] running maxima, one 128-byte line per entry
};

// A chunk = up to DQRM_SEG_CHUNK consecutive sorted lookups of one segment.  Its
// descriptor is one 16-byte record, so that the summing kernels need a single
// load to know their work:
//   x  global sorted position of the chunk's first lookup
//   y  len (bits 0..7) | index of the chunk inside its segment (bits 8..19) |
//      chunks in the segment (bits 20..31)
//   z  table-local index of the segment
//   w  table-local row of the segment
__device__ __forceinline__ int4 make_chunk_desc(int gstart, int len, int kchunk, int nchunks, int seg, unsigned row)
{
    return make_int4(gstart, len | (kchunk << 8) | (nchunks << 20), seg, (int)row);
}
__device__ __forceinline__ int desc_len(const int4 &d) { return d.y & 0xFF; }
__device__ __forceinline__ int desc_kchunk(const int4 &d) { return (d.y >> 8) & 0xFFF; }
__device__ __forceinline__ int desc_nchunks(const int4 &d) { return (int)((unsigned)d.y >> 20); }

// One launch can dedupe several batches (blockIdx.y picks the batch): the work
// depends only on the indices, and a table's sort occupies a single CU, so the
// batches of the next few steps fill the chip where one batch would use T CUs.
struct DedupeBatch {
    const int64_t *indices;
    const int64_t *offsets;
    int64_t N;
    int limit; // lookups a table may have: DQRM_MAX_TABLE_LOOKUPS or the caller's smaller bound
    BwdWs ws;
    int32_t *sorted_pos;
    int32_t *tuo;
    int32_t *num_unique;
    int64_t *uniq_rows;
    int32_t *seg_offsets;
};
struct DedupeArgs {
    DedupeBatch b[DQRM_MAX_DEDUPE_BATCHES];
    const int64_t *row_offsets;
    int T, B;
};

__global__ __launch_bounds__(kDdThreads) void dedupe_kernel(DedupeArgs args)
{
    const DedupeBatch &bt = args.b[blockIdx.y];
    const int64_t *__restrict__ indices = bt.indices;
    const int64_t *__restrict__ offsets = bt.offsets;
    const int64_t *__restrict__ row_offsets = args.row_offsets;
    const int T = args.T, B = args.B;
    const int64_t N = bt.N;
    const BwdWs ws = bt.ws;
    int32_t *__restrict__ sorted_pos = bt.sorted_pos;
    (void)T;

    __shared__ unsigned skey[kDdCap];        // 64 KB
    __shared__ unsigned short spos[kDdCap];  // 32 KB
    __shared__ unsigned cnt[kDdWaves * 256]; // 16 KB, cnt[wave * 256 + digit]
    __shared__ unsigned short shead[kDdCap + 2]; // 32 KB, sorted index of each segment's head (+ end sentinel)
    __shared__ int s_w[kDdWaves];
    __shared__ int s_w2[kDdWaves];

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
        if (tid == 0 && blockIdx.z == 0) report(DQRM_ERR_BAD_OFFSETS, t, lo);
        lo = lo < 0 ? 0 : (lo > N ? N : lo);
        disabled = true;
    } else if (hi - lo > bt.limit) {
        if (tid == 0 && blockIdx.z == 0) report(DQRM_ERR_CAPACITY, t, hi - lo);
        disabled = true;
    }
    if (disabled) hi = lo;
    const int base = (int)lo;
    // A table of up to kDdCap lookups is this workgroup's (blockIdx.z = 0) from start to end.  A larger one is cut
    // into tiles of kDdCap consecutive lookups: workgroup z sorts tile z and leaves the sorted run in the workspace;
    // dedupe_merge_kernel merges the runs and dedupe_large_kernel does the rest.
    const bool large = hi - lo > kDdCap;
    const int tile = (int)blockIdx.z;
    if (!large && tile > 0) return;
    const long long first = lo + (large ? (long long)tile * kDdCap : 0ll); // my first lookup
    if (large && first >= hi) return;
    const int n = (int)(large ? (hi - first < kDdCap ? hi - first : (long long)kDdCap) : hi - lo);
    const bool does_bags = !disabled && (!large || tile == 0);

    // ---- phase 0: bag of every lookup position ---------------------------
    // The table's keys are requested first (wave-striped: item i = wave * per_wave + r * 64 + lane), so that they
    // travel while the bags are looked at; items past the end re-read the last key and are dropped in phase 1.
    const int rounds = (n + kDdThreads - 1) / kDdThreads; // 0..16, same for the whole block
    const int per_wave = rounds * kWave;
    long long raw[kDdMaxRounds];
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        raw[r] = 0;
        if (r < rounds) raw[r] = indices[first + min(wave * per_wave + r * kWave + lane, n - 1)]; // (n >= 1 here)
    }
    // When every bag of the table holds exactly one lookup (the usual DLRM
    // batch) the bag of position p is p itself and nothing needs to be stored.
    constexpr int kBagBatch = 8;
    bool one_each = !disabled && !large && (n == B);
    if (does_bags) {
        for (int b0 = 0; b0 < B; b0 += kDdThreads * kBagBatch) {
            long long s[kBagBatch], e[kBagBatch];
#pragma unroll
            for (int q = 0; q < kBagBatch; ++q) {
                const int b = b0 + q * kDdThreads + tid;
                s[q] = lo + b;
                e[q] = s[q] + 1;
                if (b < B) {
                    s[q] = offsets[(long long)t * B + b];
                    e[q] = offsets[(long long)t * B + b + 1];
                }
            }
#pragma unroll
            for (int q = 0; q < kBagBatch; ++q) {
                const int b = b0 + q * kDdThreads + tid;
                if (b < B && (s[q] < lo || e[q] > hi || s[q] > e[q]))
                    report(DQRM_ERR_BAD_OFFSETS, t, (long long)t * B + b);
                if (s[q] != lo + b || e[q] != s[q] + 1) one_each = false;
            }
        }
    }
    one_each = __syncthreads_and(one_each ? 1 : 0) != 0;
    if (does_bags && !one_each) {
        for (int b = tid; b < B; b += kDdThreads) {
            long long s = offsets[(long long)t * B + b], e = offsets[(long long)t * B + b + 1];
            s = s < lo ? lo : (s > hi ? hi : s);
            e = e < s ? s : (e > hi ? hi : e);
            for (long long p = s; p < e; ++p) ws.bag_of_pos[p] = b;
        }
    }

    // ---- phase 1: keys checked and narrowed ------------------------------
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
                const long long v = raw[r];
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
        // (the rank inside the wave's digit group rides in the upper half of pos[]:
        //  both are below 16384)
#pragma unroll
        for (int r = 0; r < kDdMaxRounds; ++r) {
            if (r < rounds) {
                const unsigned d = (key[r] >> shift) & 255u;
                const unsigned long long peers = match_any8(d);
                const unsigned prev = cnt[wave * 256 + d];
                pos[r] |= (prev + (unsigned)__popcll(peers & lt_mask)) << 16;
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
            int ex = block_excl_scan_add<kDdWaves>((int)(c0 + c1 + c2 + c3), lane, wave, s_w, &total);
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
                const unsigned rank = cnt[wave * 256 + d] + (pos[r] >> 16);
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
    if (large) { // the sorted run of this tile; positions counted from the table's first lookup
        for (int i = tid; i < n; i += kDdThreads) {
            ws.run_key[first + i] = skey[i];
            ws.run_pos[first + i] = tile * kDdCap + (int)spos[i];
        }
        return;
    }

    // ---- phase 3: segment heads and chunk heads ---------------------------
    // (skey / spos now hold the table's rounds*1024 items in sorted order;
    //  entries that are padding or had a bad index carry the sentinel key.)
    // Per item, packed into one word to keep the register count down:
    //   bits 0..14  segment index + 1      bits 15..29  sorted index of the segment's head + 1
    //   bit  30     valid                  bit  31      head of its segment
    unsigned info[kDdMaxRounds];
    auto info_seg = [](unsigned w) { return (int)(w & 0x7FFFu) - 1; };
    auto info_start = [](unsigned w) { return (int)((w >> 15) & 0x7FFFu) - 1; };
    auto info_valid = [](unsigned w) { return (w >> 30) & 1u; };
    auto info_head = [](unsigned w) { return w >> 31; };
    int carry_heads = 0, carry_start = -1, carry_valid = 0;
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        info[r] = 0;
    }
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        if (r < rounds) {
            const int i = wave * per_wave + r * kWave + lane;
            const unsigned k = skey[i];
            const bool valid = k < rows_t;
            const bool head = valid && (i == 0 || skey[i - 1] != k);
            const int h = wave_incl_scan_add(head ? 1 : 0, lane) + carry_heads; // heads up to here, this wave
            const int st = max(wave_incl_scan_max(head ? i : -1, lane), carry_start);
            carry_heads = wave_last(h);
            carry_start = wave_last(st);
            carry_valid += __popcll(__ballot(valid));
            info[r] = (unsigned)h | ((unsigned)(st + 1) << 15) | (valid ? 1u << 30 : 0u) | (head ? 1u << 31 : 0u);
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

    // segment heads leave their sorted index in LDS, so that every item can find
    // the end of its segment
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        if (r < rounds) {
            const int i = wave * per_wave + r * kWave + lane;
            const int seg = (int)(info[r] & 0x7FFFu) + heads_before - 1;     // -1 .. 16383
            const int start = max(info_start(info[r]), start_before);        // -1 .. 16383
            info[r] = (unsigned)(seg + 1) | ((unsigned)(start + 1) << 15) | (info[r] & 0xC0000000u);
            if (info_head(info[r])) shead[seg] = (unsigned short)i;
        }
    }
    if (tid == 0) shead[n_uniq] = (unsigned short)n_valid; // end sentinel (n_valid <= 16384 fits)
    __syncthreads();

    // chunk heads: every DQRM_SEG_CHUNK-th item of a segment, counted from its
    // head.  Two classes, listed separately: "single" = a row looked up exactly
    // once (the common case, no summation needed), and all other chunks.  One
    // scan counts both (bits 0..14: singles, bits 16..30: the others; each <= 16384);
    // bits 15 / 31 of the stored word then mark what the item itself is.
    unsigned chunk_of[kDdMaxRounds];
    int carry_chunks = 0;
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        chunk_of[r] = 0;
        if (r < rounds) {
            const int i = wave * per_wave + r * kWave + lane;
            const bool chead = info_valid(info[r]) && (((i - info_start(info[r])) % DQRM_SEG_CHUNK) == 0);
            const bool single = chead && info_head(info[r]) && ((int)shead[info_seg(info[r]) + 1] == i + 1);
            const int c = wave_incl_scan_add(chead ? (single ? 1 : 0x10000) : 0, lane) + carry_chunks;
            carry_chunks = wave_last(c);
            chunk_of[r] = (unsigned)c | (chead ? (single ? 1u << 15 : 1u << 31) : 0u);
        }
    }
    __syncthreads();
    if (lane == 0) s_w[wave] = carry_chunks;
    __syncthreads();
    int singles_before = 0, chunks_before = 0, n_single = 0, n_chunk = 0;
#pragma unroll
    for (int w = 0; w < kDdWaves; ++w) {
        const int x = s_w[w];
        if (w < wave) {
            singles_before += x & 0x7FFF;
            chunks_before += x >> 16;
        }
        n_single += x & 0x7FFF;
        n_chunk += x >> 16;
    }

    // ---- phase 4: write the table-local lists -------------------------------
    if (!one_each) {
        // bag of every sorted lookup: gathered first, all at once, so that the loads overlap
#pragma unroll
        for (int r = 0; r < kDdMaxRounds; ++r) {
            if (r < rounds) {
                const int i = wave * per_wave + r * kWave + lane;
                if (info_valid(info[r])) {
                    int b = ws.bag_of_pos[base + spos[i]];
                    b = b < 0 ? 0 : (b >= B ? B - 1 : b);
                    ws.sorted_bag[base + i] = b;
                }
            }
        }
        __syncthreads(); // the singles below read their own entry back
    }
#pragma unroll
    for (int r = 0; r < kDdMaxRounds; ++r) {
        if (r < rounds) {
            const int i = wave * per_wave + r * kWave + lane;
            const int p = spos[i];
            if (i < n) sorted_pos[base + i] = base + p;
            if (one_each && info_valid(info[r])) ws.sorted_bag[base + i] = p < B ? p : B - 1;
            const int seg = info_seg(info[r]);
            if (chunk_of[r] & (1u << 31)) { // head of a chunk that is not a single
                const int c = (int)((chunk_of[r] >> 16) & 0x7FFFu) + chunks_before - 1;
                const int s0 = info_start(info[r]), s1 = shead[seg + 1];
                const int len = min(DQRM_SEG_CHUNK, s1 - i);
                const int nchunks = (s1 - s0 + DQRM_SEG_CHUNK - 1) / DQRM_SEG_CHUNK;
                ws.chunk_local[base + c] =
                    make_chunk_desc(base + i, len, (i - s0) / DQRM_SEG_CHUNK, nchunks, seg, skey[i]);
                // the arrival counter of a segment of more than one chunk starts at zero
                if (i == s0 && nchunks > 1) ws.seg_count[(base + i) / DQRM_SEG_CHUNK] = 0;
            }
            if (chunk_of[r] & (1u << 15)) { // a row looked up exactly once
                const int c = (int)(chunk_of[r] & 0x7FFFu) + singles_before - 1;
                const int b = one_each ? (p < B ? p : B - 1) : ws.sorted_bag[base + i];
                ws.single_local[base + c] = make_int4(base + i, b, seg, (int)skey[i]);
            }
        }
    }
    if (tid == 0) {
        ws.table_base[t] = base;
        ws.table_nuniq[t] = n_uniq;
        ws.table_nchunk[t] = n_chunk;
        ws.table_nsingle[t] = n_single;
    }
    if (tid < kAbsmaxSlots) *absmax_slot(ws.absmax_slots, t, tid) = 0.0f;
}

// Step 1 for a table of more than kDdCap lookups, one workgroup per sorted tile (run): every item of the run finds
// its place in the table's sorted order on its own -- its index in its own run plus, per other run, the number of
// that run's keys below it (equal keys of earlier runs count as below, which keeps equal keys in lookup order).
// Each other run in turn is staged in LDS and searched by the run's items, kept in registers, four searches in step
// (a fixed number of halvings, no branch).
__global__ __launch_bounds__(kDdThreads) void dedupe_merge_kernel(DedupeArgs args)
{
    const DedupeBatch &bt = args.b[blockIdx.y];
    const int B = args.B;
    const int64_t N = bt.N;
    const BwdWs ws = bt.ws;
    __shared__ unsigned s_run[kDdCap]; // 64 KB: the run that is being searched
    constexpr int kItems = kDdCap / kDdThreads; // 16 per thread
    const int t = blockIdx.x, r = blockIdx.z, tid = threadIdx.x;
    const long long lo = bt.offsets[(long long)t * B], hi = bt.offsets[(long long)(t + 1) * B];
    if (lo < 0 || hi > N || lo > hi || hi - lo > bt.limit || hi - lo <= kDdCap) return;
    const int n = (int)(hi - lo), base = (int)lo;
    const int runs = (n + kDdCap - 1) / kDdCap;
    if (r >= runs) return;
    const int len = min(kDdCap, n - r * kDdCap); // my run
    unsigned key[kItems];
    int rank[kItems];
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
        const int j = min(q * kDdThreads + tid, len - 1);
        key[q] = ws.run_key[base + r * kDdCap + j];
        rank[q] = j;
    }
    for (int r2 = 0; r2 < runs; ++r2) {
        if (r2 == r) continue; // (block-uniform)
        const int len2 = min(kDdCap, n - r2 * kDdCap);
        const bool ties_below = r2 < r;
        __syncthreads(); // (the searches of the run staged before are over)
        for (int i = tid; i < kDdCap; i += kDdThreads) s_run[i] = i < len2 ? ws.run_key[base + r2 * kDdCap + i] : 0xFFFFFFFFu;
        __syncthreads();
#pragma unroll
        for (int q0 = 0; q0 < kItems; q0 += 4) {
            int below[4] = {0, 0, 0, 0};
#pragma unroll 1
            for (int step = kDdCap; step >= 1; step >>= 1) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int idx = below[q] + step; // are the first idx keys of the run all below mine?
                    const unsigned k2 = s_run[min(idx, kDdCap) - 1];
                    const bool yes = idx <= len2 && (ties_below ? k2 <= key[q0 + q] : k2 < key[q0 + q]);
                    below[q] = yes ? idx : below[q];
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) rank[q0 + q] += below[q];
        }
    }
#pragma unroll
    for (int q = 0; q < kItems; ++q) {
        const int j = q * kDdThreads + tid;
        if (j < len) {
            ws.merged_key[base + rank[q]] = key[q];
            ws.merged_pos[base + rank[q]] = ws.run_pos[base + r * kDdCap + j];
        }
    }
}

// ---------------------------------------------------------------------------
// Tables with more than kDdCap lookups: dedupe_kernel has sorted their tiles of kDdCap consecutive lookups and
// dedupe_merge_kernel (above) has merged the runs; one workgroup per (table, batch) now
//  1. walks the merged order in slabs of one item per thread, carrying the counts from slab to slab: segment
//     heads, segment index and start of every item, the list of the heads;
//  2. walks it again for the chunk heads and singles (a segment's end is the next segment's head, known now) and
//     writes the same table-local lists and counts as dedupe_kernel does for a small table.
// Everything between the steps goes through global memory of the workspace, read back by the same workgroup
// after a barrier.  Slower per lookup than the in-LDS path; it exists so that no table size up to
// DQRM_MAX_TABLE_LOOKUPS is refused.
__global__ __launch_bounds__(kDdThreads) void dedupe_large_kernel(DedupeArgs args)
{
    const DedupeBatch &bt = args.b[blockIdx.y];
    const int64_t *__restrict__ offsets = bt.offsets;
    const int B = args.B;
    const int64_t N = bt.N;
    const BwdWs ws = bt.ws;
    __shared__ int s_w[kDdWaves];
    __shared__ int s_w2[kDdWaves];

    const int t = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const long long rows_ll = args.row_offsets[t + 1] - args.row_offsets[t];
    const unsigned rows_t = (unsigned)rows_ll;
    const long long lo = offsets[(long long)t * B], hi = offsets[(long long)(t + 1) * B];
    // (unusable extents and tables beyond the limit were reported and closed by dedupe_kernel)
    if (lo < 0 || hi > N || lo > hi || hi - lo > bt.limit || hi - lo <= kDdCap) return;
    const int n = (int)(hi - lo), base = (int)lo;
    const int runs = (n + kDdCap - 1) / kDdCap;

    // (the runs are not read again: their arrays now take segment index and start of every item)

    // A slab is kRounds x kDdThreads consecutive items, wave-striped as in dedupe_kernel: wave w owns the slab's items
    // w * kRounds * 64 ..., item (round r, lane l) = that + r * 64 + l.  A wave carries its counts from round to round by
    // itself; the waves meet once per slab.
    // ---- 1. segment heads, index and start of every item
    int *seg_idx = reinterpret_cast<int *>(ws.run_key) + base, *seg_start = ws.run_pos + base;
    int *head_of = ws.head_of_seg + base + t;
    int carry_heads = 0, carry_start = -1, n_valid = 0;
    {
        constexpr int kRounds = 8, kSlab = kRounds * kDdThreads, kPerWave = kRounds * kWave;
        for (int s0 = 0; s0 < n; s0 += kSlab) {
            unsigned k_of[kRounds], prev_of[kRounds];
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int i = s0 + wave * kPerWave + r * kWave + lane;
                k_of[r] = i < n ? ws.merged_key[base + i] : rows_t;
                prev_of[r] = (i > 0 && i < n) ? ws.merged_key[base + i - 1] : 0u;
            }
            int h_of[kRounds], st_of[kRounds];
            int wave_heads = 0, wave_start = -1, wave_valid = 0;
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int i = s0 + wave * kPerWave + r * kWave + lane;
                const bool valid = i < n && k_of[r] < rows_t;
                const bool head = valid && (i == 0 || prev_of[r] != k_of[r]);
                h_of[r] = wave_incl_scan_add(head ? 1 : 0, lane) + wave_heads; // heads up to here, this wave and slab
                st_of[r] = max(wave_incl_scan_max(head ? i : -1, lane), wave_start);
                wave_heads = wave_last(h_of[r]);
                wave_start = wave_last(st_of[r]);
                wave_valid += __popcll(__ballot(valid));
                h_of[r] = head ? h_of[r] : -h_of[r] - 1; // (the sign tells a head; valid or not is read off k_of)
            }
            __syncthreads(); // (s_w / s_w2 of the previous slab have been read)
            if (lane == 0) {
                s_w[wave] = wave_heads | (wave_valid << 16); // both at most 512
                s_w2[wave] = wave_start;
            }
            __syncthreads();
            int heads_before = 0, start_before = -1, heads_slab = 0, valid_slab = 0, start_slab = -1;
#pragma unroll
            for (int w = 0; w < kDdWaves; ++w) {
                const int x = s_w[w];
                if (w < wave) {
                    heads_before += x & 0xFFFF;
                    start_before = max(start_before, s_w2[w]);
                }
                heads_slab += x & 0xFFFF;
                valid_slab += x >> 16;
                start_slab = max(start_slab, s_w2[w]);
            }
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int i = s0 + wave * kPerWave + r * kWave + lane;
                if (i < n) {
                    const bool valid = k_of[r] < rows_t, head = h_of[r] >= 0;
                    const int h = head ? h_of[r] : -h_of[r] - 1;
                    seg_idx[i] = valid ? carry_heads + heads_before + h - 1 : -1;
                    seg_start[i] = max(max(carry_start, start_before), st_of[r]);
                    if (head) head_of[carry_heads + heads_before + h - 1] = i;
                }
            }
            carry_heads += heads_slab;
            carry_start = max(carry_start, start_slab);
            n_valid += valid_slab;
        }
    }
    const int n_uniq = carry_heads;
    if (tid == 0) head_of[n_uniq] = n_valid; // end of the last segment
    __syncthreads();

    // ---- 2. chunk heads and singles, the table-local lists
    int carry_single = 0, carry_chunk = 0;
    {
        constexpr int kRounds = 8, kSlab = kRounds * kDdThreads, kPerWave = kRounds * kWave;
        for (int s0 = 0; s0 < n; s0 += kSlab) {
            int seg_of[kRounds], start_of[kRounds], p_of[kRounds], end_of[kRounds], bag_of[kRounds];
            unsigned key_of[kRounds];
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int i = min(s0 + wave * kPerWave + r * kWave + lane, n - 1);
                seg_of[r] = seg_idx[i];
                start_of[r] = seg_start[i];
                p_of[r] = ws.merged_pos[base + i];
                key_of[r] = ws.merged_key[base + i];
            }
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                if (s0 + wave * kPerWave + r * kWave + lane >= n) seg_of[r] = -1;
                end_of[r] = head_of[max(seg_of[r], 0) + 1]; // (the list's region has that entry even if n_uniq = 0)
                bag_of[r] = ws.bag_of_pos[base + p_of[r]];
            }
            // one scan counts both kinds (bits 0..15: singles, bits 16..31: the other chunk heads; each <= 8192 a slab)
            int c_of[kRounds];
            int wave_count = 0;
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int i = s0 + wave * kPerWave + r * kWave + lane;
                const bool valid = seg_of[r] >= 0;
                const bool chead = valid && ((i - start_of[r]) % DQRM_SEG_CHUNK) == 0;
                const bool single = chead && i == start_of[r] && end_of[r] == i + 1;
                c_of[r] = wave_incl_scan_add(chead ? (single ? 1 : 0x10000) : 0, lane) + wave_count;
                wave_count = wave_last(c_of[r]);
                // what the item itself is rides in p_of's spare bits (a position inside the table is below 2^17)
                p_of[r] |= chead ? (single ? 1 << 30 : 1 << 29) : 0;
            }
            __syncthreads(); // (s_w of the previous slab has been read)
            if (lane == 0) s_w[wave] = wave_count;
            __syncthreads();
            int singles_before = 0, chunks_before = 0, singles_slab = 0, chunks_slab = 0;
#pragma unroll
            for (int w = 0; w < kDdWaves; ++w) {
                const int x = s_w[w];
                if (w < wave) {
                    singles_before += x & 0xFFFF;
                    chunks_before += x >> 16;
                }
                singles_slab += x & 0xFFFF;
                chunks_slab += x >> 16;
            }
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                const int i = s0 + wave * kPerWave + r * kWave + lane;
                if (i >= n) continue;
                const int seg = seg_of[r], start = start_of[r], end = end_of[r], p = p_of[r] & 0x1FFFFFFF;
                const bool is_single = (p_of[r] >> 30) & 1, is_chunk = (p_of[r] >> 29) & 1;
                bt.sorted_pos[base + i] = base + p;
                int b = 0;
                if (seg >= 0) {
                    b = bag_of[r];
                    b = b < 0 ? 0 : (b >= B ? B - 1 : b);
                    ws.sorted_bag[base + i] = b;
                }
                if (is_chunk) {
                    const int c = carry_chunk + chunks_before + (c_of[r] >> 16) - 1;
                    const int nchunks = (end - start + DQRM_SEG_CHUNK - 1) / DQRM_SEG_CHUNK;
                    ws.chunk_local[base + c] = make_chunk_desc(base + i, min(DQRM_SEG_CHUNK, end - i),
                                                               (i - start) / DQRM_SEG_CHUNK, nchunks, seg, key_of[r]);
                    if (i == start && nchunks > 1) ws.seg_count[(base + i) / DQRM_SEG_CHUNK] = 0;
                }
                if (is_single) {
                    const int c = carry_single + singles_before + (c_of[r] & 0xFFFF) - 1;
                    ws.single_local[base + c] = make_int4(base + i, b, seg, (int)key_of[r]);
                }
            }
            carry_single += singles_slab;
            carry_chunk += chunks_slab;
        }
    }
    if (tid == 0) {
        ws.table_base[t] = base;
        ws.table_nuniq[t] = n_uniq;
        ws.table_nchunk[t] = carry_chunk;
        ws.table_nsingle[t] = carry_single;
    }
    if (tid < kAbsmaxSlots) *absmax_slot(ws.absmax_slots, t, tid) = 0.0f;
}

// ---------------------------------------------------------------------------
// Kernel 2 of dqrm_dedupe: table-local lists -> one dense, global chunk list and
// the index-only outputs (unique rows, segment offsets, table offsets, count).

// Turns the per-table counts into offsets in LDS (every block does this; T is
// small).  s_tuo / s_tco / s_tso receive T+1 entries (segments, chunks, singles),
// s_base T.
__device__ __forceinline__ void table_offsets_to_lds(const BwdWs &ws, int T, int *s_tuo, int *s_tco, int *s_tso,
                                                     int *s_base, int *s_w)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    if (T <= kWave) {
        // the usual case: one wave scans the counts, no block-wide scan needed
        if (wave == 0) {
            int u = 0, c = 0, g = 0;
            if (lane < T) {
                u = ws.table_nuniq[lane];
                c = ws.table_nchunk[lane];
                g = ws.table_nsingle[lane];
                s_base[lane] = ws.table_base[lane];
            }
            const int iu = wave_incl_scan_add(u, lane), ic = wave_incl_scan_add(c, lane),
                      ig = wave_incl_scan_add(g, lane);
            if (lane < T) {
                s_tuo[lane] = iu - u;
                s_tco[lane] = ic - c;
                s_tso[lane] = ig - g;
            }
            if (lane == T - 1) {
                s_tuo[T] = iu;
                s_tco[T] = ic;
                s_tso[T] = ig;
            }
        }
        __syncthreads();
        return;
    }
    // kSegThreads threads, each owns a run of consecutive tables
    constexpr int kPer = (DQRM_MAX_TABLES + kSegThreads - 1) / kSegThreads; // 4
    int u[kPer], c[kPer], g[kPer], su = 0, sc = 0, sg = 0;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int t = tid * kPer + q;
        u[q] = c[q] = g[q] = 0;
        if (t < T) {
            u[q] = ws.table_nuniq[t];
            c[q] = ws.table_nchunk[t];
            g[q] = ws.table_nsingle[t];
            s_base[t] = ws.table_base[t];
        }
        su += u[q];
        sc += c[q];
        sg += g[q];
    }
    int tot_u, tot_c, tot_g;
    int eu = block_excl_scan_add<kSegThreads / kWave>(su, lane, wave, s_w, &tot_u);
    int ec = block_excl_scan_add<kSegThreads / kWave>(sc, lane, wave, s_w, &tot_c);
    int eg = block_excl_scan_add<kSegThreads / kWave>(sg, lane, wave, s_w, &tot_g);
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int t = tid * kPer + q;
        if (t < T) {
            s_tuo[t] = eu;
            s_tco[t] = ec;
            s_tso[t] = eg;
        }
        eu += u[q];
        ec += c[q];
        eg += g[q];
    }
    if (tid == 0) {
        s_tuo[T] = tot_u;
        s_tco[T] = tot_c;
        s_tso[T] = tot_g;
    }
    __syncthreads();
}

// Dense chunk descriptor, as the summing kernels read it:
//   x  global sorted position of the chunk's first lookup
//   y  len | index of the chunk inside its segment | chunks in the segment (as above)
//   z  global index of the segment (row of `values`)
//   w  table
// Dense single descriptor: x bag, y global index of the segment, z table.
__global__ __launch_bounds__(kSegThreads) void dedupe_finish_kernel(DedupeArgs args)
{
    struct {
        BwdWs ws;
        int32_t *tuo;
        int32_t *num_unique;
        int64_t *uniq_rows;
        int32_t *seg_offsets;
        int64_t N;
        int T;
    } a = {args.b[blockIdx.y].ws,        args.b[blockIdx.y].tuo,         args.b[blockIdx.y].num_unique,
           args.b[blockIdx.y].uniq_rows, args.b[blockIdx.y].seg_offsets, args.b[blockIdx.y].N,
           args.T};
    __shared__ int s_tco[DQRM_MAX_TABLES + 1];
    __shared__ int s_tso[DQRM_MAX_TABLES + 1];
    __shared__ int s_tuo[DQRM_MAX_TABLES + 1];
    __shared__ int s_base[DQRM_MAX_TABLES];
    __shared__ int s_w[kSegThreads / kWave];
    const int T = a.T;
    table_offsets_to_lds(a.ws, T, s_tuo, s_tco, s_tso, s_base, s_w);
    const int C = s_tco[T], U = s_tuo[T], S = s_tso[T];
    if (blockIdx.x == 0) {
        for (int k = threadIdx.x; k <= T; k += kSegThreads) a.tuo[k] = s_tuo[k];
        if (threadIdx.x == 0) {
            *a.num_unique = U;
            a.seg_offsets[U] = (int32_t)a.N;
            a.ws.totals[0] = C;
            a.ws.totals[1] = U;
            a.ws.totals[2] = S;
        }
    }
    const int first = (int)(blockIdx.x * kSegThreads + threadIdx.x), step = (int)(gridDim.x * kSegThreads);
    for (int c = first; c < C; c += step) {
        const int t = table_of(s_tco, T, c);
        const int4 d = a.ws.chunk_local[s_base[t] + (c - s_tco[t])];
        const int j = s_tuo[t] + d.z;
        if (desc_kchunk(d) == 0) { // first chunk of its segment: d.x is the segment's head
            a.uniq_rows[j] = (int64_t)(unsigned)d.w;
            a.seg_offsets[j] = d.x;
        }
        a.ws.chunk_desc[c] = make_int4(d.x, d.y, j, t);
    }
    // the bags of chunk c's lookups at a place that depends on c alone (a chunk has at least two lookups,
    // so there are at most N / 2 chunks): DQRM_SEG_CHUNK consecutive threads per chunk
    for (int64_t w = first; w < (int64_t)C * DQRM_SEG_CHUNK; w += step) {
        const int c = (int)(w / DQRM_SEG_CHUNK), i = (int)(w % DQRM_SEG_CHUNK);
        const int t = table_of(s_tco, T, c);
        const int4 d = a.ws.chunk_local[s_base[t] + (c - s_tco[t])];
        if (i < desc_len(d)) a.ws.chunk_bags[w] = a.ws.sorted_bag[d.x + i];
    }
    for (int c = first; c < S; c += step) {
        const int t = table_of(s_tso, T, c);
        const int4 d = a.ws.single_local[s_base[t] + (c - s_tso[t])]; // {sorted position, bag, segment, row}
        const int j = s_tuo[t] + d.z;
        a.uniq_rows[j] = (int64_t)(unsigned)d.w;
        a.seg_offsets[j] = d.x;
        a.ws.single_desc[c] = make_int4(d.y, j, t, 0);
    }
}

// ---------------------------------------------------------------------------
// dqrm_segment_sum: chunk sums, then the combine of long segments, then absmax.

struct SegArgs {
    const float *grad_out;
    BwdWs ws;
    float *values;
    float *g_absmax;
    int64_t N;
    int T, B, D;
};

__device__ __forceinline__ float4 f4_add(float4 a, float4 b)
{
    return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
}

// 16 bytes that this kernel reads exactly once (a gradient row is added into one segment only): a streaming
// load, so that they do not push the lists and sums that are read again out of the caches
__device__ __forceinline__ float4 load_once_f4(const float *p)
{
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    return make_float4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ float f4_absmax(float4 a)
{
    return fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w)));
}

// Per-block maxima of |values| by table, kept in LDS (bit patterns of
// non-negative floats order like unsigned integers) and flushed once per block.
struct BlockAbsmax {
    unsigned *s_max; // [T] in LDS
    __device__ __forceinline__ void init(unsigned *lds, int T)
    {
        s_max = lds;
        for (int k = threadIdx.x; k < T; k += blockDim.x) s_max[k] = 0u;
        // the caller synchronises before the first add()
    }
    __device__ __forceinline__ void add(int t, float v)
    {
        const unsigned b = __float_as_uint(v);
        if (b > s_max[t]) atomicMax(s_max + t, b);
    }
    // all threads of the block; publishes the block's maxima
    __device__ __forceinline__ void flush(float *slots, int T)
    {
        __syncthreads();
        for (int k = threadIdx.x; k < T; k += blockDim.x) {
            const unsigned b = s_max[k];
            if (b != 0u)
                atomicMax(reinterpret_cast<unsigned *>(absmax_slot(slots, k, blockIdx.x & (kAbsmaxSlots - 1))), b);
        }
    }
};

// entries of a chunk's bag list that each lane of a group of g lanes holds
constexpr int kChunkIdsPerLane(int g) { return (DQRM_SEG_CHUNK + g - 1) / g; }

// The chunk's bag list: each lane fetches its share once (the whole 32-entry record, whatever the chunk's
// length: the list sits at a place known from the chunk's index, so no descriptor is needed to ask for it).
template <int G>
__device__ __forceinline__ void load_chunk_bags(const SegArgs &a, int c, int lg, int (&my_bags)[kChunkIdsPerLane(G)])
{
    const int *bags = a.ws.chunk_bags + (int64_t)c * DQRM_SEG_CHUNK;
#pragma unroll
    for (int q = 0; q < kChunkIdsPerLane(G); ++q) {
        const int i = q * G + lg;
        my_bags[q] = i < DQRM_SEG_CHUNK ? bags[i] : 0;
    }
}

// Sum of one chunk: its gradient rows, left to right.
//
// Every load of a batch is issued before the first is used, and none sits under a
// per-lane branch: a lane without a row at position i reads the row of bag 0
// instead and leaves it out of the sum.  (With loads under divergent branches the
// compiler cannot count the loads in flight and waits for all of them before each
// next one.)  `wave_len` is the longest chunk among the wave's groups: batches
// and quarters of batches beyond it are skipped by the whole wave.
template <int G>
__device__ __forceinline__ float4 sum_chunk(const int (&my_bags)[kChunkIdsPerLane(G)], int len, int wave_len, int leader,
                                            const float *g0, unsigned tD)
{
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    constexpr int kBatch = kSegBatch, kQuarter = kBatch / 4;
#pragma unroll
    for (int i0 = 0; i0 < DQRM_SEG_CHUNK; i0 += kBatch) {
        if (i0 < wave_len) {
            float4 g[kBatch];
#pragma unroll
            for (int q0 = 0; q0 < kBatch; q0 += kQuarter) {
                if (q0 == 0 || i0 + q0 < wave_len) {
#pragma unroll
                    for (int q = q0; q < q0 + kQuarter; ++q) {
                        const int i = i0 + q;
                        int b = __shfl(my_bags[i / G], leader + (i % G), kWave); // the group passes the bags round
                        b = i < len ? b : 0;
                        g[q] = load_once_f4(g0 + (uint64_t)(unsigned)b * tD);
                    }
                } else {
#pragma unroll
                    for (int q = q0; q < q0 + kQuarter; ++q) g[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
#pragma unroll
            for (int q = 0; q < kBatch; ++q) {
                const int i = i0 + q;
                if (i < len) acc = (i == 0) ? g[q] : f4_add(acc, g[q]);
            }
        }
    }
    return acc;
}

// Where the sum of chunk k of a segment of more than one chunk is parked: full chunks are disjoint runs of
// DQRM_SEG_CHUNK sorted positions, so (position / DQRM_SEG_CHUNK) names them uniquely; the last chunk of a
// segment is filed under the slot of the segment's first chunk, in a second array.  The segment's arrival
// counter sits at the first chunk's slot number too.
__device__ __forceinline__ float *partial_slot(const BwdWs &ws, int head_pos, int k, int nchunks, int D)
{
    return k == nchunks - 1 ? ws.partial_last + (int64_t)(head_pos / DQRM_SEG_CHUNK) * D
                            : ws.partial_full + (int64_t)(head_pos / DQRM_SEG_CHUNK + k) * D;
}

// Parked chunk sums and arrival counters are the only data that one workgroup of this kernel hands to another.
// They travel by device-scope atomic stores, loads and adds (each coherent across the chip by itself: they go
// past the caches that are private to a part of the chip), in this order: a chunk's sum is stored and the
// stores are waited for; then the chunk is counted in; the wave that sees the count complete then loads the
// sums.  No fence is used: a device-scope release or acquire writes back or drops whole caches, which costs more
// than the entire kernel when thousands of waves do it.
__device__ __forceinline__ void park_f4(float *p, float4 v)
{
    __hip_atomic_store(p + 0, v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 1, v.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 2, v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 3, v.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int kCombineBatch = 64; // chunk sums of one column requested together

// One column of the sum of a segment of `nchunks` > 1 chunks: its parked chunk sums, left to right.  (4 bytes per
// chunk and lane, so that even kCombineBatch chunks cost a single round trip: a wave per segment, a lane per column.)
__device__ __forceinline__ float combine_column(const BwdWs &ws, int head_pos, int nchunks, int D, int col)
{
    float acc = 0.f;
    for (int k0 = 0; k0 < nchunks; k0 += kCombineBatch) {
        float pv[kCombineBatch];
#pragma unroll
        for (int q = 0; q < kCombineBatch; ++q)
            if (k0 + q < nchunks)
                pv[q] = __hip_atomic_load(partial_slot(ws, head_pos, k0 + q, nchunks, D) + col, __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int q = 0; q < kCombineBatch; ++q)
            if (k0 + q < nchunks) acc = (k0 + q == 0) ? pv[q] : acc + pv[q];
    }
    return acc;
}

// The same for rows narrower than a wave: the wave's lanes are split among several segments, so `head_pos` and
// `nchunks` differ from lane to lane (nchunks = 0: a lane without a column to add).  All lanes go through the
// motions up to `wave_n`, the largest nchunks in the wave; a lane past its own last chunk asks for that chunk again.
__device__ __forceinline__ float combine_column_shared_wave(const BwdWs &ws, int head_pos, int nchunks, int wave_n, int D,
                                                            int col)
{
    float acc = 0.f;
    for (int k0 = 0; k0 < wave_n; k0 += kCombineBatch) {
        float pv[kCombineBatch];
#pragma unroll
        for (int q = 0; q < kCombineBatch; ++q) {
            pv[q] = 0.f;
            if (k0 + q < wave_n) {
                const float *p = nchunks > 0 ? partial_slot(ws, head_pos, min(k0 + q, nchunks - 1), nchunks, D) + col
                                             : ws.partial_full;
                pv[q] = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
#pragma unroll
        for (int q = 0; q < kCombineBatch; ++q)
            if (k0 + q < nchunks) acc = (k0 + q == 0) ? pv[q] : acc + pv[q];
    }
    return acc;
}

// Work of one workgroup of kSumThreads / G lane groups:
//  * singles (rows looked up once: a plain copy of one gradient row), a few per
//    group, spread evenly over all groups of the grid;
//  * chunks, one per lane group and round.  The sum of a segment's only chunk is
//    final.  The sum of a chunk of a longer segment is parked; the chunk then counts
//    itself in, and if it completes its segment's count, its whole wave (a lane per
//    column) adds the segment's parked sums in chunk order, stores the row of
//    `values`, and clears the counter for the next use.
// No load sits under a per-lane branch: a group without work goes through the
// motions on bag 0 of table 0 and stores nothing.
constexpr int kSinglesPerGroup = 4;

template <int G>
__device__ __forceinline__ void segment_sum_body(const SegArgs &a)
{
    constexpr int kGroups = kSumThreads / G; // lane groups per workgroup
    __shared__ unsigned s_max[DQRM_MAX_TABLES];
    const int T = a.T, D = a.D;
    BlockAbsmax amax;
    amax.init(s_max, T);

    const int lg = threadIdx.x & (G - 1);
    const int grp = (int)threadIdx.x / G;
    const int col = lg * 4;
    const bool col_ok = col < D;
    const float *grad_col = a.grad_out + (col_ok ? col : 0); // lanes beyond the row read column 0 and store nothing
    const int lane = threadIdx.x & (kWave - 1);
    const int leader = lane & ~(G - 1);
    const unsigned tD = (unsigned)T * (unsigned)D;
    const int cap = (int)a.N;       // both lists have N slots, so descriptors may be requested before the counts are known
    const int cap_chunks = cap / 2; // a chunk has at least two lookups
    const int ngroups = (int)gridDim.x * kGroups;
    const int gi = (int)blockIdx.x * kGroups + grp;

    // ---- requests that need no count: the first chunk's descriptor and bag list, the first singles
    // Wide rows: consecutive chunks for the groups of a wave (they are alike in length, so few lanes idle).  Narrow
    // rows (many groups per wave): the wave's groups take chunks a whole grid's waves apart, or the chunks of a small
    // table's rows would all complete their segments in one wave, which adds them up a few per round trip.
    int c = gi;
    if constexpr (G < 16) {
        constexpr int kWavesPerBlock = kSumThreads / kWave, kGroupsPerWave = kWave / G;
        c = ((int)blockIdx.x * kWavesPerBlock + (int)threadIdx.x / kWave) + (grp % kGroupsPerWave) * ((int)gridDim.x * kWavesPerBlock);
    }
    int4 d = make_int4(0, 0, 0, 0);
    int my_bags[kChunkIdsPerLane(G)] = {};
    if (c < cap_chunks) {
        d = a.ws.chunk_desc[c];
        load_chunk_bags<G>(a, c, lg, my_bags);
    }
    int s0 = gi * kSinglesPerGroup;
    int4 sd[kSinglesPerGroup];
#pragma unroll
    for (int k = 0; k < kSinglesPerGroup; ++k) sd[k] = a.ws.single_desc[min(s0 + k, max(cap - 1, 0))];
    const int C = min(a.ws.totals[0], cap_chunks), S = min(a.ws.totals[2], cap);
    __syncthreads(); // s_max is cleared

    // ---- singles: the wave's first group holds the lowest positions
    while (__builtin_amdgcn_readfirstlane(s0) < S) {
        float4 r[kSinglesPerGroup];
        int4 cur[kSinglesPerGroup];
#pragma unroll
        for (int k = 0; k < kSinglesPerGroup; ++k) {
            cur[k] = s0 + k < S ? sd[k] : make_int4(0, 0, 0, 0);
            r[k] = load_once_f4(grad_col + (uint64_t)(unsigned)cur[k].x * tD + (unsigned)cur[k].z * (unsigned)D);
        }
        const int s_next = s0 + ngroups * kSinglesPerGroup;
#pragma unroll
        for (int k = 0; k < kSinglesPerGroup; ++k) sd[k] = a.ws.single_desc[min(s_next + k, cap - 1)];
#pragma unroll
        for (int k = 0; k < kSinglesPerGroup; ++k) {
            if (s0 + k < S && col_ok) {
                *reinterpret_cast<float4 *>(a.values + (int64_t)cur[k].y * D + col) = r[k];
                amax.add(cur[k].z, f4_absmax(r[k]));
            }
        }
        s0 = s_next;
    }

    // ---- chunks: the wave's first group holds the lowest index
    while (__builtin_amdgcn_readfirstlane(c) < C) {
        const int c_next = c + ngroups;
        int4 d_next = make_int4(0, 0, 0, 0);
        int next_bags[kChunkIdsPerLane(G)] = {};
        if (__builtin_amdgcn_readfirstlane(c_next) < C) { // whole wave or none; groups past C - 1 read slots that exist
            d_next = a.ws.chunk_desc[min(c_next, cap_chunks - 1)];
            load_chunk_bags<G>(a, min(c_next, cap_chunks - 1), lg, next_bags);
        }
        const bool live = c < C;
        int len = live ? desc_len(d) : 0;
        len = len > DQRM_SEG_CHUNK ? DQRM_SEG_CHUNK : len;
        const int wave_len = __builtin_amdgcn_readfirstlane(wave_max_int(len));
        const int nchunks = desc_nchunks(d), kchunk = desc_kchunk(d);
        const int t = live ? d.w : 0;
        const float4 acc = sum_chunk<G>(my_bags, len, wave_len, leader, grad_col + (unsigned)t * (unsigned)D, tD);
        const bool parks = live && nchunks > 1;
        const int head_pos = d.x - kchunk * DQRM_SEG_CHUNK; // sorted position of the segment's head
        if (live && col_ok) {
            if (parks) {
                park_f4(partial_slot(a.ws, head_pos, kchunk, nchunks, D) + col, acc);
            } else {
                *reinterpret_cast<float4 *>(a.values + (int64_t)d.z * D + col) = acc;
                amax.add(t, f4_absmax(acc));
            }
        }
        if (__any(parks)) { // wave-uniform
            // the parked sums have reached the chip-wide level before any of this wave's chunks is counted in
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            int before = -1;
            if (parks && lg == 0)
                before = __hip_atomic_fetch_add(a.ws.seg_count + head_pos / DQRM_SEG_CHUNK, 1, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("" ::: "memory"); // (the loads below stay below)
            // the groups whose chunk completed its segment's count: the wave adds up their segments
            unsigned long long todo = __ballot(parks && lg == 0 && before == nchunks - 1);
            if constexpr (G >= 16) { // a row fills the wave: a lane per column, the segments one by one
                while (todo != 0ull) {
                    const int src = __ffsll((long long)todo) - 1;
                    todo &= todo - 1ull;
                    const int s_head = __builtin_amdgcn_readlane(head_pos, src), s_n = __builtin_amdgcn_readlane(nchunks, src);
                    const int s_seg = __builtin_amdgcn_readlane(d.z, src), s_t = __builtin_amdgcn_readlane(d.w, src);
                    float m = 0.0f;
                    for (int cc = lane; cc < D; cc += kWave) {
                        const float sum = combine_column(a.ws, s_head, s_n, D, cc);
                        a.values[(int64_t)s_seg * D + cc] = sum;
                        m = fmaxf(m, fabsf(sum));
                    }
                    m = wave_max(m);
                    if (lane == 0) {
                        amax.add(s_t, m);
                        // (ready for another run of the segment sums on the same dedupe)
                        __hip_atomic_store(a.ws.seg_count + s_head / DQRM_SEG_CHUNK, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            } else { // narrow rows: 4 G lanes per segment, 16 / G segments in one round trip
                constexpr int kLanesPerSeg = 4 * G, kSegsPerPass = kWave / kLanesPerSeg;
                const int slot = lane / kLanesPerSeg, cc = lane % kLanesPerSeg;
                while (todo != 0ull) {
                    int src = -1;
#pragma unroll
                    for (int j = 0; j < kSegsPerPass; ++j) {
                        if (todo != 0ull) {
                            if (slot == j) src = __ffsll((long long)todo) - 1;
                            todo &= todo - 1ull;
                        }
                    }
                    const int from = src < 0 ? 0 : src;
                    const int s_head = __shfl(head_pos, from, kWave);
                    const int n_from = __shfl(nchunks, from, kWave);
                    const int s_n = src >= 0 && cc < D ? n_from : 0;
                    const int s_seg = __shfl(d.z, from, kWave), s_t = __shfl(d.w, from, kWave);
                    const int wave_n = __builtin_amdgcn_readfirstlane(wave_max_int(s_n));
                    const float sum = combine_column_shared_wave(a.ws, s_head, s_n, wave_n, D, cc);
                    if (s_n > 0) a.values[(int64_t)s_seg * D + cc] = sum;
                    float m = s_n > 0 ? fabsf(sum) : 0.0f;
#pragma unroll
                    for (int o = kLanesPerSeg / 2; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, kWave));
                    if (src >= 0 && cc == 0) {
                        amax.add(s_t, m);
                        __hip_atomic_store(a.ws.seg_count + s_head / DQRM_SEG_CHUNK, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
        }
        c = c_next;
        d = d_next;
#pragma unroll
        for (int q = 0; q < kChunkIdsPerLane(G); ++q) my_bags[q] = next_bags[q];
    }
    amax.flush(a.ws.absmax_slots, T);
}

template <int G>
__global__ __launch_bounds__(kSumThreads, 4) void segment_sum_kernel(SegArgs a)
{
    segment_sum_body<G>(a);
}

// The segment sums of several batches in one launch (blockIdx.y picks the batch): small batches, such as the
// micro-batches of simulated data parallelism, are a chain of dependent round trips with little else to do, and
// several of them side by side cost hardly more than one.
struct SegMulti {
    SegArgs b[DQRM_MAX_DEDUPE_BATCHES];
};

template <int G>
__global__ __launch_bounds__(kSumThreads, 4) void segment_sum_multi_kernel(SegMulti m)
{
    segment_sum_body<G>(m.b[blockIdx.y]);
}

// g_absmax[t] = max over the table's slots
// (and clears them, so that the segment sums may be repeated on the same dedupe)
__device__ __forceinline__ void absmax_finalize_body(float *__restrict__ slots, int T, float *__restrict__ g_absmax)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    float v[kAbsmaxSlots];
#pragma unroll
    for (int k = 0; k < kAbsmaxSlots; ++k) v[k] = *absmax_slot(slots, t, k);
    float m = 0.0f;
#pragma unroll
    for (int k = 0; k < kAbsmaxSlots; ++k) {
        m = fmaxf(m, v[k]);
        *absmax_slot(slots, t, k) = 0.0f;
    }
    g_absmax[t] = m;
}

__global__ void absmax_finalize_kernel(float *__restrict__ slots, int T, float *__restrict__ g_absmax)
{
    absmax_finalize_body(slots, T, g_absmax);
}

struct AbsmaxMulti {
    float *slots[DQRM_MAX_DEDUPE_BATCHES];
    float *g_absmax[DQRM_MAX_DEDUPE_BATCHES]; // an entry may be null: that batch's maxima are not wanted
    int T;
};

__global__ void absmax_finalize_multi_kernel(AbsmaxMulti m)
{
    if (m.g_absmax[blockIdx.y]) absmax_finalize_body(m.slots[blockIdx.y], m.T, m.g_absmax[blockIdx.y]);
}

} // namespace dqrm
