/*
 * CPU oracle for the embedding-table hot path of DQRM (arXiv 2410.20046).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * single-threaded restatement of what the path computes, written so that it
 * can be checked against the paper by eye.  Only the tests, the smoke check and
 * the benchmark's "cpu_baseline" leg may call it.  It shares no code, header,
 * table or constant with the GPU library.
 *
 * What the paper fixes (and where):
 *   - Sec. 3.1 "Reducing Memory of Unused Weights": the embedding lookup runs
 *     first and only the rows a batch touches are copied and quantised; the
 *     fp32 table stays the master copy.
 *   - Sec. 3.2 "Periodic Update to Find Quantization Scale": the scale comes
 *     from a traversal of the whole table and is then reused (cached) for
 *     many iterations.
 *   - Sec. 4.1 "Quantization of Embedding Tables": uniform INT4, ONE scale per
 *     table (not per row).
 *   - Sec. 4.3 and Appendix "Distributed Environment with Gradient
 *     Quantization": the table gradient is kept in sparse (indices, values)
 *     form over the touched rows only ("specified sparsity", lossless); the
 *     scale of a gradient tensor follows from the bit width (INT8) and the
 *     tensor's own values; only the values are quantised, the indices are left
 *     alone; the update dequantises them.
 *
 * What the paper leaves open, and the reading taken here (each is also stated
 * at the function that uses it):
 *   - quantiser: symmetric uniform, scale = max|x| / (2^(b-1) - 1), code =
 *     clamp(round_half_even(x / scale), -2^(b-1), 2^(b-1) - 1), value = scale *
 *     code.  True division, no reciprocal.  Scale floored at 1e-8 so an
 *     all-zero tensor gives all-zero codes.
 *   - a stale (cached) scale clamps out-of-range weights to -8 / +7.
 *   - backward through the quantiser is the identity (straight-through): the
 *     gradient of the quantised row is applied to the fp32 master row.
 *   - pooling is a sum; plain SGD.
 *   - all arithmetic is IEEE binary32 with one rounding per operation (no fused
 *     multiply-add): the codes are decided in that precision.
 *   - order of a segment's floating-point sum: contributions in ascending
 *     lookup position, cut into consecutive chunks of ORACLE_SEG_CHUNK; each
 *     chunk summed left to right starting from its first element; the chunk
 *     sums then summed left to right starting from the first.
 *   - packed INT4 layout: byte k of a row holds element 2k in bits 0..3 and
 *     element 2k+1 in bits 4..7, 4-bit two's complement.
 *
 *   - simulated data parallelism (appendix "Simulated Data Parallelism
 *     Environment"): see oracle_simdp_accumulate.
 *
 * Parity pins (tests/test_oracle_*.py): hand-worked quantiser example, range
 * and round-trip invariants, torch-CPU embedding_bag / sparse coalesce special
 * cases, brute-force dense gradient, integer closed form on dyadic gradients.
 * The paper's accuracy figures need its datasets: parity unpinned for those.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_SEG_CHUNK 32

/* ---- the quantiser (Sec. 4.1: uniform, per table; formula = reading above) */

static float scale_from_absmax(float absmax, int bits)
{
    float qmax = (float)((1 << (bits - 1)) - 1); /* 7 for INT4, 127 for INT8 */
    float s = absmax / qmax;
    return s < 1e-8f ? 1e-8f : s;
}

static int quantize_code(float x, float scale, int bits)
{
    float lo = -(float)(1 << (bits - 1));
    float hi = (float)((1 << (bits - 1)) - 1);
    float r = rintf(x / scale); /* round half to even (default rounding mode) */
    if (r < lo) r = lo;
    if (r > hi) r = hi;
    return (int)r;
}

int oracle_quantize_code(float x, float scale, int bits) { return quantize_code(x, scale, bits); }
float oracle_scale_from_absmax(float absmax, int bits) { return scale_from_absmax(absmax, bits); }
int oracle_seg_chunk(void) { return ORACLE_SEG_CHUNK; }

/* ---- Sec. 3.2: find the per-table weight scale by traversing the table */

void oracle_find_scale(const float *W, const int64_t *row_offsets, int T, int D, float *w_scale)
{
    for (int t = 0; t < T; ++t) {
        float a = 0.0f;
        for (int64_t r = row_offsets[t]; r < row_offsets[t + 1]; ++r)
            for (int j = 0; j < D; ++j) {
                float v = fabsf(W[r * D + j]);
                if (v > a) a = v;
            }
        w_scale[t] = scale_from_absmax(a, 4);
    }
}

/* ---- packed INT4 storage (layout = reading above) */

static void pack_row(const float *w, int D, float scale, uint8_t *dst)
{
    for (int k = 0; k < D / 2; ++k) {
        int q0 = quantize_code(w[2 * k], scale, 4);
        int q1 = quantize_code(w[2 * k + 1], scale, 4);
        dst[k] = (uint8_t)((q0 & 0xF) | ((q1 & 0xF) << 4));
    }
}

static int nibble_to_code(int nib) { return nib >= 8 ? nib - 16 : nib; }

void oracle_pack_int4(const float *W, const int64_t *row_offsets, int T, int D,
                      const float *w_scale, uint8_t *packed)
{
    for (int t = 0; t < T; ++t)
        for (int64_t r = row_offsets[t]; r < row_offsets[t + 1]; ++r)
            pack_row(W + r * D, D, w_scale[t], packed + r * (D / 2));
}

void oracle_unpack_int4(const uint8_t *packed, int64_t rows, int D, int8_t *codes)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int k = 0; k < D / 2; ++k) {
            uint8_t b = packed[r * (D / 2) + k];
            codes[r * D + 2 * k] = (int8_t)nibble_to_code(b & 0xF);
            codes[r * D + 2 * k + 1] = (int8_t)nibble_to_code(b >> 4);
        }
}

/* ---- Sec. 3.1: lookup first, then quantise only the touched rows, then pool.
 *
 * indices [N]  table-local row ids, table-major: table t's bags are bags
 *              t*B .. t*B+B-1
 * offsets [T*B+1]  bag i holds lookups offsets[i] .. offsets[i+1]-1
 * out     [B][T][D]
 * codes   [N][D] or NULL: the INT4 code of every gathered element
 * mode 0: quantise the fp32 master row with the cached scale
 * mode 1: read the packed row (codes already stored)
 * quantise = 0 switches the quantiser off (identity); only the tests use it, to
 * compare the gather + pooling with a library embedding-bag.
 */
void oracle_embbag_fwd(const float *W, const uint8_t *packed, const int64_t *row_offsets,
                       const float *w_scale, int T, int D, int B,
                       const int64_t *indices, const int64_t *offsets,
                       int mode, int quantise, float *out, int8_t *codes)
{
    for (int t = 0; t < T; ++t) {
        float s = w_scale ? w_scale[t] : 1.0f;
        for (int b = 0; b < B; ++b) {
            float *acc = out + ((int64_t)b * T + t) * D;
            for (int j = 0; j < D; ++j) acc[j] = 0.0f;
            int64_t bag = (int64_t)t * B + b;
            for (int64_t i = offsets[bag]; i < offsets[bag + 1]; ++i) {
                int64_t r = row_offsets[t] + indices[i];
                for (int j = 0; j < D; ++j) {
                    float wq;
                    int q = 0;
                    if (!quantise) {
                        wq = W[r * D + j];
                    } else {
                        if (mode == 0) {
                            q = quantize_code(W[r * D + j], s, 4);
                        } else {
                            uint8_t byte = packed[r * (D / 2) + j / 2];
                            q = nibble_to_code((j & 1) ? (byte >> 4) : (byte & 0xF));
                        }
                        wq = s * (float)q; /* dequantised value */
                    }
                    acc[j] = acc[j] + wq; /* sum pooling, left to right */
                    if (codes) codes[i * D + j] = (int8_t)q;
                }
            }
        }
    }
}

/* ---- Sec. 4.3 / Appendix: the sparse ("specified sparsity") table gradient.
 *
 * Because the backward of the quantiser is the identity and pooling is a sum,
 * d loss / d W_t[r] = sum over lookups i of table t with indices[i] == r of
 * grad_out[bag(i)].  The sparse form lists each touched row once (coalesced).
 *
 * Outputs:
 *   sorted_pos [N]   lookup positions ordered by (table, row, position)
 *   uniq_rows  [U]   table-local row of each segment, ascending inside a table
 *   seg_offsets[U+1] start of each segment in sorted_pos; seg_offsets[U] = N
 *   table_uniq_offsets [T+1]  segments of table t are [tuo[t], tuo[t+1])
 *   values [U][D]    the row gradients, summed in the order stated in the header
 *   g_absmax [T]     max |values| over the table's segments (0 if it has none)
 * Returns U.
 */
typedef struct {
    int64_t row;
    int64_t pos;
} lookup_t;

static int cmp_lookup(const void *a, const void *b)
{
    const lookup_t *x = (const lookup_t *)a, *y = (const lookup_t *)b;
    if (x->row != y->row) return x->row < y->row ? -1 : 1;
    if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
    return 0;
}

int64_t oracle_embbag_bwd(int T, int D, int B, const int64_t *indices, const int64_t *offsets,
                          const float *grad_out, int32_t *sorted_pos, int64_t *uniq_rows,
                          int32_t *seg_offsets, int32_t *table_uniq_offsets, float *values,
                          float *g_absmax)
{
    int64_t N = offsets[(int64_t)T * B];
    lookup_t *lk = (lookup_t *)malloc(sizeof(lookup_t) * (size_t)(N > 0 ? N : 1));
    int64_t *bag_of = (int64_t *)malloc(sizeof(int64_t) * (size_t)(N > 0 ? N : 1));
    float *partial = (float *)malloc(sizeof(float) * (size_t)D);
    int64_t U = 0;

    for (int64_t bag = 0; bag < (int64_t)T * B; ++bag)
        for (int64_t i = offsets[bag]; i < offsets[bag + 1]; ++i) bag_of[i] = bag;

    for (int t = 0; t < T; ++t) {
        int64_t lo = offsets[(int64_t)t * B], hi = offsets[(int64_t)(t + 1) * B];
        for (int64_t i = lo; i < hi; ++i) {
            lk[i].row = indices[i];
            lk[i].pos = i;
        }
        qsort(lk + lo, (size_t)(hi - lo), sizeof(lookup_t), cmp_lookup);

        table_uniq_offsets[t] = (int32_t)U;
        float amax = 0.0f;
        int64_t i = lo;
        while (i < hi) {
            int64_t e = i;
            while (e < hi && lk[e].row == lk[i].row) ++e; /* segment [i, e) */
            uniq_rows[U] = lk[i].row;
            seg_offsets[U] = (int32_t)i;
            float *v = values + U * D;
            for (int64_t c = i; c < e; c += ORACLE_SEG_CHUNK) {
                int64_t ce = c + ORACLE_SEG_CHUNK < e ? c + ORACLE_SEG_CHUNK : e;
                for (int64_t k = c; k < ce; ++k) {
                    int64_t b = bag_of[lk[k].pos] - (int64_t)t * B;
                    const float *g = grad_out + (b * T + t) * D;
                    for (int j = 0; j < D; ++j) partial[j] = (k == c) ? g[j] : partial[j] + g[j];
                }
                for (int j = 0; j < D; ++j) v[j] = (c == i) ? partial[j] : v[j] + partial[j];
            }
            for (int j = 0; j < D; ++j)
                if (fabsf(v[j]) > amax) amax = fabsf(v[j]);
            ++U;
            i = e;
        }
        g_absmax[t] = amax;
        for (int64_t k = lo; k < hi; ++k) sorted_pos[k] = (int32_t)lk[k].pos;
    }
    table_uniq_offsets[T] = (int32_t)U;
    seg_offsets[U] = (int32_t)N;
    free(lk);
    free(bag_of);
    free(partial);
    return U;
}

/* ---- Appendix: INT8 quantisation of the sparse gradient's values only.  One
 * scale per table per step, from the table's own values (on one device the
 * "unified" scale is the local one). */
void oracle_grad_quant_int8(int T, int D, const float *values, const int32_t *table_uniq_offsets,
                            const float *g_absmax, int8_t *gq, float *g_scale)
{
    for (int t = 0; t < T; ++t) {
        float gs = scale_from_absmax(g_absmax[t], 8);
        g_scale[t] = gs;
        for (int64_t u = table_uniq_offsets[t]; u < table_uniq_offsets[t + 1]; ++u)
            for (int j = 0; j < D; ++j)
                gq[u * D + j] = (int8_t)quantize_code(values[u * D + j], gs, 8);
    }
}

/* ---- Appendix: dequantise and apply the local (sparse) SGD step to the fp32
 * master rows; if a packed mirror exists, re-encode the touched rows with the
 * cached weight scale. */
void oracle_sparse_update(float *W, uint8_t *packed, const int64_t *row_offsets,
                          const float *w_scale, int T, int D, const int64_t *uniq_rows,
                          const int32_t *table_uniq_offsets, const int8_t *gq,
                          const float *g_scale, float lr)
{
    for (int t = 0; t < T; ++t)
        for (int64_t u = table_uniq_offsets[t]; u < table_uniq_offsets[t + 1]; ++u) {
            int64_t r = row_offsets[t] + uniq_rows[u];
            for (int j = 0; j < D; ++j) {
                float g = g_scale[t] * (float)gq[u * D + j];
                float step = lr * g;
                W[r * D + j] = W[r * D + j] - step;
            }
            if (packed) pack_row(W + r * D, D, w_scale[t], packed + r * (D / 2));
        }
}

/* ---- Appendix "Simulated Data Parallelism Environment" (its algorithm), for the
 * embedding tables, with the INT8 gradient quantisation of the appendix on
 * distributed training.
 *
 * Every parameter has a gradient buffer of its own shape.  The batch is split
 * into micro-batches, one per simulated node; each micro-batch runs forward and
 * backward on the unchanged weights and its gradient is added to the buffer;
 * after the last micro-batch of a group the weights are updated from the buffer,
 * and the buffer is cleared before the next gradient arrives.  With quantised
 * gradients the scale of the group's first micro-batch is reused for the others
 * (the two all-reduce rounds of the real run are not simulated), so later
 * micro-batches may clip.
 *
 * Readings (the appendix does not say): the buffer holds what an all-reduce of
 * the integer gradients would deliver, the SUM OF THE INT8 CODES (exact integer
 * arithmetic, independent of order), and is dequantised once:
 * step = lr * (g_scale[t] * (float)sum), two roundings.  Nothing is divided by
 * the number of nodes: the algorithm adds, the caller's lr decides.  Rows that
 * no micro-batch touched keep their weights and nibbles (their buffer is zero).
 *
 * oracle_simdp_accumulate is the algorithm's buffer update for one micro-batch:
 * buffer [rows][D] int32 and touched [rows] cover all tables (row_offsets). */
void oracle_simdp_accumulate(int T, int D, const int64_t *row_offsets, const int64_t *uniq_rows,
                             const int32_t *table_uniq_offsets, const int8_t *gq, int32_t *buffer,
                             uint8_t *touched)
{
    for (int t = 0; t < T; ++t)
        for (int64_t u = table_uniq_offsets[t]; u < table_uniq_offsets[t + 1]; ++u) {
            int64_t r = row_offsets[t] + uniq_rows[u];
            touched[r] = 1;
            for (int j = 0; j < D; ++j) buffer[r * D + j] += (int32_t)gq[u * D + j];
        }
}

/* ... and its weight update from the buffer (the caller clears the buffer before
 * the next group, as the algorithm does). */
void oracle_simdp_weight_update(float *W, uint8_t *packed, const int64_t *row_offsets,
                                const float *w_scale, int T, int D, const int32_t *buffer,
                                const uint8_t *touched, const float *g_scale, float lr)
{
    for (int t = 0; t < T; ++t)
        for (int64_t r = row_offsets[t]; r < row_offsets[t + 1]; ++r) {
            if (!touched[r]) continue;
            for (int j = 0; j < D; ++j) {
                float g = g_scale[t] * (float)buffer[r * D + j];
                float step = lr * g;
                W[r * D + j] = W[r * D + j] - step;
            }
            if (packed) pack_row(W + r * D, D, w_scale[t], packed + r * (D / 2));
        }
}
