/*
 * dqrm.h -- C ABI of the MI355X (gfx950) library for the embedding-table hot path
 * of DQRM (arXiv 2410.20046): quantisation-aware training of DLRM embedding
 * tables with INT4 weights and INT8 sparse gradients.
 *
 * One training step of the path, in call order:
 *
 *   dqrm_find_scale      every P steps   per-table weight scale      (Sec. 3.2)
 *   dqrm_pack_int4       after the above packed INT4 mirror          (Sec. 4.2, sizes; demo appendix)
 *   dqrm_embbag_fwd      every step      gather -> INT4 fake-quant -> sum-pool   (Sec. 3.1, Sec. 4.1)
 *   dqrm_embbag_bwd      every step      dedupe -> segment-sum = sparse gradient (Sec. 4.3, "specified sparsity")
 *   dqrm_grad_quant_int8 every step      INT8 codes of the gradient values       (Appendix, gradient quantisation)
 *   dqrm_sparse_update   every step      dequantise + SGD on touched rows        (same appendix)
 *   dqrm_sparse_merge    per group       sum of several micro-batches' integer gradients (Appendix, simulated data parallelism)
 * and, between the forward and the backward of the tables, the dense part of the model:
 *   dqrm_dense_step      every step      MLPs, interaction, loss, their backward, dense SGD
 *   dqrm_dense_step_quant  the same with channel-wise INT4 weights and / or INT8 gradients + error compensation
 *
 * Conventions common to every entry point
 *   - Returns 0 (DQRM_OK) or a negative DQRM_ERR_* code.  Never throws, never aborts.
 *   - Arguments are validated on the host BEFORE anything is launched; on a
 *     validation error nothing is enqueued and no buffer is written.
 *   - Unless a parameter is documented as "host", every pointer is a DEVICE
 *     pointer owned by the caller.  The library allocates nothing, frees
 *     nothing, and keeps no pointer after the call returns.
 *   - `stream` is a hipStream_t passed as void*.  Every call only enqueues work
 *     on that stream and returns; only dqrm_check_status() synchronises.
 *   - Data-dependent problems (an index outside its table, offsets that go
 *     backwards, more lookups in one table than the dedupe kernel holds) cannot
 *     be seen by the host.  Kernels never act on such data (the lookup is
 *     skipped, so every access stays inside the caller's buffers); they record
 *     the first problem in a per-device status word that dqrm_check_status()
 *     reads and clears.
 *   - All floating point is IEEE binary32, one rounding per operation (no fused
 *     multiply-add), true division.
 *
 * The quantiser (the paper states "uniform", "one scale per table"; the formula
 * is this library's reading): scale = max(absmax / (2^(b-1) - 1), 1e-8),
 * code = clamp(round_half_even(x / scale), -2^(b-1), 2^(b-1) - 1), value =
 * scale * code; b = 4 for weights, b = 8 for gradients.
 */
#ifndef DQRM_H
#define DQRM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DQRM_OK 0
#define DQRM_ERR_INVALID_ARG (-1)         /* null pointer, negative size, unknown mode */
#define DQRM_ERR_UNSUPPORTED (-2)         /* dim, table count or table size outside the limits below */
#define DQRM_ERR_WORKSPACE_TOO_SMALL (-3) /* workspace_bytes below what the call's *_workspace_bytes() query returns */
#define DQRM_ERR_INDEX_OUT_OF_RANGE (-4)  /* (device status) an index < 0 or >= its table's rows */
#define DQRM_ERR_HIP (-5)                 /* a HIP runtime call failed; see dqrm_last_hip_error() */
#define DQRM_ERR_CAPACITY (-6)            /* (device status) one table has > DQRM_MAX_TABLE_LOOKUPS lookups in a batch;
                                             dqrm_sparse_merge: the outputs cannot hold the blocks' rows */
#define DQRM_ERR_BAD_OFFSETS (-7)         /* (device status) offsets decrease or leave [0, num_indices];
                                             dqrm_sparse_merge: a block's offsets or row order break its rules */

#define DQRM_ERR_SCRATCH_LIMIT (-8)       /* dqrm_embbag_bwd_noalloc: the shape needs more scratch than the built-in array holds */

#define DQRM_MAX_DIM 256             /* dim must be a multiple of 8 in [8, 256] */
#define DQRM_MAX_TABLES 1024
#define DQRM_MAX_TABLE_ROWS 2147483646LL /* rows of one table */
#define DQRM_MAX_TABLE_LOOKUPS 65536 /* lookups one table may receive in one batch (up to 16384 are sorted in LDS by
                                        one workgroup; more take a slower path through the workspace).
                                        NOTE: a table beyond the limit is SKIPPED for that batch -- it contributes
                                        no unique rows, so its rows get no update -- and the only trace is
                                        DQRM_ERR_CAPACITY in the device status word.  The host cannot refuse such
                                        a batch beforehand (the per-table counts are device data), so a training
                                        loop has to call dqrm_check_status now and then to notice. */
#define DQRM_MAX_DEDUPE_BATCHES 8    /* batches one dqrm_dedupe_multi call may take */

/* Order of a segment's floating-point sum (the paper does not fix one; results
 * must be reproducible bit for bit, because the INT8 scale and codes depend on
 * the last bit): contributions in ascending lookup position are cut into
 * consecutive chunks of DQRM_SEG_CHUNK; each chunk is summed left to right
 * starting from its first element; the chunk sums are summed left to right. */
#define DQRM_SEG_CHUNK 32

#define DQRM_FWD_MASTER 0 /* forward quantises the fp32 master rows */
#define DQRM_FWD_PACKED 1 /* forward reads the packed INT4 mirror */

/* The embedding layer.  T tables are stored back to back: table t owns rows
 * row_offsets[t] .. row_offsets[t+1]-1 of `master` ([R][dim] fp32, row-major)
 * and of `packed` ([R][dim/2] bytes; byte k of a row = element 2k in bits 0..3,
 * element 2k+1 in bits 4..7, 4-bit two's complement).  `packed` may be NULL if
 * no call uses it.  The struct itself is read on the host during the call. */
typedef struct {
    int32_t num_tables;              /* T, 1 .. DQRM_MAX_TABLES */
    int32_t dim;                     /* D */
    const int64_t *row_offsets_host; /* HOST [T+1], row_offsets[0] = 0, non-decreasing */
    const int64_t *row_offsets_dev;  /* device copy of the same [T+1] */
    float *master;                   /* device [R][D] */
    uint8_t *packed;                 /* device [R][D/2] or NULL */
    float *w_scale;                  /* device [T] per-table weight scale (the cached scale of Sec. 3.2) */
} dqrm_tables_t;

/* Sec. 3.2 (find the quantisation scale by traversing the table):
 * w_scale[t] = max(max|master_t| / 7, 1e-8).  Reads all of `master`. */
int32_t dqrm_find_scale(const dqrm_tables_t *tables, void *stream);

/* Packed INT4 storage (2 codes per byte: the 8x model-size reduction of the
 * results tables): re-encodes every row of `master` into `packed` with the
 * current w_scale.  Requires tables->packed. */
int32_t dqrm_pack_int4(const dqrm_tables_t *tables, void *stream);

/* Sec. 3.1 + Sec. 4.1: lookup first, quantise only the gathered rows, sum-pool.
 *   indices [num_indices] int64  table-local row ids, table-major: bags
 *                                t*batch .. t*batch+batch-1 belong to table t
 *   offsets [T*batch+1]   int64  bag i = lookups offsets[i] .. offsets[i+1]-1;
 *                                offsets[0] = 0, offsets[T*batch] = num_indices;
 *                                empty bags are legal (their output is zero)
 *   out     [batch][T][D] fp32   out[b][t] = sum over the bag, in lookup order, of
 *                                w_scale[t] * code
 *   codes_dbg [num_indices][D] int8 or NULL: the INT4 code of every gathered element
 *   mode    DQRM_FWD_MASTER: code = quantise(master row);  DQRM_FWD_PACKED: code =
 *           stored nibble (identical results when `packed` is in sync) */
int32_t dqrm_embbag_fwd(const dqrm_tables_t *tables, const int64_t *indices, const int64_t *offsets,
                        int32_t batch, int64_t num_indices, int32_t mode, float *out, int8_t *codes_dbg,
                        void *stream);

/* Scratch for dqrm_embbag_bwd, in bytes (256-byte aligned device memory; needs
 * no initialisation; its contents mean nothing between calls).  Two calls that
 * may overlap in time need two workspaces.  Returns 0 for invalid arguments. */
size_t dqrm_embbag_bwd_workspace_bytes(int32_t num_tables, int32_t dim, int32_t batch, int64_t num_indices);

/* Sec. 4.3 / distributed-training appendix: the table gradient in sparse
 * (indices, values) form over the touched rows only -- lossless "specified
 * sparsity", coalesced.  The backward of the quantiser is the identity, so the
 * gradient of row r of table t is the sum of grad_out[bag(i)] over the lookups
 * i of table t with indices[i] == r.
 *   grad_out [batch][T][D] fp32        gradient w.r.t. `out` of the forward
 *   sorted_pos [num_indices] int32     lookup positions ordered by (table, row, position)
 *   uniq_rows  [num_indices] int64     first U entries: table-local row of each segment,
 *                                      ascending inside a table, tables in order
 *   seg_offsets [num_indices+1] int32  first U+1 entries: start of each segment in
 *                                      sorted_pos; seg_offsets[U] = num_indices
 *   table_uniq_offsets [T+1] int32     table t's segments are [tuo[t], tuo[t+1])
 *   num_unique [1] int32               U (stays on the device: the following calls read it there)
 *   values [num_indices][D] fp32       first U rows: the summed row gradients (order: DQRM_SEG_CHUNK)
 *   g_absmax [T] fp32                  max |values| over the table's segments, 0 if none
 * Entries past U (U+1) of the capacity-sized outputs are left untouched.
 * Equivalent to dqrm_dedupe followed by dqrm_segment_sum on the same stream. */
int32_t dqrm_embbag_bwd(const dqrm_tables_t *tables, const int64_t *indices, const int64_t *offsets,
                        int32_t batch, int64_t num_indices, const float *grad_out, int32_t *sorted_pos,
                        int64_t *uniq_rows, int32_t *seg_offsets, int32_t *table_uniq_offsets,
                        int32_t *num_unique, float *values, float *g_absmax, void *workspace,
                        size_t workspace_bytes, void *stream);

/* dqrm_embbag_bwd for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, outputs and results as dqrm_embbag_bwd, minus
 * the workspace: the scratch is an array of DQRM_NOALLOC_SCRATCH_BYTES built into
 * the library (one copy per GPU, held until the process ends; its address is
 * looked up at the first call on each device).  Shapes for which
 * dqrm_embbag_bwd_workspace_bytes() exceeds DQRM_NOALLOC_SCRATCH_BYTES are rejected
 * with DQRM_ERR_SCRATCH_LIMIT before anything is launched (the text of
 * dqrm_last_hip_error() then names both sizes); at 26 tables of dim 64 the array
 * holds batches of about 50,000 lookups.  Calls no hipMalloc / hipFree or any
 * other allocating routine.  All calls on one GPU share that GPU's array (it needs
 * no clearing between calls), so two calls that may overlap in time on one GPU,
 * on whatever streams, race: order them. */
#define DQRM_NOALLOC_SCRATCH_BYTES (8u << 20)
int32_t dqrm_embbag_bwd_noalloc(const dqrm_tables_t *tables, const int64_t *indices, const int64_t *offsets,
                                int32_t batch, int64_t num_indices, const float *grad_out, int32_t *sorted_pos,
                                int64_t *uniq_rows, int32_t *seg_offsets, int32_t *table_uniq_offsets,
                                int32_t *num_unique, float *values, float *g_absmax, void *stream);

/* The two halves of dqrm_embbag_bwd, for callers that overlap them with other
 * work.  dqrm_dedupe (the sparse-tensor coalescing of Sec. 4.3: sort the lookups
 * by table, row, position and find the distinct rows) needs only the batch's
 * indices, so it can run on a second stream beside the forward pass, or one
 * step ahead; it writes every index-only output (sorted_pos, uniq_rows,
 * seg_offsets, table_uniq_offsets, num_unique) and leaves the work list of the
 * segment sums in `workspace`.  dqrm_segment_sum then needs that workspace (the
 * caller orders the two, e.g. with an event) and grad_out, and writes `values`
 * and `g_absmax`; it may be repeated on the same dedupe result.  g_absmax may be
 * NULL if dqrm_quant_update follows (see there) or if the maxima are not wanted
 * (the next dqrm_dedupe into the same workspace starts them afresh). */
int32_t dqrm_dedupe(const dqrm_tables_t *tables, const int64_t *indices, const int64_t *offsets, int32_t batch,
                    int64_t num_indices, int32_t *sorted_pos, int64_t *uniq_rows, int32_t *seg_offsets,
                    int32_t *table_uniq_offsets, int32_t *num_unique, void *workspace, size_t workspace_bytes,
                    void *stream);
int32_t dqrm_segment_sum(const dqrm_tables_t *tables, int32_t batch, int64_t num_indices, const float *grad_out,
                         float *values, float *g_absmax, void *workspace, size_t workspace_bytes, void *stream);

/* dqrm_dedupe for up to DQRM_MAX_DEDUPE_BATCHES batches in one launch pair.  A
 * table's sort occupies one CU, so one batch keeps only T CUs busy; the batches
 * of the next few steps (a data loader has their indices long before the model
 * needs them) fill the chip instead.  `batches` is a HOST array; each element
 * holds the arguments dqrm_dedupe takes for one batch (its own outputs and its
 * own workspace of at least `workspace_bytes` bytes, sized for the largest
 * num_indices).  All batches have `batch` bags per table.
 * max_table_lookups: the lookups one table has in a batch are device data (the
 * offsets), so a batch of more than 16384 lookups costs a launch of the pass
 * that serves tables of more than 16384 lookups even when no table is that
 * large.  A caller who knows a bound on the lookups of any one table in this
 * batch (bags per table x the longest bag) states it here and is spared that
 * launch when the bound is at most 16384; 0 = no bound known (what dqrm_dedupe
 * and dqrm_embbag_bwd pass).  A table with more lookups than a stated bound is
 * treated like one beyond DQRM_MAX_TABLE_LOOKUPS: skipped, DQRM_ERR_CAPACITY in
 * dqrm_check_status. */
typedef struct {
    const int64_t *indices;
    const int64_t *offsets;
    int64_t num_indices;
    int32_t *sorted_pos;
    int64_t *uniq_rows;
    int32_t *seg_offsets;
    int32_t *table_uniq_offsets;
    int32_t *num_unique;
    void *workspace;
    int32_t max_table_lookups;
} dqrm_dedupe_batch_t;
int32_t dqrm_dedupe_multi(const dqrm_tables_t *tables, int32_t batch, int32_t num_batches,
                          const dqrm_dedupe_batch_t *batches, size_t workspace_bytes, void *stream);

/* dqrm_segment_sum for up to DQRM_MAX_DEDUPE_BATCHES batches in one launch (the
 * companion of dqrm_dedupe_multi).  The segment sums of a small batch -- a
 * micro-batch of simulated data parallelism (appendix "Simulated Data Parallelism
 * Environment") -- are a chain of dependent memory round trips with little else to
 * do; several side by side cost hardly more than one.  `batches` is a HOST array;
 * each element holds what dqrm_segment_sum takes for one batch (its own workspace,
 * as its dqrm_dedupe left it, of at least `workspace_bytes` bytes; g_absmax may be
 * NULL).  All batches have `batch` bags per table. */
typedef struct {
    int64_t num_indices;
    const float *grad_out; /* [batch][T][D] */
    float *values;
    float *g_absmax;       /* [T] or NULL */
    void *workspace;
} dqrm_segsum_batch_t;
int32_t dqrm_segment_sum_multi(const dqrm_tables_t *tables, int32_t batch, int32_t num_batches,
                               const dqrm_segsum_batch_t *batches, size_t workspace_bytes, void *stream);

/* Distributed-training appendix (only the values of the sparse gradient are
 * quantised; the indices are left alone): one scale per table per step,
 * g_scale[t] = max(g_absmax[t] / 127, 1e-8); gq = clamp(round_half_even(values /
 * g_scale[t]), -128, 127).  `capacity` = rows allocated in values / gq (>= U). */
int32_t dqrm_grad_quant_int8(int32_t num_tables, int32_t dim, int64_t capacity, const float *values,
                             const int32_t *table_uniq_offsets, const float *g_absmax, int8_t *gq,
                             float *g_scale, void *stream);

/* dqrm_grad_quant_int8 for up to DQRM_MAX_DEDUPE_BATCHES blocks of values in one
 * launch (`blocks` is a HOST array of that call's arguments).  The blocks may name
 * the same g_absmax: the micro-batches of one group of simulated data parallelism
 * are all quantised with the first one's scale. */
typedef struct {
    int64_t capacity;
    const float *values;
    const int32_t *table_uniq_offsets;
    const float *g_absmax;
    int8_t *gq;
    float *g_scale;
} dqrm_quant_block_t;
int32_t dqrm_grad_quant_int8_multi(int32_t num_tables, int32_t dim, int32_t num_blocks,
                                   const dqrm_quant_block_t *blocks, void *stream);

/* Same appendix (dequantise, then the local parameter update): for every
 * segment u of table t, master[row] -= lr * (g_scale[t] * gq[u]) (two
 * roundings); if tables->packed is not NULL the row's nibbles are re-encoded
 * from the new master row with the cached w_scale[t]. */
int32_t dqrm_sparse_update(const dqrm_tables_t *tables, int64_t capacity, const int64_t *uniq_rows,
                           const int32_t *table_uniq_offsets, const int8_t *gq, const float *g_scale,
                           float lr, void *stream);

/* Simulated data parallelism on one device (appendix "Simulated Data Parallelism
 * Environment": the gradients of `simulated_nodes` micro-batches are added into a
 * buffer, then the weights are updated once) and, equally, the sum of the integer
 * gradients that the all-reduce of the distributed-training appendix delivers.
 * A block is one micro-batch's sparse gradient after dqrm_grad_quant_int8 (the
 * appendix reuses the scale of the group's first micro-batch for the others: pass
 * that micro-batch's g_absmax to every dqrm_grad_quant_int8 call of the group).
 * The "buffer" is kept sparse: dqrm_sparse_merge returns the union of the blocks'
 * rows, table by table in ascending row order, and the 32-bit integer sums of
 * their INT8 codes (exact: no order matters); dqrm_sparse_update_sums is
 * dqrm_sparse_update for such sums, master[row] -= lr * (g_scale[t] * (float)sum)
 * (two roundings; nothing is divided by the number of blocks).
 *   blocks     HOST array of num_blocks (<= DQRM_MAX_DEDUPE_BATCHES) descriptors of
 *              device arrays: uniq_rows [U_k] int64 table-local, ascending and
 *              distinct inside each table; table_uniq_offsets [T+1] int32; gq
 *              [U_k][D] int8 (4-byte aligned); capacity = rows allocated (>= U_k)
 *   max_total  rows allocated in the outputs uniq_rows [max_total] / sums
 *              [max_total][D] (16-byte aligned); must be >= the sum of the U_k
 *   outputs    uniq_rows, table_uniq_offsets [T+1], num_unique [1], sums; rows
 *              past num_unique are not written
 * Blocks that break these rules are reported through dqrm_check_status
 * (DQRM_ERR_BAD_OFFSETS: offsets that do not start at 0, go backwards or pass the
 * capacity - the whole block then contributes nothing - or rows that are not
 * ascending - the sums of the rows concerned are then unspecified;
 * DQRM_ERR_CAPACITY: the outputs cannot hold the blocks' rows, the rest is left
 * out); every access stays in bounds.  The workspace (256-byte aligned, no
 * initialisation needed) is the library's scratch; the caller owns everything. */
typedef struct {
    const int64_t *uniq_rows;
    const int32_t *table_uniq_offsets;
    const int8_t *gq;
    int64_t capacity;
} dqrm_sparse_block_t;
size_t dqrm_sparse_merge_workspace_bytes(int32_t num_tables, int32_t dim, int32_t num_blocks, int64_t max_total);
int32_t dqrm_sparse_merge(const dqrm_tables_t *tables, int32_t num_blocks, const dqrm_sparse_block_t *blocks,
                          int64_t max_total, int64_t *uniq_rows, int32_t *table_uniq_offsets, int32_t *num_unique,
                          int32_t *sums, void *workspace, size_t workspace_bytes, void *stream);
int32_t dqrm_sparse_update_sums(const dqrm_tables_t *tables, int64_t capacity, const int64_t *uniq_rows,
                                const int32_t *table_uniq_offsets, const int32_t *sums, const float *g_scale,
                                float lr, void *stream);

/* B4 and B5 in one pass, for callers that do not exchange anything between the
 * two (one GPU): same outputs as dqrm_grad_quant_int8 followed by
 * dqrm_sparse_update -- gq, g_scale, the updated master rows and packed nibbles
 * -- and it also writes g_absmax.  It is called after a dqrm_segment_sum that
 * was given g_absmax = NULL (which then skips its last small kernel and leaves
 * the per-table maxima in `workspace`; in that mode dqrm_segment_sum may run
 * only once per dqrm_dedupe).  `workspace` / `num_indices` as for dqrm_dedupe. */
int32_t dqrm_quant_update(const dqrm_tables_t *tables, int64_t capacity, int64_t num_indices, const float *values,
                          const int64_t *uniq_rows, const int32_t *table_uniq_offsets, float *g_absmax, int8_t *gq,
                          float *g_scale, float lr, void *workspace, size_t workspace_bytes, void *stream);

/* The dense part of the DLRM train step (model-architecture table; Fig. 1(a)):
 * bottom MLP over the dense features (ReLU after every layer), pairwise-dot
 * interaction of its output with the T pooled embeddings, top MLP (ReLU after
 * every layer but the last), sigmoid, mean binary cross-entropy against the
 * labels; then the backward of all of it and a plain SGD step on the MLP weights
 * and biases, in FP32 (the paper's "MLP in FP32" variant).  The matrix products
 * run on the matrix cores.
 *   Interaction: vectors Z = [bottom output, table 0 .. T-1] (V = T+1, width dim);
 *   R[b] = [Z[0] (dim values), dot(Z[i], Z[j]) for i = 1..V-1, j = 0..i-1, row-major],
 *   so the top MLP's input width is dim + V(V-1)/2 (367 for 26 tables of dim 16).
 *   Loss: -mean(y log max(p,1e-12) + (1-y) log max(1-p,1e-12)), p = sigmoid(logit).
 * The descriptor and its arrays are HOST memory; W_l is a device matrix
 * [dims[l+1]][dims[l]] row-major, b_l a device vector [dims[l+1]]; both are
 * updated in place.  Limits: T + 1 <= 64, (T+1)*dim <= 4096, at most 16 layers
 * per MLP.
 *   dense_x [batch][num_dense], emb_out [batch][T][dim] (= `out` of
 *   dqrm_embbag_fwd), labels [batch] (0 or 1, as floats)  -> loss [1] (device),
 *   grad_emb [batch][T][dim] (= `grad_out` of dqrm_embbag_bwd). */
typedef struct {
    int32_t num_dense;         /* dense features per sample (13) */
    int32_t num_tables;        /* T */
    int32_t dim;               /* embedding width = bottom MLP output width */
    int32_t bot_layers;        /* number of linear layers of the bottom MLP */
    const int32_t *bot_dims;   /* HOST [bot_layers+1], bot_dims[0] = num_dense, last = dim */
    float *const *bot_w;       /* HOST array of device pointers */
    float *const *bot_b;
    int32_t top_layers;
    const int32_t *top_dims;   /* HOST [top_layers+1], top_dims[0] = dim + V(V-1)/2, last = 1 */
    float *const *top_w;
    float *const *top_b;
} dqrm_dense_model_t;
size_t dqrm_dense_workspace_bytes(const dqrm_dense_model_t *model, int32_t batch);
int32_t dqrm_dense_step(const dqrm_dense_model_t *model, int32_t batch, const float *dense_x, const float *emb_out,
                        const float *labels, float lr, float *loss, float *grad_emb, void *workspace,
                        size_t workspace_bytes, void *stream);

/* The quantised variants of the dense part.
 *   weight_bits = 4 (or 8): every linear layer's weights are fake-quantised channel-wise for the forward and
 *     the input gradients -- one scale per output row, s_o = max(max_i |W[o][i]| / (2^(bits-1)-1), 1e-8),
 *     Wq = s_o * clamp(rint(W / s_o)) -- while the step goes to the FP32 weights (straight-through);
 *     biases and activations stay FP32 (model-quantisation appendix: "a scale for every row inside the
 *     linear layer weights"; whole-model results section).  weight_bits = 0: FP32 weights.
 *   grad_bits = 8: the gradient of every parameter tensor (each layer's weight matrix and each bias vector
 *     on its own) is quantised to INT8 with one scale per tensor before the step, with error compensation
 *     when grad_error is given (distributed-training section: INT8 gradients, compensation for the MLP
 *     layers only; gradient-quantisation appendix).  The paper only cites the compensation scheme; the
 *     reading taken is error feedback:  g' = g + e;  s = max(max|g'| / 127, 1e-8);
 *     code = clamp(rint(g' / s), -128, 127);  e <- g' - s * code;  parameter <- parameter - lr * (s * code).
 *     On one GPU the "unified" scale is the local one.  grad_bits = 0: FP32 gradients.
 * Flat parameter order of grad_error / grad_codes / grads: the layers of the top MLP (0 .. top_layers-1), then
 * those of the bottom MLP; layer l contributes out * (in + 1) values, row-major [out][in + 1], column `in`
 * being the bias.  dqrm_dense_param_count returns the total P.  Tensor order of grad_scale: two per layer in
 * the same layer order, weights then bias.  wq: the layers' quantised weights in the same layer order,
 * [out][in] each (P - sum of out values in total).
 * All pointers are DEVICE memory owned by the caller; the descriptor itself is HOST memory. */
typedef struct {
    int32_t weight_bits; /* 0, 4 or 8 */
    int32_t grad_bits;   /* 0 or 8 */
    float *grad_error;   /* [P] in/out: residuals carried from step to step (zero them before the first step);
                            NULL: INT8 gradients without compensation */
    float *grad_scale;   /* [2 * (top_layers + bot_layers)] out; required when grad_bits = 8 */
    int8_t *grad_codes;  /* [P] out, or NULL: the INT8 codes (what a data-parallel run would exchange) */
    float *grads;        /* [P] out, or NULL: this step's FP32 gradients before compensation */
    float *wq;           /* out, or NULL: the fake-quantised weights this step used */
    /* Simulated data parallelism for the MLPs (appendix "Simulated Data Parallelism Environment": a gradient
     * buffer per parameter collects the micro-batches of a group, then the parameters are updated once);
     * grad_bits = 0 only.  With grad_buffer set, the call adds this micro-batch's gradient to the buffer
     * (buffer_add != 0) or starts the buffer with it (buffer_add = 0: the first micro-batch of a group, which is
     * how the buffer is "cleared"), and the parameters either stay as they are (buffer_update = 0) or take
     * parameter <- parameter - lr * buffer (buffer_update != 0: the group's last micro-batch). */
    float *grad_buffer;  /* [P] in/out, flat parameter order, or NULL: a plain step */
    int32_t buffer_add;
    int32_t buffer_update;
} dqrm_dense_quant_t;
int64_t dqrm_dense_param_count(const dqrm_dense_model_t *model); /* P, or -1 for an invalid descriptor */
/* As dqrm_dense_step; `quant` may be NULL (then it IS dqrm_dense_step).  Same workspace. */
int32_t dqrm_dense_step_quant(const dqrm_dense_model_t *model, const dqrm_dense_quant_t *quant, int32_t batch,
                              const float *dense_x, const float *emb_out, const float *labels, float lr, float *loss,
                              float *grad_emb, void *workspace, size_t workspace_bytes, void *stream);

/* Synchronises `stream`, returns the first data-dependent problem recorded on
 * the current device since the last call (DQRM_OK if none) and clears it.
 * first_bad_table / first_bad_index (host pointers, may be NULL) receive the
 * table and the offending value (index value, lookup count or bag number). */
int32_t dqrm_check_status(void *stream, int32_t *first_bad_table, int64_t *first_bad_index);

/* Text of the last HIP error seen by this thread's DQRM calls ("" if none). */
const char *dqrm_last_hip_error(void);

/* Library version, "major.minor". */
const char *dqrm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DQRM_H */
