/*
 * som.h - C ABI of libsom: batch-mode self-organizing-map training on one AMD MI355X (gfx950).
 *
 * The library implements the data-parallel hot path of the batch SOM the paper describes
 * (section "Self-organizing maps in batch mode"): one training epoch = best-matching-unit
 * search + batch code-book update, plus cooling schedules and the U-matrix.  The paper's
 * own entry point is the single function `trainOneEpoch` (section "As an application
 * programming interface"); the calls below split it into an init call that fixes the map
 * geometry, one-epoch calls for dense and sparse data, a whole-schedule call, and the
 * U-matrix.
 *
 * Conventions shared by every call
 *   - Every array pointer is a DEVICE pointer to memory the CALLER owns (for instance a
 *     torch tensor's data_ptr()); the library borrows it for the duration of the call's
 *     work on the stream and never frees it.  The library owns only the scratch memory
 *     inside `som_ctx`, which it allocates with hipMalloc and grows on demand.
 *   - All work is enqueued on the HIP stream given to som_init (NULL = the default
 *     stream) and is asynchronous: outputs are valid once that stream has been
 *     synchronised.  No call synchronises unless its description says so, with one
 *     exception: a call that has to grow the context's scratch (more instances, or more
 *     nonzeros, than any call before it on this context) waits for the stream first, because
 *     work already enqueued may still use the old buffers.
 *   - Node index i = y * cols + x, x = column in 0..cols-1, y = row in 0..rows-1
 *     (options -x/-y of the paper's command line).  The code book is node-major
 *     [rows*cols][dim], fp32, as in the paper's API (`float *codebook`).
 *   - Every call returns a status (SOM_OK = 0).  On SOM_ERR_INVALID_ARG nothing has been
 *     written or enqueued.  som_last_error gives a human-readable message.
 *   - A context is used by one host thread at a time.
 */
#ifndef SOM_H
#define SOM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct som_ctx som_ctx;

enum { SOM_OK = 0, SOM_ERR_INVALID_ARG = 1, SOM_ERR_ALLOC = 2, SOM_ERR_DEVICE = 3, SOM_ERR_STATE = 4 };
enum { SOM_MAP_PLANAR = 0, SOM_MAP_TOROID = 1 };          /* option -m: planar (default) or toroid   */
enum { SOM_GRID_SQUARE = 0, SOM_GRID_HEXAGONAL = 1 };     /* option -g: square (default) or hexagonal */
enum { SOM_COOL_AS_RADIUS = -1, SOM_COOL_LINEAR = 0, SOM_COOL_EXPONENTIAL = 1 };   /* options -t / -T */
enum { SOM_FILTER_FP32 = 0, SOM_FILTER_SPLIT_F16 = 1, SOM_FILTER_TWO_LEVEL = 2, SOM_FILTER_AUTO = 3 };   /* see som_set_filter */
enum { SOM_NEIGHBORHOOD_GAUSSIAN = 0, SOM_NEIGHBORHOOD_BUBBLE = 1 };   /* option -n               */
enum { SOM_SMOOTH_AUTO = 0, SOM_SMOOTH_VECTOR = 1, SOM_SMOOTH_MATRIX = 2, SOM_SMOOTH_MATRIX_SPLIT = 3 };   /* see som_set_smoothing */

/* Neighbourhood mass below which a node keeps its weights (see som_train_epoch_dense). */
#define SOM_EPS_MASS 1e-20

/*
 * som_init - create a context for a rows x cols map over dim-dimensional data.
 * (Paper: options -x, -y, -g, -m, -c; without an initial code book the map starts from random values.)
 *   out        host pointer that receives the context.
 *   codebook   device [rows*cols][dim] fp32.  seed == 0: left as the caller filled it
 *              (option -c, initial code book).  seed != 0: overwritten with uniform [0,1)
 *              values drawn from a counter-based generator keyed by (seed, element index).
 *   hip_stream hipStream_t cast to void*, or NULL for the default stream.
 * Errors: rows, cols or dim < 1, rows*cols > 2^24, unknown enum, NULL pointers ->
 * SOM_ERR_INVALID_ARG; scratch allocation failure -> SOM_ERR_ALLOC.
 */
int som_init(som_ctx **out, int rows, int cols, int dim, int map_type, int grid_type,
             float *codebook, uint64_t seed, void *hip_stream);

/* Release the context and its scratch memory (synchronises the stream first). */
void som_destroy(som_ctx *ctx);

/* Message of the last failing call on ctx; ctx == NULL: of the last failing call that takes no
 * context (som_init, som_bmu_distances_dense_static). */
const char *som_last_error(const som_ctx *ctx);

/*
 * som_train_epoch_dense - one epoch on dense data.
 * (Paper: BMU equation; batch equation; neighbourhood equation read as
 *  h = exp(-d^2 / (2 radius^2)) with d the grid distance between two nodes.)
 *   data      device [n][dim] fp32, row-major (the paper's `float *data`), read only.
 *   codebook  device [rows*cols][dim] fp32, in: current weights, out: updated weights.
 *   radius    > 0, neighbourhood radius of this epoch (already cooled).
 *   scale     learning rate of this epoch, 0 < scale <= 1.  It multiplies numerator and
 *             denominator of the batch equation alike and therefore has no effect on the
 *             result; it is validated and otherwise ignored.
 *   bmus      device [n] int32 out: for each instance the node nearest (Euclidean) to it
 *             in the INCOMING code book; exact ties go to the lowest node index.
 * Update: w_i <- sum_j h(bmu_j, i) x_j / sum_j h(bmu_j, i); a node whose denominator is
 * below SOM_EPS_MASS keeps its weights.  Square grid: unit spacing.  Hexagonal grid: odd
 * rows shifted right by half a cell, row pitch sqrt(3)/2.  Toroid: distances wrap in both
 * directions (a hexagonal torus is seamless only for an even number of rows).
 * Errors: NULL pointer, n < 1, n >= 2^31, radius <= 0 or not finite, scale outside (0,1]
 * -> SOM_ERR_INVALID_ARG; scratch growth failure -> SOM_ERR_ALLOC; launch failure ->
 * SOM_ERR_DEVICE.
 */
int som_train_epoch_dense(som_ctx *ctx, const float *data, int64_t n, float *codebook,
                          float radius, float scale, int32_t *bmus);

/*
 * som_train_epoch_csr - the same epoch on sparse rows in CSR form.
 * (Paper: sparse kernel; sparse file format with zero-based index:value pairs.)
 *   indptr    device [n+1] int64, indptr[0] = 0, non-decreasing, indptr[n] = nnz.
 *   indices   device [nnz] int32, zero-based column indices in 0..dim-1, strictly
 *             increasing within a row.
 *   values    device [nnz] fp32.
 * Unlisted coordinates are zero; an empty row is legal (its BMU is the node of smallest
 * norm).  The code book stays dense.  The epoch and search calls do not check the CSR
 * structure: rows that violate the contract give undefined results (indices are still clamped
 * so that no access leaves the code book); som_validate_csr checks it on request.  Other
 * arguments, outputs and errors as for the dense call;
 * nnz < 0 or nnz >= 2^31 -> SOM_ERR_INVALID_ARG.
 * The per-node sums of this call are accumulated with fp32 atomic adds, so the last bits
 * of the new code book may vary from run to run; the BMUs do not.
 * Scratch of the sparse search, allocated with the first sparse call on the context: a
 * transposed code book of 2 bytes per weight, and, if it takes no more than 16 GiB, a
 * transposed fp32 copy (4 bytes per weight) for the instances that have to be compared with
 * every node exactly.
 */
int som_train_epoch_csr(som_ctx *ctx, const int64_t *indptr, const int32_t *indices,
                        const float *values, int64_t n, int64_t nnz, float *codebook,
                        float radius, float scale, int32_t *bmus);

/*
 * som_validate_csr - debug pass over a CSR data set (paper: sparse file format, zero-based
 * index:value pairs).  Checks indptr[0] = 0, indptr non-decreasing, indptr[n] = nnz, every column
 * index in [0, dim) and strictly increasing within its row.  Arguments as in som_train_epoch_csr.
 * Synchronises the stream.  Returns SOM_OK, or SOM_ERR_INVALID_ARG with the kind of violation in
 * som_last_error (a row whose bounds leave [0, nnz] is reported, not read).
 */
int som_validate_csr(som_ctx *ctx, const int64_t *indptr, const int32_t *indices, const float *values,
                     int64_t n, int64_t nnz);

/*
 * som_bmus_dense / som_bmus_csr - BMU search only (BMU equation), code book unchanged:
 * the mapping of data onto a trained map.  Arguments as in the epoch calls.
 * Non-finite input is not an error: an instance with a NaN or infinite component has no
 * finite distance to any node and is mapped to node 0, as a plain scan with a strict
 * comparison gives; a node with such a component is never chosen.  (In an epoch call such an
 * instance then enters the sums of node 0 and the non-finite values spread through the
 * update, as the batch equation says.)
 */
int som_bmus_dense(som_ctx *ctx, const float *data, int64_t n, const float *codebook, int32_t *bmus);
int som_bmus_csr(som_ctx *ctx, const int64_t *indptr, const int32_t *indices, const float *values,
                 int64_t n, int64_t nnz, const float *codebook, int32_t *bmus);

/*
 * som_update_dense / som_update_csr - the batch update alone (batch equation) for given
 * BMUs: per-node sums of the instances, neighbourhood smoothing over the map, division.
 *   bmus  device [n] int32, each in 0..rows*cols-1, read only (values outside that range
 *         give undefined results but no out-of-bounds access: they are clamped).
 * Other arguments as in the epoch calls.
 */
int som_update_dense(som_ctx *ctx, const float *data, int64_t n, const int32_t *bmus,
                     float *codebook, float radius, float scale);
int som_update_csr(som_ctx *ctx, const int64_t *indptr, const int32_t *indices, const float *values,
                   int64_t n, int64_t nnz, const int32_t *bmus, float *codebook,
                   float radius, float scale);

/*
 * som_set_data_dense / som_set_data_csr - register the training set som_train works on.
 * The pointers are borrowed until the next som_set_data_* or som_destroy; the data must
 * stay unchanged meanwhile.  Arguments as in the epoch calls.
 * Per-instance quantities that depend on the data alone (squared norms, the centring vector
 * of the dense search) are computed once per registration, on first use.  The epoch and
 * BMU calls reuse them when they are handed the registered pointer(s) and n; on any other
 * data they recompute them on every call.
 */
int som_set_data_dense(som_ctx *ctx, const float *data, int64_t n);
int som_set_data_csr(som_ctx *ctx, const int64_t *indptr, const int32_t *indices,
                     const float *values, int64_t n, int64_t nnz);

/*
 * som_train - n_epochs epochs on the registered data with cooled radius and scale, all
 * enqueued without any host synchronisation; the schedule is evaluated on the device.
 * (Paper: options -e, -r/-R, -l/-L, -t/-T.)
 *   Epoch e = 0..n_epochs-1 uses v_e = v0 + (vN - v0) e / (n_epochs-1) (linear) or
 *   v_e = v0 (vN / v0)^(e / (n_epochs-1)) (exponential); one epoch uses v0.
 *   radius0 <= 0: default, half the smaller map side (at least 1); radiusN <= 0: 1.
 *   scale0 <= 0: 1.0; scaleN <= 0: 0.01 (the paper's defaults).
 *   cooling   SOM_COOL_LINEAR or SOM_COOL_EXPONENTIAL for the radius (option -t), and for the
 *             learning rate too unless som_set_scale_cooling chose another kind for it (option -T).
 *   codebook  device, in/out as in the epoch calls.
 *   bmus      device [n] int32 out: BMUs found in the LAST epoch (against the code book
 *             that entered it).
 * Errors: no data registered -> SOM_ERR_STATE; n_epochs < 1 or bad enum -> SOM_ERR_INVALID_ARG.
 */
int som_train(som_ctx *ctx, int n_epochs, float radius0, float radiusN, float scale0,
              float scaleN, int cooling, float *codebook, int32_t *bmus);

/*
 * som_train_snapshots - som_train with the interim outputs of option -s.
 *   snapshots 0: none (exactly som_train; the three pointers below are ignored).
 *             1: the U-matrix of the code book after every epoch.
 *             2: also the code book after every epoch and the BMUs that epoch found.
 *   umatrices  device [n_epochs][rows][cols] fp32 out (snapshots >= 1).
 *   codebooks  device [n_epochs][rows*cols][dim] fp32 out (snapshots == 2).
 *   bmus_all   device [n_epochs][n] int32 out (snapshots == 2), n = registered instances.
 * Everything is written on the context's stream in epoch order; the caller owns the buffers
 * (for large maps `codebooks` is the big one: n_epochs code books).  Other arguments, defaults
 * and errors as in som_train; a missing buffer or snapshots outside 0..2 -> SOM_ERR_INVALID_ARG.
 */
int som_train_snapshots(som_ctx *ctx, int n_epochs, float radius0, float radiusN, float scale0,
                        float scaleN, int cooling, float *codebook, int32_t *bmus, int snapshots,
                        float *umatrices, float *codebooks, int32_t *bmus_all);

/*
 * som_bmu_distances_dense / som_bmu_distances_csr - post-training output: how far every
 * instance lies from the node it is mapped to.  (The paper lists the BMUs, the code book and
 * the U-matrix as results and prints no formula for a quality figure; this is the usual
 * quantisation error.)
 *   data / indptr, indices, values, n, nnz   as in the epoch calls, read only.
 *   codebook   device [rows*cols][dim] fp32, read only.
 *   bmus       device [n] int32, read only: node of every instance, normally from som_bmus_*
 *              against the same code book.  An index outside [0, rows*cols) gives NaN for that
 *              instance and for the mean.
 *   distances  device [n] fp32 out, or NULL: Euclidean distance ||x_j - w_bmus[j]||, summed in
 *              fp64 and rounded once.
 *   qerror     device [1] fp64 out, or NULL: the mean of the (unrounded) distances; the order
 *              of the additions is fixed, so equal inputs give equal bits.
 * At least one of the two outputs must be given.  Nothing is allocated.
 */
int som_bmu_distances_dense(som_ctx *ctx, const float *data, int64_t n, const float *codebook,
                            const int32_t *bmus, float *distances, double *qerror);
int som_bmu_distances_csr(som_ctx *ctx, const int64_t *indptr, const int32_t *indices,
                          const float *values, int64_t n, int64_t nnz, const float *codebook,
                          const int32_t *bmus, float *distances, double *qerror);

/*
 * som_bmu_distances_dense_static - som_bmu_distances_dense for callers that cannot allocate device
 * memory or create a context at the point of the call: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  It takes no context and calls no allocating routine;
 * its only scratch (one fp64 partial sum per workgroup, 1,024 of them = 8 KB) is a fixed array in
 * the library's device image, which every GPU the library is used on holds until the process ends.
 *   data       device [n][dim] fp32, read only.
 *   codebook   device [n_nodes][dim] fp32, read only.
 *   bmus, distances, qerror   as in som_bmu_distances_dense (same kernels, same bits).
 *   hip_stream hipStream_t cast to void*, or NULL for the default stream; the work is enqueued
 *              there, asynchronously.
 * The scratch never limits n (the instances are dealt to at most 1,024 workgroups), so the size
 * limits are those of the other calls: n outside [1, 2^31), dim < 1, n_nodes outside [1, 2^24],
 * n_nodes * dim >= 2^40, a NULL input or both outputs NULL -> SOM_ERR_INVALID_ARG, nothing
 * enqueued (message: som_last_error(NULL)).
 * All calls on one GPU share that GPU's array: two calls whose work may overlap on the same GPU
 * (different streams, or different threads) race on it and must be ordered by the caller; calls
 * on one stream are ordered already.  Nothing has to be cleared between calls: a call overwrites
 * every partial sum it later reads.  The array's address is looked up once per device, by som_init
 * or else by the first call of this function on that device; make that first call outside a
 * graph capture.
 */
int som_bmu_distances_dense_static(const float *data, int64_t n, int dim, const float *codebook, int n_nodes,
                                   const int32_t *bmus, float *distances, double *qerror, void *hip_stream);

/*
 * som_cool_schedule - evaluate the cooling schedule of som_train on the device.
 *   radius_out, scale_out  device [n_epochs] fp64 out (either may be NULL).
 * Defaults and formulas as in som_train.
 */
int som_cool_schedule(som_ctx *ctx, int n_epochs, float radius0, float radiusN, float scale0,
                      float scaleN, int cooling, double *radius_out, double *scale_out);

/*
 * som_set_scale_cooling - cooling kind of the learning rate (option -T) where it differs from the
 * radius' (option -t): SOM_COOL_LINEAR, SOM_COOL_EXPONENTIAL, or SOM_COOL_AS_RADIUS (default) =
 * whatever kind som_train / som_train_snapshots / som_cool_schedule are given for the radius.  The
 * learning rate cancels in the batch equation, so this changes what som_cool_schedule reports, not the
 * code book.  Errors: unknown value -> SOM_ERR_INVALID_ARG.
 */
int som_set_scale_cooling(som_ctx *ctx, int cooling);

/*
 * som_umatrix - U-matrix of a code book (U-matrix equation): for every node the mean
 * Euclidean distance between its weight vector and those of its immediate neighbours
 * (grid distance <= 1: up to 4 on a square grid, up to 6 on a hexagonal one; fewer on the
 * border of a planar map; a node without neighbours gets 0).
 *   codebook  device [rows*cols][dim] fp32, read only.
 *   umatrix   device [rows][cols] fp32 out.
 */
int som_umatrix(som_ctx *ctx, const float *codebook, float *umatrix);

/*
 * som_set_neighborhood - neighbourhood function of the batch update (options -n and -p; the
 * paper's trainOneEpoch carries them as `gaussian` and `compact_support`).
 *   function         SOM_NEIGHBORHOOD_GAUSSIAN (default): exp(-d^2 / (2 r^2)) of the grid distance
 *                    d and the epoch's radius r; SOM_NEIGHBORHOOD_BUBBLE: 1 for d <= r, else 0.
 *   compact_support  non-zero: the Gaussian is cut off to 0 beyond d > r (the bubble always is).
 * The default (Gaussian, no cut-off) factorises over the two grid directions and is applied in
 * two passes; the others use a one-pass kernel over a table of weights.  Takes effect from the
 * next update on.  Errors: unknown function -> SOM_ERR_INVALID_ARG; table allocation ->
 * SOM_ERR_ALLOC.
 */
int som_set_neighborhood(som_ctx *ctx, int function, int compact_support);

/*
 * som_set_sparse_hot_block - whether a REGISTERED sparse training set may be split into a dense block of
 * its 256 most frequent columns, multiplied with the code book on the matrix cores, and a sparse rest
 * (paper: sparse kernel).  On by default; the split is used only when those columns hold at least 30 % of
 * the nonzeros, dim >= 1,024 and the table of partial sums (4 bytes per instance and node) stays under
 * 8 GiB.  The BMUs do not depend on it (the exact stage decides on the caller's full rows).  It is
 * prepared at the first epoch or search after registration, which waits for the stream once, and costs
 * about 1 KB of device memory per instance plus a copy of the remaining nonzeros.
 */
int som_set_sparse_hot_block(som_ctx *ctx, int enable);

/* 1 if the registered sparse set has been examined and its hot-column block is in use, else 0. */
int som_sparse_hot_block_active(const som_ctx *ctx);

/*
 * som_set_sparse_dense_filter - whether the BMU search over a REGISTERED sparse training set of modest
 * dimension may run the DENSE filter pass (som_set_filter) on fp16 planes of the centred rows instead of
 * the gather sweep (paper: sparse kernel; its comparison of sparse and dense runs on the same 5 % dense
 * data).  A centred sparse row is dense anyway, and the matrix cores do n x nodes x dim multiply-adds
 * faster than the vector units do nnz x nodes when the rows are short and well filled.  On by default;
 * used when dim <= 4,096, at least 4 % of the entries are nonzero and the filter is not SOM_FILTER_FP32.
 * The exact stage and the update keep working on the caller's sparse rows, so BMUs and code book do not
 * depend on it.  Prepared at the first epoch or search after registration; costs 4 to 6 bytes of device
 * memory per entry of the dense matrix.
 */
int som_set_sparse_dense_filter(som_ctx *ctx, int enable);

/* 1 if the registered sparse set has been examined and is searched through dense planes, else 0. */
int som_sparse_dense_filter_active(const som_ctx *ctx);

/*
 * som_set_smoothing - which units run the two passes of the Gaussian neighbourhood smoothing (batch
 * equation; neighbourhood equation).  The result is the same up to the order of the fp32 additions.
 *   SOM_SMOOTH_AUTO (default)  a pass over map lines of at least 32 nodes runs as a matrix product on
 *                  the matrix cores, a shorter one on the vector units; from 96 nodes on the product
 *                  runs on the bf16 matrix cores with every fp32 operand carried as three bf16 parts
 *                  (six part products, fp32 accumulation: what is dropped is below 2^-23 of a term),
 *                  below that on the fp32 ones;
 *   SOM_SMOOTH_VECTOR  always the vector units;  SOM_SMOOTH_MATRIX  the fp32 matrix cores for any line
 *                  length;  SOM_SMOOTH_MATRIX_SPLIT  the bf16 ones with three-part operands for any
 *                  line length (maps with a side above 1,024 nodes always use the vector units).
 * Errors: unknown value -> SOM_ERR_INVALID_ARG.
 */
int som_set_smoothing(som_ctx *ctx, int form);

/*
 * som_set_filter - choose the arithmetic of the dense BMU filter pass (paper, "Parallelism":
 * the GPU variant obtains the distances through linear algebra).  The result of a BMU search
 * does not depend on it: every filter only shortlists nodes within a proven rounding bound,
 * and exact fp64 distances decide.
 *   SOM_FILTER_SPLIT_F16  every fp32 operand is split into two fp16 numbers and the
 *                  dot products run as three fp16 matrix instructions with fp32 accumulation:
 *                  fp32-grade scores at several times the fp32 matrix rate; needs 4 bytes per
 *                  element of extra device memory for instances and code book.
 *   SOM_FILTER_TWO_LEVEL  a coarse pass with ONE fp16 product per feature (the hi halves alone) finds, per
 *                  instance and block of 128 nodes, the smallest coarse score; the blocks that cannot
 *                  hold the BMU by the proven bound of those scores are dropped, the instances are
 *                  ordered by their best block, and the split-fp16 pass runs over the remaining
 *                  (128 instances, block) pairs only.  Needs 6 bytes per element of extra device memory
 *                  and 4 bytes per instance and node block.
 *   SOM_FILTER_AUTO (default)  SOM_FILTER_TWO_LEVEL for maps of 1,024 nodes or more whose table of
 *                  block minima (4 bytes x instances x nodes / 128) stays under 8 GiB, else
 *                  SOM_FILTER_SPLIT_F16.
 *   SOM_FILTER_FP32  fp32 matrix instructions on the operands as they are.
 * Errors: unknown value -> SOM_ERR_INVALID_ARG.
 */
int som_set_filter(som_ctx *ctx, int filter);

/*
 * som_debug_scores_dense / som_debug_scores_csr - test hooks (not operations of the paper): run the
 * filter pass of the BMU search (the dense one selected by som_set_filter, or the sparse sweep) on
 * the given data against codebook and write EVERY score, not just the candidates:
 *   scores[j * rows*cols + i] = c_i - 2 x_j . w'_i as the filter computed it, w' = fl(w - mu),
 *   c_i = |w'_i|^2 + 2 mu . w'_i  (the sparse sweep multiplies with a 16-bit quantisation of w');
 *   mu_out [dim]    the centring vector mu that was used;
 *   margin_out [n]  fp64: the margin the exact stage applies to instance j - two scores of j whose
 *                   difference exceeds it are taken as decided - evaluated by the same device
 *                   function on the same inputs.  It is meant to cover the error of both scores.
 * All pointers are device pointers; scores must hold n * rows*cols floats.  A test compares the
 * scores with their exact values and checks that no error exceeds half the margin.
 * Errors: NULL pointers, n / nnz out of range -> SOM_ERR_INVALID_ARG.
 */
int som_debug_scores_dense(som_ctx *ctx, const float *data, int64_t n, const float *codebook, float *scores,
                           float *mu_out, double *margin_out);
int som_debug_scores_csr(som_ctx *ctx, const int64_t *indptr, const int32_t *indices, const float *values,
                         int64_t n, int64_t nnz, const float *codebook, float *scores, float *mu_out,
                         double *margin_out);

/*
 * som_debug_mfma_f16 - test hook (not an operation of the paper): `count` independent
 * executions of the 32x32x16 fp16 matrix instruction, D = A B^T + C with A [32][16] and
 * B [32][16] given as fp16 bit patterns, C and D [32][32] fp32, problem t at offsets 512 t
 * (A, B) and 1024 t (C, D); device pointers.  Lets a test check the rounding behaviour that
 * the split-fp16 filter's error bound assumes of the instruction.
 */
int som_debug_mfma_f16(const uint16_t *a, const uint16_t *b, const float *c_in, float *d_out, int count,
                       void *hip_stream);

/*
 * som_debug_xcc_ids - test hook (not an operation of the paper): launches n_blocks one-wavefront
 * workgroups and writes the id of the XCD (accelerator complex) each of them ran on to out[0..n_blocks)
 * (device pointer).  The dense filter and the sparse sweep put workgroups that share operands 8 apart
 * in a launch, expecting consecutive workgroups to be dealt round-robin to the eight XCDs so that those
 * land on one L2; only speed depends on it, and a test checks it through this call.
 */
int som_debug_xcc_ids(int32_t *out, int n_blocks, void *hip_stream);

/*
 * som_get_stats - counters of the most recent BMU search on ctx (synchronises the stream).
 *   rows_refined   instances whose fp32 scores left two to four candidate nodes, decided by
 *                  the exact fp64 distances of those candidates;
 *   rows_collected instances with more candidates than that: a second fp32 sweep listed all
 *                  nodes under the instance's threshold, then exact distances decided
 *                  (dense data only);
 *   rows_rescanned instances that needed an exact fp64 scan of all nodes.
 * out is a HOST pointer to three int64 values, in that order.
 */
int som_get_stats(som_ctx *ctx, int64_t *out);

/*
 * som_two_level_stats - how selective the coarse pass of the most recent dense BMU search on ctx was
 * (see som_set_filter, SOM_FILTER_TWO_LEVEL; synchronises the stream).  out is a HOST pointer to two
 * int64 values: the (tile of 128 instances, block of 128 nodes) pairs the second pass worked on, and all
 * such pairs.  Both are 0 when that search ran in one level (or no dense search has run yet).
 */
int som_two_level_stats(som_ctx *ctx, int64_t *out);

/*
 * som_profile_enable / som_profile_read - measurement support (not an operation of the paper).
 * While enabled, the library brackets the stages of every epoch with HIP events recorded on
 * the context's stream, so a benchmark can report per-stage device time without a profiler:
 *   stage 0  dense BMU filter pass (one MFMA kernel launch per epoch)
 *   stage 1  sparse BMU filter pass (transpose + CSR kernel)
 *   stage 2  exact BMU stage (certify, candidate collection, refine, rescan)
 *   stage 3  per-node sums (sort by BMU, chunk sums / sparse scatter)
 *   stage 4  neighbourhood smoothing and division
 *   stage 5  preparation of the dense filter pass (centring vector and norms of unregistered
 *            data, centred code book, fp16 planes)
 * som_profile_read synchronises the stream, adds up the elapsed time of all brackets recorded
 * since the last read, stores milliseconds in total_ms[0..5] and bracket counts in
 * launches[0..5] (HOST pointers), and clears the record.  At most 512 brackets per stage are
 * kept between two reads; further ones are not recorded.
 */
#define SOM_PROFILE_STAGES 6
int som_profile_enable(som_ctx *ctx, int on);
int som_profile_read(som_ctx *ctx, double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* SOM_H */
