// Internal declarations shared by the translation units of libsom (gfx950 only).
// Nothing here is part of the C ABI; see include/som.h for that.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "som.h"

namespace som {

// ---------------------------------------------------------------- constants
constexpr int kWave = 64;                 // CDNA wavefront width
constexpr int kCand = 4;                  // candidate nodes kept per instance by the fp32 pass
constexpr int kListCap = 256;             // nodes a collected candidate list can hold per instance
constexpr int kChunkRows = 32;            // instances summed by one block of the segmented accumulation
// Stable radix sort of n keys below key_range (segsum.hip): passes of at most 8 bits, the bits spread evenly over
// the passes (12 bits: two passes of 6, not 8 + 4 - the table of digit counts per tile, which one workgroup has to
// scan, shrinks with the digit), and tiles of `tile` keys, one wavefront each.  The scan takes a step per 4,096
// table entries, the scatter a step per 64 keys of a tile, and the two cost about the same per step: the number
// of tiles that balances them is 8 sqrt(n / bins).
struct RadixPlan {
  int passes, digit_bits, tile, nblk;
};
inline RadixPlan radix_plan_for_digits(int64_t n, int passes, int digit_bits) {
  RadixPlan p;
  p.passes = passes;
  p.digit_bits = digit_bits;
  const double bins = (double)(1 << digit_bits);
  int64_t want = (int64_t)(8.0 * __builtin_sqrt((double)(n < 1 ? 1 : n) / bins));
  if (want < 64) want = 64;
  int64_t tile = ((n + want - 1) / want + 63) / 64 * 64;
  if (tile < 64) tile = 64;
  p.tile = (int)tile;
  p.nblk = (int)((n + tile - 1) / tile);
  if (p.nblk < 1) p.nblk = 1;
  return p;
}
inline RadixPlan radix_plan(int64_t n, int key_range) {
  int bits = 1;
  while ((1ll << bits) < (long long)key_range) ++bits;
  const int passes = (bits + 7) / 8;
  return radix_plan_for_digits(n, passes, (bits + passes - 1) / passes);
}
// Entries of the digit-count table that serve any number of keys up to n and any key range: a plan never has
// more tiles than the number it aims for (at least 64), and that number grows with the key count.
inline size_t radix_table_entries(int64_t n) {
  size_t most = 0;
  for (int db = 1; db <= 8; ++db) {
    const double bins = (double)(1 << db);
    double want = 8.0 * __builtin_sqrt((double)(n < 1 ? 1 : n) / bins);
    if (want < 64.0) want = 64.0;
    const size_t e = ((size_t)1 << db) * ((size_t)want + 2);
    if (e > most) most = e;
  }
  return most + 1;
}
constexpr int kSmoothMatMax = 1024;        // largest map side for which the smoothing filters are stored as matrices
constexpr int kSmoothMfmaMin = 32;         // shortest map line whose smoothing pass runs on the matrix cores by default
constexpr int kSmoothSplitMin = 96;        // ... and on the bf16 ones with three-part operands
constexpr int kCsrDenseMaxDim = 4096;      // registered sparse sets up to this many columns may be searched through dense planes
constexpr double kCsrDenseMinDensity = 0.04;   // ... if at least this share of their entries is nonzero
constexpr int kHot = 256;                  // columns of the dense hot block of a registered sparse training set
constexpr double kHotMinShare = 0.3;       // share of the nonzeros those columns must hold for the split to be used
constexpr int kProfMax = 512;              // event brackets kept per stage between two reads
#ifndef SOM_FLUSH_BLOCK
#define SOM_FLUSH_BLOCK 32
#endif
constexpr int kDenseAccumBlock = SOM_FLUSH_BLOCK;      // k-extent after which the fp32 MFMA accumulator is flushed

// Scores the fp32 pass hands to the exact pass: per instance kCand (value, node) pairs,
// smallest first where the producer sorts them, plus the smallest value it dropped.
struct CandView {
  float *val;      // [n][kCand]
  int32_t *idx;    // [n][kCand], -1 = empty slot
  float *over;     // [n] smallest score not kept (+inf if none)
};

// Epoch parameters produced on the device by the cooling kernel.
struct EpochParams {
  double radius;
  double scale;
  double inv8r2;   // 1 / (8 radius^2)
};

}  // namespace som

// ---------------------------------------------------------------- context
struct som_ctx {
  int rows, cols, dim, k;
  int map_type, grid_type;
  hipStream_t stream;
  int n_cu;

  // per-map scratch (allocated in som_init)
  float *wn32;            // [k rounded up to 128] node constants c_i of the BMU filters, fp32; +inf past k
  double *wn64;           // [k] the same in fp64
  unsigned *wmax_bits;    // [2] bit patterns of max_i |w'_i|^2 and of the largest |w'| element (non-negative floats order like uints)
  int32_t *counts;        // [k] instances per BMU
  int32_t *seg_off;       // [k+1] exclusive scan of counts
  int32_t *chunk_off;     // [k+1] exclusive scan of chunks per node
  double *massD;          // [k] neighbourhood mass per node
  double *dist_partial;   // [1024] per-workgroup sums of the distances to the BMUs
  uint64_t *row_hash;     // [k] hashes of the code-book rows (bubble neighbourhood only, lazily allocated)
  uint64_t *dedup_keys;   // [dedup_slots] open-addressing table of those hashes
  int32_t *dedup_lowest;  // [dedup_slots] lowest node index per key
  int dedup_slots;        // power of two >= 2 k
  double *cntT;           // [2][k] count channel after the pass along x
  float *gx;              // [2*cols+1] neighbourhood factor along x, index = twice the x offset
  float *gy;              // [rows] neighbourhood factor along y
  float *GxT, *GyT;       // the two filters as transposed coefficient matrices (maps with sides <= kSmoothMatMax)
  int xi_pad, e_pad;      // padded output extents of GxT / GyT (multiples of 32)
  int smooth_mfma_min;    // a smoothing pass over lines of at least this many nodes runs on the matrix cores (0: never)
  int smooth_split_min;   // ... and from this many nodes on with bf16 operands in three parts (0: never)
  int32_t *hit_x, *hit_n; // [k] columns of the chosen nodes per map row, [rows] their number
  int32_t *hit_rows;      // [rows+1] map rows with chosen nodes, last entry = their number
  int nb_function;        // SOM_NEIGHBORHOOD_*
  int nb_compact;         // Gaussian cut off at the current radius
  int scale_cooling;      // SOM_COOL_* of the learning rate, or -1: the kind the call gives for the radius
  float *H2;              // neighbourhood weights by (parity class, row distance, column offset), lazily allocated
  som::EpochParams *params;   // [1]
  float *S;               // [k][dim] per-node sums
  float *T;               // [1 or 2][k][dim] sums after the pass along x
  float *Wt;              // [dim][kpad] centred transposed code book of the sparse BMU search, int16 multiples
                          // of the column steps (lazily allocated)
  int kpad;               // 512 * csr_acc * csr_sweeps >= k
  float *Wt32;            // [dim][kt32] transposed fp32 copy of the code book for the sparse full rescan (allocated with
  int64_t kt32;           // the first sparse search if it fits kRescanCopyMax; written only in searches that rescan)
  int Wt32_tried;
  int csr_acc, csr_sweeps;    // sparse BMU kernel: scores per lane and sweep, sweeps per node slice
  float *col_range;       // [2][64][dim] slab minima and maxima of the code-book columns (with Wt)
  float *qstep;           // [dim] quantisation step of every column of Wt (with Wt)
  double *ct_partial;     // [kCtMaxSlabs][k][3] row sums per column slab of the fused centring / transpose pass (with Wt)
  unsigned *qstep_max_bits;   // [1] bit pattern of the largest step
  float *Wc;              // [k][dim] centred code book w' = fl(w - mu) of the dense BMU search (lazily allocated)
  _Float16 *Wh;           // [k][ceil(dim/32)][64] centred code book as fp16 hi/lo planes (lazily allocated)
  _Float16 *Wh1;          // [k][ceil(dim/64)][64] its hi halves alone (two-level search)
  float *wscale;          // [1] the power of two the centred code book was divided by
  int filter;             // SOM_FILTER_*: which matrix format the dense BMU filter runs on
  float *zero16;          // 64 bytes of zeros: source of out-of-range direct-to-LDS loads
  float *mu_norm2;        // [1] |mu|^2
  float *mu;              // [dim] centring vector of the dense BMU search
  double *mu_partial;     // [64][dim] partial column sums

  // per-data scratch (grown on demand to n_cap rows)
  int64_t n_cap;
  float *xn32;            // [n] squared norms of the instances (split-fp16 filter: of the centred instances x - mu)
  float *vq;              // [vq_cap] sparse search: value of every nonzero times the step of its column
  int64_t vq_cap;
  float *row_q;           // [n] sparse rows: sum over the nonzeros of |value| x quantisation step of the column
  _Float16 *Xh;           // [n][ceil(dim/32)][64] dense instances as fp16 hi/lo planes (lazily allocated)
  float *xscale;          // [n] the power of two each instance was divided by
  // two-level dense search (bmu_two_level.hip), lazily allocated with Xh
  _Float16 *Xh1;          // [n][ceil(dim/64)][64] the hi halves alone
  float *coarse_min;      // [ceil(k/128)][n] smallest coarse score per node block and instance
  int32_t *coarse_key;    // [n] sort key of every instance: size class of its block set, lowest block of the set
  uint32_t *coarse_mask;  // [ceil(blocks/32)][n] node blocks an instance's BMU may lie in
  int32_t *tile_cnt;      // [ceil(n/128)] node blocks listed per instance tile of the sorted order
  int32_t *tile_list;     // [ceil(n/128)][ceil(k/128)] those blocks, ascending
  int32_t *ctile_cnt, *ctile_list;   // the same for the tiles of collect_rows (second sweep of the exact stage)
  int64_t two_level_n;    // instances of the most recent dense search if it ran in two levels, else 0
  int64_t cand_cap;       // instance slots in the three candidate arrays (node groups x instances)
  float *cand_val;        // [groups][n][kCand]
  int32_t *cand_idx;      // [groups][n][kCand]
  float *cand_over;       // [groups][n]
  int32_t *cand_n;        // [n] number of candidates to evaluate exactly
  int32_t *refine_list;   // [n] instances with 2..kCand candidates
  int32_t *collect_rows;  // [n] instances whose candidates have to be collected by a second sweep
  float *collect_thr;     // [n] their score thresholds (indexed by slot in collect_rows)
  int32_t *collect_cnt;   // [n] nodes found under the threshold
  int32_t *collect_list;  // [n][kListCap] those nodes (dense path only, lazily allocated)
  int32_t *rescan_list;   // [n] instances that need an exact scan of all nodes
  int32_t *list_counts;   // [0..2] lengths of refine_list, collect_rows, rescan_list; [3] flag of som_validate_csr;
                          // [4..11] lengths of unit_work per slice; behind these kListCounts words the
                          // list comparison's entry counters, kListTicketStride words apart
  int64_t *unit_work;     // [8][unit_cap] sparse search: (collect slot, node range) units to sweep again
  int64_t unit_cap;
  int32_t *sort_key[2];   // [n] each
  int32_t *sort_val[2];   // [n] each
  int32_t *radix_hist;    // [bins * sort tiles], radix_table_entries(n_cap)
  int32_t *chunk_node;    // [n/kChunkRows + k]
  float *partial;         // [n/kChunkRows + k][dim]
  int64_t max_chunks;

  // hot-column split of the registered sparse training set (csr_hot.hip); built on first use
  int hot_valid;          // 0: not examined yet; 1: examined (hot_on says whether the split is in use)
  int hot_on;
  int hot_enabled;        // som_set_sparse_hot_block
  int64_t hot_n_cap, hot_nnz_cap;
  int32_t *hot_counts;    // [dim] nonzeros per column
  int32_t *hot_rank;      // [dim] position of a column in the hot block, or -1
  int32_t *hot_cols;      // [kHot] the hot columns, ascending
  int32_t *tail_start;    // [n+1] nonzeros of the rows outside the hot columns, then their exclusive scan
  int64_t *tail_indptr;   // [n+1] the tail as a CSR set of its own
  int32_t *tail_indices;  // [tail nonzeros]
  float *tail_values;
  int64_t tail_nnz;
  _Float16 *hot_Xh;       // [n][kHot/32][64] hot part of the instances as fp16 hi/lo planes
  float *hot_xscale;      // [n] their power-of-two scales
  float *hot_xn;          // [n] |x_hot|^2
  float *hot_Wc;          // [k][kHot] hot columns of the centred code book
  _Float16 *hot_Wh;       // [k][kHot/32][64] the same as planes
  float *hot_wscale;      // [1]
  unsigned *hot_wmax_bits;    // [1]
  float *hot_P;           // [ceil(k/128)][n][128] dot products of the hot parts divided by the instance scale

  // dense planes of the registered sparse training set (som_set_sparse_dense_filter); built on first use
  int csrd_valid;         // 0: not examined yet; 1: examined (csrd_on says whether the planes are in use)
  int csrd_on;
  int csrd_enabled;
  float *csrd_mu;         // [dim] column means of the sparse set: the centring vector of its planes
  float *csrd_mu_norm2;   // [1]
  float *csrd_xn;         // [n] squared norms of the centred rows
  int64_t csrd_n_cap;

  // registered training set for som_train
  int data_kind;          // 0 none, 1 dense, 2 csr
  const float *d_data;
  const int64_t *d_indptr;
  const int32_t *d_indices;
  const float *d_values;
  int64_t d_n, d_nnz;
  int d_norms_valid;      // xn32 (and mu for dense data) currently describe the registered set
  int d_split_valid;      // Xh / xscale currently describe the registered dense set

  // optional per-stage event brackets (som_profile_enable)
  int prof_on;
  int prof_used[SOM_PROFILE_STAGES];
  hipEvent_t *prof_ev[SOM_PROFILE_STAGES];   // 2 * kProfMax events each, created on first enable

  char err[256];
};

namespace som {

// Every launcher enqueues on ctx->stream and returns hipGetLastError().

// norms.hip
hipError_t launch_sample_col_means(som_ctx *c, const float *A, int64_t nrows, int dim, float *mu);
hipError_t launch_codebook_means_and_steps(som_ctx *c, const float *W);      // -> mu, qstep, qstep_max_bits
hipError_t launch_vec_sqnorm(som_ctx *c, const float *v, int dim, float *out);
hipError_t launch_center_codebook(som_ctx *c, const float *W, bool store_centered, bool want_wn64,
                                  bool x_centered);   // -> Wc, wn32 (= c_i; without the 2 mu.w' term if the instances are centred too), wmax_bits, wn64
hipError_t launch_row_sqnorms(som_ctx *c, const float *A, int64_t nrows, int dim, const float *mu,
                              float *out32, double *out64, unsigned *max_bits);
hipError_t launch_csr_row_sqnorms(som_ctx *c, const int64_t *indptr, const float *values, int64_t n,
                                  float *out32);

// bmu_dense.hip
int bmu_dense_groups(const som_ctx *c, int64_t n);
hipError_t launch_bmu_dense(som_ctx *c, const float *X, int64_t n, float *dump);   // dump: test hook, all scores [n][k], or null
hipError_t launch_bmu_dense_collect(som_ctx *c, const float *X, int64_t n);
hipError_t launch_bmu_dense_dl(som_ctx *c, const float *X, int64_t n, dim3 grid, bool collect, float *dump);   // bmu_dense_dl.hip

// bmu_dense_h.hip, split_f16.hip
// Chunks of 32 features a wavefront of the split-fp16 pass multiplies into its MFMA accumulators
// before it adds them to the running totals (a power of two; the margin prices the chain length).
// Longer chains save additions and widen the margin: measured, four chunks pay from 256 features on.
inline int split_flush_chunks(int dim) { return dim >= 256 ? 4 : 2; }
// Two-level search (bmu_two_level.hip): by default from this many node blocks of 128 on, and only
// while its table of block minima stays under this many bytes.
constexpr int kTwoLevelMinBlocks = 8;
constexpr int64_t kTwoLevelMaxTable = 8ll << 30;
int bmu_dense_h_groups(const som_ctx *c, int64_t n);
hipError_t launch_bmu_dense_h(som_ctx *c, int64_t n, float *dump);            // Xh, Wh -> candidates (or all scores)
int bmu_dense_h_fine_groups(const som_ctx *c, int64_t n);
hipError_t launch_bmu_coarse(som_ctx *c, int64_t n, float *dump);              // bmu_coarse.hip: Xh1, Wh1 -> coarse_min (or all scores)
hipError_t launch_bmu_dense_h_fine(som_ctx *c, int64_t n);                     // sort_val[0], tile_cnt, tile_list -> candidates
// bmu_two_level.hip
hipError_t launch_select_blocks(som_ctx *c, int64_t n);                        // coarse_min -> coarse_key, coarse_mask
int two_level_key_range(int blocks);                                           // keys of coarse_key are below this
hipError_t launch_tile_lists(som_ctx *c, int64_t n);                           // coarse_mask, sort_val[0] -> tile_cnt, tile_list
hipError_t launch_collect_tile_lists(som_ctx *c, int64_t n);                   // coarse_mask, collect_rows -> ctile_cnt, ctile_list
hipError_t launch_bmu_dense_h_collect(som_ctx *c, int64_t n, bool lists = false);   // rows of collect_rows -> collect_list
hipError_t launch_split_rows_f16(som_ctx *c, const float *A, int64_t nrows, const unsigned *global_max_bits,
                                 const float *mu /* subtracted first, or null */, _Float16 *out, float *scale_out,
                                 int dim = 0 /* row length; 0: the context's */,
                                 _Float16 *out_hi = nullptr /* the hi halves alone, rows padded to 64 columns */);
hipError_t launch_probe_mfma_f16(hipStream_t stream, const uint16_t *A, const uint16_t *B, const float *C, float *D,
                                 int count);

// bmu_exact.hip
// Work list of the sparse search's second sweep: per node slice, entries slot * sweeps + range.
struct UnitWork {
  int sweeps;             // 0: not a sparse search, every collected instance is swept whole
  int64_t cap;            // entries per slice
  int64_t *units;         // [8][cap]
  int32_t *counts;        // [8]
  int32_t *list;          // [slots][kListCap] candidate lists, seeded with the nodes of the complete ranges
};
constexpr size_t kRescanCopyMax = (size_t)16 << 30;      // bytes: no transposed copy for the full rescan beyond this
constexpr int kListCounts = 16;    // words of lengths and flags at the head of som_ctx::list_counts
constexpr int kListTickets = 8;    // entry counters of the list comparison behind them ...
constexpr int kListTicketStride = 1088;      // ... 4 KB + 256 B apart: another memory channel each
constexpr int kListWords = kListCounts + kListTickets * kListTicketStride;
constexpr int kUnitCounts = 4;     // first of the eight work-list lengths in it
enum { kCertifyFp32 = 0, kCertifySplit = 1, kCertifyCsr = 2, kCertifyCoarse = 3 };      // whose rounding bound the margin uses
hipError_t launch_certify(som_ctx *c, int64_t n, int groups, int mode, const int64_t *indptr, int32_t *bmus,
                          bool hot = false, const int32_t *order = nullptr /* visit the instances in this order */);
hipError_t launch_margins(som_ctx *c, int64_t n, int mode, const int64_t *indptr, double *out,
                          bool hot = false);   // test hook: the margin per instance
hipError_t launch_refine_dense(som_ctx *c, const float *X, const float *W, int32_t *bmus);
hipError_t launch_refine_lists_dense(som_ctx *c, const float *X, const float *W, int32_t *bmus);
hipError_t launch_rescan_dense(som_ctx *c, const float *X, const float *W, int32_t *bmus);
hipError_t launch_refine_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices,
                             const float *values, const float *W, int32_t *bmus);
hipError_t launch_refine_lists_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices,
                                   const float *values, const float *W, int32_t *bmus);
hipError_t launch_rescan_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices,
                             const float *values, const float *W, int32_t *bmus);

// Workgroups of the distance kernel = partial sums it leaves (and the capacity of every buffer for them).
constexpr int kDistBlocks = 1024;
hipError_t launch_bmu_distances_on(hipStream_t stream, const float *X, const int64_t *indptr, const int32_t *indices,
                                   const float *values, int64_t n, const float *W, int k, int dim,
                                   const int32_t *bmus, float *dist, double *qerror,
                                   double *partial /* [kDistBlocks] device scratch */);
hipError_t launch_bmu_distances(som_ctx *c, const float *X, const int64_t *indptr, const int32_t *indices,
                                const float *values, int64_t n, const float *W, const int32_t *bmus, float *dist,
                                double *qerror);     // X != NULL: dense rows, else CSR

// csr_hot.hip
hipError_t launch_csr_col_sums(som_ctx *c, const int32_t *indices, const float *values, int64_t nnz, float *sums);
hipError_t launch_csr_densify(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                              int64_t row0, int64_t nrows, float *out /* [nrows][dim] */);
hipError_t launch_scale_vector(som_ctx *c, float *v, int len, float factor);
hipError_t launch_hot_histogram(som_ctx *c, const int32_t *indices, int64_t nnz, int32_t *counts);
hipError_t launch_tail_lengths(som_ctx *c, const int64_t *indptr, const int32_t *indices, int64_t n, int32_t *len);
hipError_t launch_split_hot_tail(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                                 int64_t n);
hipError_t launch_gather_hot_codebook(som_ctx *c, const float *W);   // -> hot_Wc, hot_wmax_bits
hipError_t launch_hot_partial(som_ctx *c, int64_t n);                // bmu_dense_h.hip: hot_Xh, hot_Wh -> hot_P
hipError_t launch_scan_exclusive_i32(som_ctx *c, const int32_t *in, int32_t *out, int len);   // segsum.hip

// dedup.hip
hipError_t launch_mask_duplicate_rows(som_ctx *c, const float *W);   // wn32[i] = +inf for rows equal to a lower-indexed row

// bmu_csr.hip
constexpr int kCtMaxSlabs = 64;            // column slabs of the fused centring / transpose pass
hipError_t launch_center_transpose_codebook(som_ctx *c, const float *W);   // mu, qstep -> Wt, wn32, wn64, wmax_bits
void csr_slice_geometry(int k, int *acc, int *sweeps, int *kpad);
hipError_t launch_scale_values(som_ctx *c, const int32_t *indices, const float *values, int64_t nnz);   // -> vq
enum { kCsrBadSorted = 1, kCsrBadIndex = 2, kCsrBadOrder = 3, kCsrBadLast = 4, kCsrBadFirst = 5 };   // k_validate_csr: the largest is reported
hipError_t launch_validate_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, int64_t n, int64_t nnz,
                               int32_t *flag);
hipError_t launch_bmu_csr_sliced(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                                 int64_t n, bool collect, float *dump = nullptr,   // dump: test hook, all scores [n][k]
                                 bool hot = false);   // the rows are the tail of the registered set: sums start from hot_P

// segsum.hip
hipError_t launch_sort_by_bmu(som_ctx *c, const int32_t *bmus, int64_t n);   // -> sort_val[0] = row ids
hipError_t launch_sort_keys(som_ctx *c, const int32_t *keys, int64_t n, int key_range);   // the permutation alone
hipError_t launch_accumulate_dense(som_ctx *c, const float *X, int64_t n);   // -> S, counts
hipError_t launch_accumulate_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices,
                                 const float *values, int64_t n, const int32_t *bmus);   // -> S, counts

// smooth.hip
hipError_t launch_epoch_params(som_ctx *c, int epoch, int n_epochs, double r0, double rN, double s0,
                               double sN, int cooling);
hipError_t launch_cool_schedule(som_ctx *c, int n_epochs, double r0, double rN, double s0, double sN,
                                int cooling, double *radius_out, double *scale_out);
hipError_t launch_smooth_and_divide(som_ctx *c, float *W);

// umatrix.hip
hipError_t launch_umatrix(som_ctx *c, const float *W, float *U);

// init.hip
hipError_t launch_fill_uniform(som_ctx *c, float *W, int64_t count, uint64_t seed);
hipError_t launch_fill_zero_u32(hipStream_t s, void *p, int64_t count_u32);
hipError_t launch_probe_xcc(hipStream_t stream, int32_t *out, int n_blocks);

// ---------------------------------------------------------------- device helpers
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Grid geometry: q = 4 x squared grid distance between nodes (xi, yi) and (xb, yb).
// Hexagonal rows of odd y are shifted right by half a cell, row pitch sqrt(3)/2.
__device__ __forceinline__ long long grid_q(int rows, int cols, int toroid, int hex, int xi, int yi,
                                            int xb, int yb) {
  long long a = yi > yb ? yi - yb : yb - yi;
  long long m = 2ll * (xi - xb) + (hex ? ((yi & 1) - (yb & 1)) : 0);
  if (m < 0) m = -m;
  if (toroid) {
    if (rows - a < a) a = rows - a;
    if (2ll * cols - m < m) m = 2ll * cols - m;
  }
  return m * m + (hex ? 3 : 4) * a * a;
}

}  // namespace som
