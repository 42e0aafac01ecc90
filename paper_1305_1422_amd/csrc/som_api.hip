// C ABI of libsom: argument validation, scratch management and the order in which the kernels
// of one epoch are enqueued.  See include/som.h for the contract of every entry point.
//
// One epoch (paper: "Self-organizing maps in batch mode"; API section, trainOneEpoch):
//   node norms and centring -> BMU filter pass (split-fp16 or fp32 MFMA, or the CSR sweep) ->
//   certify / exact refine / second sweep with exact comparison of the collected lists / exact
//   rescan -> stable sort by BMU, chunked per-node sums -> neighbourhood smoothing (two passes
//   for the Gaussian, one over a weight table for the others) with the division fused in.
// The stream is synchronised only where scratch has to grow (the old buffers may still be in
// use), by som_destroy, som_get_stats and som_profile_read.
#include "som_internal.hpp"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <vector>

using namespace som;

static char g_init_error[256] = "";

// Scratch of the entry point that must not allocate (som_bmu_distances_dense_static): one partial sum per
// workgroup of the distance kernel.  Every GPU the library runs on holds its own copy of this array
// for the life of the process, at its own address; the name below is only a host-side handle of the
// symbol, so host code resolves the address once per device and passes that pointer to the kernels.
static __device__ __align__(256) double scratch[kDistBlocks];      // 8 KB
constexpr int kMaxDevices = 64;
static double *g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Address of `scratch` on the current device (resolved on first use, then cached); null on failure.
static double *static_scratch(hipError_t *err) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
  double *p = nullptr;
  if (e == hipSuccess) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void *sym = nullptr;
      e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
      if (e == hipSuccess) g_scratch_ptr[dev] = static_cast<double *>(sym);
    }
    p = g_scratch_ptr[dev];
  }
  if (err) *err = e;
  return e == hipSuccess ? p : nullptr;
}

static int fail(som_ctx *c, int code, const char *fmt, ...) {
  char *dst = c ? c->err : g_init_error;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 256, fmt, ap);
  va_end(ap);
  return code;
}

static int dev_fail(som_ctx *c, hipError_t e, const char *what) {
  return fail(c, SOM_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

#define SOM_LAUNCH(ctx, expr)                                   \
  do {                                                          \
    hipError_t e_ = (expr);                                     \
    if (e_ != hipSuccess) return dev_fail((ctx), e_, #expr);    \
  } while (0)

template <typename T>
static bool dev_alloc(T **p, size_t count) {
  *p = nullptr;
  if (count == 0) count = 1;
  return hipMalloc((void **)p, count * sizeof(T)) == hipSuccess;
}

template <typename T>
static void dev_free(T *&p) {
  if (p) (void)hipFree((void *)p);
  p = nullptr;
}

// The dense filter runs on fp16 planes (one-level split pass or the two-level search).
static bool uses_planes(const som_ctx *c) { return c->filter != SOM_FILTER_FP32; }

// Two-level search for n instances?  Asked for outright, or by default when the map has enough node
// blocks for the coarse pass to leave most of them out; never when its table of block minima would
// not be a modest share of the device memory.
static bool two_level(const som_ctx *c, int64_t n) {
  if (c->filter != SOM_FILTER_TWO_LEVEL && c->filter != SOM_FILTER_AUTO) return false;
  const int64_t blocks = (c->k + 127) / 128;
  if (c->filter == SOM_FILTER_AUTO && blocks < kTwoLevelMinBlocks) return false;
  return blocks * n * 4 <= kTwoLevelMaxTable;
}

// ... and its scratch is there (ensure_rows sizes it for the largest row count seen, whose table may not fit
// when that of a smaller n would: then the one-level pass serves)
static bool two_level_ready(const som_ctx *c, int64_t n) {
  return two_level(c, n) && c->Xh1 != nullptr && c->Wh1 != nullptr && n <= c->n_cap;
}

static void free_row_scratch(som_ctx *c) {
  dev_free(c->xn32); dev_free(c->row_q); dev_free(c->cand_val); dev_free(c->cand_idx); dev_free(c->cand_over);
  dev_free(c->cand_n); dev_free(c->refine_list); dev_free(c->rescan_list);
  dev_free(c->collect_rows); dev_free(c->collect_thr); dev_free(c->collect_cnt); dev_free(c->collect_list);
  dev_free(c->sort_key[0]); dev_free(c->sort_key[1]); dev_free(c->sort_val[0]); dev_free(c->sort_val[1]);
  dev_free(c->radix_hist); dev_free(c->chunk_node); dev_free(c->partial);
  dev_free(c->Xh); dev_free(c->xscale);
  dev_free(c->Xh1); dev_free(c->coarse_min); dev_free(c->coarse_key); dev_free(c->coarse_mask);
  dev_free(c->tile_cnt); dev_free(c->tile_list); dev_free(c->ctile_cnt); dev_free(c->ctile_list);
  c->two_level_n = 0;
  c->n_cap = 0;
  c->cand_cap = 0;
  c->d_norms_valid = 0;
  c->d_split_valid = 0;
  c->csrd_valid = 0;
  c->csrd_on = 0;
}

// Scratch that scales with the number of instances; grown (never shrunk) on demand.
static int ensure_rows(som_ctx *c, int64_t n, bool dense) {
  const bool split = dense && uses_planes(c);
  // sized for the rows the scratch is (or will be) allocated for, so that it serves every n up to n_cap
  const bool coarse = split && two_level(c, n > c->n_cap ? n : c->n_cap);
  const bool need_partial = (dense && (c->partial == nullptr || c->Wc == nullptr)) || c->collect_list == nullptr ||
                            (split && (c->Xh == nullptr || c->Wh == nullptr)) ||
                            (coarse && (c->Xh1 == nullptr || c->Wh1 == nullptr));
  if (n <= c->n_cap && !need_partial) return SOM_OK;
  if (n > c->n_cap) {
    (void)hipStreamSynchronize(c->stream);
    free_row_scratch(c);
    const size_t N = (size_t)n;
    bool ok = dev_alloc(&c->xn32, N) && dev_alloc(&c->row_q, N) && dev_alloc(&c->cand_val, N * kCand) && dev_alloc(&c->cand_idx, N * kCand) &&
              dev_alloc(&c->cand_over, N) && dev_alloc(&c->cand_n, N) && dev_alloc(&c->refine_list, N) &&
              dev_alloc(&c->rescan_list, N) && dev_alloc(&c->collect_rows, N) && dev_alloc(&c->collect_thr, N) &&
              dev_alloc(&c->collect_cnt, N) && dev_alloc(&c->sort_key[0], N) && dev_alloc(&c->sort_key[1], N) &&
              dev_alloc(&c->sort_val[0], N) && dev_alloc(&c->sort_val[1], N) &&
              dev_alloc(&c->radix_hist, radix_table_entries(n));
    c->max_chunks = (int64_t)(N / kChunkRows) + c->k;
    ok = ok && dev_alloc(&c->chunk_node, (size_t)c->max_chunks);
    if (!ok) {
      free_row_scratch(c);
      return fail(c, SOM_ERR_ALLOC, "cannot allocate scratch for %lld instances", (long long)n);
    }
    c->n_cap = n;
    c->cand_cap = n;
  }
  if (dense && c->partial == nullptr) {
    if (!dev_alloc(&c->partial, (size_t)c->max_chunks * c->dim))
      return fail(c, SOM_ERR_ALLOC, "cannot allocate %lld x %d partial sums", (long long)c->max_chunks, c->dim);
  }
  if (c->collect_list == nullptr) {
    if (!dev_alloc(&c->collect_list, (size_t)c->n_cap * kListCap))
      return fail(c, SOM_ERR_ALLOC, "cannot allocate candidate lists for %lld instances", (long long)c->n_cap);
  }
  if (dense && c->Wc == nullptr) {
    if (!dev_alloc(&c->Wc, (size_t)c->k * c->dim))
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the centred code book (%d x %d)", c->k, c->dim);
  }
  if (split) {
    const size_t row_halves = (size_t)((c->dim + 31) / 32) * 64;
    if (c->Wh == nullptr && !dev_alloc(&c->Wh, (size_t)c->k * row_halves))
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the fp16 planes of the code book");
    if (c->Xh == nullptr) {
      c->d_split_valid = 0;
      c->csrd_valid = 0;
      if (!(dev_alloc(&c->Xh, (size_t)c->n_cap * row_halves) && dev_alloc(&c->xscale, (size_t)c->n_cap)))
        return fail(c, SOM_ERR_ALLOC, "cannot allocate the fp16 planes of %lld instances", (long long)c->n_cap);
    }
  }
  if (coarse) {
    const size_t row_halves = (size_t)((c->dim + 63) / 64) * 64;
    const size_t blocks = (size_t)(c->k + 127) / 128, tiles = ((size_t)c->n_cap + 127) / 128;
    if (c->Wh1 == nullptr && !dev_alloc(&c->Wh1, (size_t)c->k * row_halves))
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the fp16 plane of the code book");
    if (c->Xh1 == nullptr) {
      c->d_split_valid = 0;
      c->csrd_valid = 0;
      if (!(dev_alloc(&c->Xh1, (size_t)c->n_cap * row_halves) && dev_alloc(&c->coarse_min, blocks * (size_t)c->n_cap) &&
            dev_alloc(&c->coarse_key, (size_t)c->n_cap) && dev_alloc(&c->coarse_mask, (blocks + 31) / 32 * (size_t)c->n_cap) &&
            dev_alloc(&c->tile_cnt, tiles) && dev_alloc(&c->tile_list, tiles * blocks) &&
            dev_alloc(&c->ctile_cnt, tiles) && dev_alloc(&c->ctile_list, tiles * blocks))) {
        dev_free(c->Xh1); dev_free(c->coarse_min); dev_free(c->coarse_key); dev_free(c->coarse_mask);
        dev_free(c->tile_cnt); dev_free(c->tile_list); dev_free(c->ctile_cnt); dev_free(c->ctile_list);
        return fail(c, SOM_ERR_ALLOC, "cannot allocate the two-level search's scratch for %lld instances", (long long)c->n_cap);
      }
    }
  }
  return SOM_OK;
}

// The dense fp32 pass writes one candidate list per node group and instance.
static int ensure_candidates(som_ctx *c, int64_t n, bool dense) {
  int groups_h = dense && uses_planes(c) ? bmu_dense_h_groups(c, n) : 1;
  if (dense && two_level_ready(c, n) && bmu_dense_h_fine_groups(c, n) > groups_h) groups_h = bmu_dense_h_fine_groups(c, n);
  const int groups_f = dense ? bmu_dense_groups(c, n) : 8 * c->csr_sweeps;      // sparse: one list per node range
  const int64_t need = (int64_t)(groups_h > groups_f ? groups_h : groups_f) * n;
  if (!dense && n * c->csr_sweeps > c->unit_cap) {
    (void)hipStreamSynchronize(c->stream);
    dev_free(c->unit_work);
    c->unit_work = nullptr;
    c->unit_cap = 0;
    if (!dev_alloc(&c->unit_work, (size_t)8 * n * c->csr_sweeps))
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the work list of the sparse search");
    c->unit_cap = n * c->csr_sweeps;
  }
  if (need <= c->cand_cap) return SOM_OK;
  (void)hipStreamSynchronize(c->stream);
  dev_free(c->cand_val); dev_free(c->cand_idx); dev_free(c->cand_over);
  c->cand_cap = 0;
  if (!(dev_alloc(&c->cand_val, (size_t)need * kCand) && dev_alloc(&c->cand_idx, (size_t)need * kCand) &&
        dev_alloc(&c->cand_over, (size_t)need)))
    return fail(c, SOM_ERR_ALLOC, "cannot allocate candidate lists for %lld slots", (long long)need);
  c->cand_cap = need;
  return SOM_OK;
}

static int ensure_transposed(som_ctx *c) {
  if (c->Wt) return SOM_OK;
  const size_t words = ((size_t)c->dim * c->kpad + 1) / 2;      // int16 entries
  if (!(dev_alloc(&c->Wt, words) && dev_alloc(&c->col_range, (size_t)2 * 64 * c->dim) &&
        dev_alloc(&c->qstep, (size_t)c->dim) && dev_alloc(&c->qstep_max_bits, 1) &&
        dev_alloc(&c->ct_partial, (size_t)kCtMaxSlabs * c->k * 3))) {
    dev_free(c->Wt); dev_free(c->col_range); dev_free(c->qstep); dev_free(c->qstep_max_bits); dev_free(c->ct_partial);
    return fail(c, SOM_ERR_ALLOC, "cannot allocate the transposed code book (%d x %d)", c->dim, c->kpad);
  }
  SOM_LAUNCH(c, launch_fill_zero_u32(c->stream, c->Wt, (int64_t)words));
  return SOM_OK;
}

// The transposed copy the full sparse rescan reads (bmu_exact.hip).  Optional: without it the rescan walks the
// row-major code book.
static void ensure_rescan_copy(som_ctx *c) {
  if (c->Wt32 || c->Wt32_tried) return;
  c->Wt32_tried = 1;
  c->kt32 = ((int64_t)c->k + 63) / 64 * 64;
  const size_t words = (size_t)c->dim * (size_t)c->kt32;
  if (words * sizeof(float) > kRescanCopyMax) return;
  if (!dev_alloc(&c->Wt32, words)) {
    (void)hipGetLastError();      // not an error of the search: it goes on without the copy
    c->Wt32 = nullptr;
  }
}

static int check_epoch_scalars(som_ctx *c, float radius, float scale) {
  if (!(radius > 0.f) || !isfinite(radius)) return fail(c, SOM_ERR_INVALID_ARG, "radius must be finite and > 0");
  if (!(scale > 0.f) || !(scale <= 1.f)) return fail(c, SOM_ERR_INVALID_ARG, "scale must be in (0, 1]");
  return SOM_OK;
}

static int check_rows(som_ctx *c, int64_t n) {
  if (n < 1 || n >= (1ll << 31)) return fail(c, SOM_ERR_INVALID_ARG, "n must be in [1, 2^31)");
  return SOM_OK;
}

static int check_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                     int64_t nnz) {
  if (!indptr) return fail(c, SOM_ERR_INVALID_ARG, "indptr is NULL");
  if (nnz < 0 || nnz >= (1ll << 31)) return fail(c, SOM_ERR_INVALID_ARG, "nnz must be in [0, 2^31)");
  if (nnz > 0 && (!indices || !values)) return fail(c, SOM_ERR_INVALID_ARG, "indices/values are NULL");
  return check_rows(c, n);
}

// ---------------------------------------------------------------- per-stage event brackets
struct StageTimer {
  som_ctx *c;
  int stage, slot;
  StageTimer(som_ctx *ctx, int st) : c(ctx), stage(st), slot(-1) {
    if (c->prof_on && c->prof_ev[stage] && c->prof_used[stage] < kProfMax) {
      slot = c->prof_used[stage]++;
      (void)hipEventRecord(c->prof_ev[stage][2 * slot], c->stream);
    }
  }
  ~StageTimer() {
    if (slot >= 0) (void)hipEventRecord(c->prof_ev[stage][2 * slot + 1], c->stream);
  }
};

// ---------------------------------------------------------------- stages
// Everything the filter pass needs besides the instances' own norms: centring vector (unless the
// data are the registered set, whose vector is kept), centred code book and node constants, and
// for the split-fp16 filter the fp16 planes of both operands.
static int prepare_dense(som_ctx *c, const float *X, int64_t n, const float *W, bool have_xn) {
  StageTimer t(c, 5);
  const bool split = uses_planes(c);
  const bool coarse = two_level_ready(c, n);
  if (!have_xn) {
    c->d_norms_valid = 0;
    c->d_split_valid = 0;
    c->csrd_valid = 0;          // the planes are about to hold other rows
    SOM_LAUNCH(c, launch_sample_col_means(c, X, n, c->dim, c->mu));
    SOM_LAUNCH(c, launch_vec_sqnorm(c, c->mu, c->dim, c->mu_norm2));
    SOM_LAUNCH(c, launch_row_sqnorms(c, X, n, c->dim, split ? c->mu : nullptr, c->xn32, nullptr, nullptr));
  }
  if (split && !(have_xn && c->d_split_valid)) {
    SOM_LAUNCH(c, launch_split_rows_f16(c, X, n, nullptr, c->mu, c->Xh, c->xscale, 0, coarse ? c->Xh1 : nullptr));
    c->d_split_valid = have_xn ? 1 : 0;
  }
  SOM_LAUNCH(c, launch_center_codebook(c, W, true, false, split));
  if (c->nb_function == SOM_NEIGHBORHOOD_BUBBLE) SOM_LAUNCH(c, launch_mask_duplicate_rows(c, W));
  if (split)
    SOM_LAUNCH(c, launch_split_rows_f16(c, c->Wc, c->k, c->wmax_bits + 1, nullptr, c->Wh, c->wscale, 0,
                                        coarse ? c->Wh1 : nullptr));
  SOM_LAUNCH(c, launch_fill_zero_u32(c->stream, c->list_counts, kListWords));
  return SOM_OK;
}

// The filter pass over the planes (or, with the fp32 filter, over X itself): candidates per instance.
static int dense_filter_stage(som_ctx *c, const float *X, int64_t n, bool split, bool coarse) {
  if (coarse) {
    SOM_LAUNCH(c, launch_bmu_coarse(c, n, nullptr));
    SOM_LAUNCH(c, launch_select_blocks(c, n));
    SOM_LAUNCH(c, launch_sort_keys(c, c->coarse_key, n, two_level_key_range((c->k + 127) / 128)));
    SOM_LAUNCH(c, launch_tile_lists(c, n));
    SOM_LAUNCH(c, launch_bmu_dense_h_fine(c, n));
  } else if (split) {
    SOM_LAUNCH(c, launch_bmu_dense_h(c, n, nullptr));
  } else {
    SOM_LAUNCH(c, launch_bmu_dense(c, X, n, nullptr));
  }
  return SOM_OK;
}

static int bmu_search_dense(som_ctx *c, const float *X, int64_t n, const float *W, int32_t *bmus, bool have_xn) {
  int rc = ensure_candidates(c, n, true);
  if (!rc) rc = prepare_dense(c, X, n, W, have_xn);
  if (rc) return rc;
  const bool split = uses_planes(c);
  const bool coarse = two_level_ready(c, n);
  c->two_level_n = coarse ? n : 0;
  {
    StageTimer t(c, 0);
    rc = dense_filter_stage(c, X, n, split, coarse);
    if (rc) return rc;
  }
  StageTimer t(c, 2);
  SOM_LAUNCH(c, launch_certify(c, n, coarse ? bmu_dense_h_fine_groups(c, n) : split ? bmu_dense_h_groups(c, n) : bmu_dense_groups(c, n),
                               split ? kCertifySplit : kCertifyFp32, nullptr, bmus, false, coarse ? c->sort_val[0] : nullptr));
  SOM_LAUNCH(c, launch_refine_dense(c, X, W, bmus));
  if (coarse) SOM_LAUNCH(c, launch_collect_tile_lists(c, n));
  if (split) SOM_LAUNCH(c, launch_bmu_dense_h_collect(c, n, coarse));
  else SOM_LAUNCH(c, launch_bmu_dense_collect(c, X, n));
  SOM_LAUNCH(c, launch_refine_lists_dense(c, X, W, bmus));
  SOM_LAUNCH(c, launch_rescan_dense(c, X, W, bmus));
  return SOM_OK;
}

// Everything the sparse sweep needs: scratch, norms of the instances (unless registered), the centring
// vector (mean of the code-book rows) with the quantisation steps, node constants, the transposed 16-bit
// code book and the scaled values.
static int prepare_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                       int64_t nnz, const float *W, bool have_xn) {
  if (nnz > c->vq_cap) {
    (void)hipStreamSynchronize(c->stream);
    dev_free(c->vq);
    c->vq_cap = 0;
    if (!dev_alloc(&c->vq, (size_t)nnz)) return fail(c, SOM_ERR_ALLOC, "cannot allocate %lld scaled values", (long long)nnz);
    c->vq_cap = nnz;
  }
  int rc = ensure_transposed(c);
  if (!rc) rc = ensure_candidates(c, n, false);
  if (rc) return rc;
  if (!have_xn) {
    c->d_norms_valid = 0;
    SOM_LAUNCH(c, launch_csr_row_sqnorms(c, indptr, values, n, c->xn32));
  }
  // centring vector of the sparse search: the mean of the code-book rows (changes every epoch);
  // it overwrites the one a registered dense training set may have cached
  if (c->data_kind == 1) { c->d_norms_valid = 0; c->d_split_valid = 0; }
  SOM_LAUNCH(c, launch_codebook_means_and_steps(c, W));
  SOM_LAUNCH(c, launch_vec_sqnorm(c, c->mu, c->dim, c->mu_norm2));
  SOM_LAUNCH(c, launch_fill_zero_u32(c->stream, c->list_counts, kListWords));
  return SOM_OK;
}

// First part of the sparse filter pass: the code book read once - centred, quantised, transposed, its node
// constants and norms taken on the way - and, under a bubble neighbourhood, its duplicate rows masked.
static int codebook_for_sweep(som_ctx *c, const float *W) {
  SOM_LAUNCH(c, launch_center_transpose_codebook(c, W));
  if (c->nb_function == SOM_NEIGHBORHOOD_BUBBLE) SOM_LAUNCH(c, launch_mask_duplicate_rows(c, W));
  return SOM_OK;
}

// Sparse rows searched through their dense planes: the dense filter stage against the data-centred code
// book, then the exact stage on the sparse rows themselves.  The centring vector and the norms of the
// centred rows are the registration's own copies, put in place of the context's for the launches.
struct PlaneOperands {
  som_ctx *c;
  float *mu, *mu_norm2, *xn32;
  explicit PlaneOperands(som_ctx *ctx) : c(ctx), mu(ctx->mu), mu_norm2(ctx->mu_norm2), xn32(ctx->xn32) {
    c->mu = c->csrd_mu; c->mu_norm2 = c->csrd_mu_norm2; c->xn32 = c->csrd_xn;
  }
  ~PlaneOperands() { c->mu = mu; c->mu_norm2 = mu_norm2; c->xn32 = xn32; }
};

static int dense_filter_stage(som_ctx *c, const float *X, int64_t n, bool split, bool coarse);

static int bmu_search_csr_planes(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                                 int64_t n, const float *W, int32_t *bmus) {
  int rc = ensure_candidates(c, n, true);
  if (rc) return rc;
  ensure_rescan_copy(c);
  PlaneOperands swap(c);
  const bool coarse = two_level_ready(c, n);
  c->two_level_n = coarse ? n : 0;
  {
    StageTimer t(c, 5);
    SOM_LAUNCH(c, launch_center_codebook(c, W, true, true /* |w|^2 in fp64 for the sparse exact kernels */, true));
    if (c->nb_function == SOM_NEIGHBORHOOD_BUBBLE) SOM_LAUNCH(c, launch_mask_duplicate_rows(c, W));
    SOM_LAUNCH(c, launch_split_rows_f16(c, c->Wc, c->k, c->wmax_bits + 1, nullptr, c->Wh, c->wscale, 0,
                                        coarse ? c->Wh1 : nullptr));
    SOM_LAUNCH(c, launch_fill_zero_u32(c->stream, c->list_counts, kListWords));
  }
  {
    StageTimer t(c, 1);
    rc = dense_filter_stage(c, nullptr, n, true, coarse);
    if (rc) return rc;
  }
  StageTimer t(c, 2);
  SOM_LAUNCH(c, launch_certify(c, n, coarse ? bmu_dense_h_fine_groups(c, n) : bmu_dense_h_groups(c, n), kCertifySplit,
                               nullptr, bmus, false, coarse ? c->sort_val[0] : nullptr));
  SOM_LAUNCH(c, launch_refine_csr(c, indptr, indices, values, W, bmus));
  if (coarse) SOM_LAUNCH(c, launch_collect_tile_lists(c, n));
  SOM_LAUNCH(c, launch_bmu_dense_h_collect(c, n, coarse));
  SOM_LAUNCH(c, launch_refine_lists_csr(c, indptr, indices, values, W, bmus));
  SOM_LAUNCH(c, launch_rescan_csr(c, indptr, indices, values, W, bmus));
  return SOM_OK;
}

static int bmu_search_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                          int64_t n, int64_t nnz, const float *W, int32_t *bmus, bool have_xn) {
  if (have_xn && c->csrd_valid && c->csrd_on) return bmu_search_csr_planes(c, indptr, indices, values, n, W, bmus);
  int rc = prepare_csr(c, indptr, indices, values, n, nnz, W, have_xn);
  if (rc) return rc;
  ensure_rescan_copy(c);
  // registered rows whose frequent columns were split off: the sweeps walk the tail and start from the
  // matrix-core pass over the hot block; the exact kernels keep the caller's full rows
  const bool hot = have_xn && c->hot_on;
  const int64_t *sw_indptr = hot ? c->tail_indptr : indptr;
  const int32_t *sw_indices = hot ? c->tail_indices : indices;
  const float *sw_values = hot ? c->tail_values : values;
  const int64_t sw_nnz = hot ? c->tail_nnz : nnz;
  {
    StageTimer t(c, 1);
    rc = codebook_for_sweep(c, W);
    if (rc) return rc;
    if (hot) {
      SOM_LAUNCH(c, launch_gather_hot_codebook(c, W));
      SOM_LAUNCH(c, launch_split_rows_f16(c, c->hot_Wc, c->k, c->hot_wmax_bits, nullptr, c->hot_Wh, c->hot_wscale, kHot));
      SOM_LAUNCH(c, launch_hot_partial(c, n));
    }
    SOM_LAUNCH(c, launch_scale_values(c, sw_indices, sw_values, sw_nnz));
    SOM_LAUNCH(c, launch_bmu_csr_sliced(c, sw_indptr, sw_indices, c->vq, n, false, nullptr, hot));
  }
  StageTimer t(c, 2);
  SOM_LAUNCH(c, launch_certify(c, n, 8 * c->csr_sweeps, kCertifyCsr, sw_indptr, bmus, hot));
  SOM_LAUNCH(c, launch_refine_csr(c, indptr, indices, values, W, bmus));
  SOM_LAUNCH(c, launch_bmu_csr_sliced(c, sw_indptr, sw_indices, c->vq, n, true, nullptr, hot));
  SOM_LAUNCH(c, launch_refine_lists_csr(c, indptr, indices, values, W, bmus));
  SOM_LAUNCH(c, launch_rescan_csr(c, indptr, indices, values, W, bmus));
  return SOM_OK;
}

static int update_dense(som_ctx *c, const float *X, int64_t n, const int32_t *bmus, float *W) {
  {
    StageTimer t(c, 3);
    SOM_LAUNCH(c, launch_sort_by_bmu(c, bmus, n));
    SOM_LAUNCH(c, launch_accumulate_dense(c, X, n));
  }
  StageTimer t(c, 4);
  SOM_LAUNCH(c, launch_smooth_and_divide(c, W));
  return SOM_OK;
}

static int update_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                      const int32_t *bmus, float *W) {
  {
    StageTimer t(c, 3);
    SOM_LAUNCH(c, launch_accumulate_csr(c, indptr, indices, values, n, bmus));
  }
  StageTimer t(c, 4);
  SOM_LAUNCH(c, launch_smooth_and_divide(c, W));
  return SOM_OK;
}

// Norms (and the centring vector) of the registered training set, computed once.
static int registered_norms(som_ctx *c) {
  if (c->d_norms_valid) return SOM_OK;
  if (c->data_kind == 1) {
    SOM_LAUNCH(c, launch_sample_col_means(c, c->d_data, c->d_n, c->dim, c->mu));
    SOM_LAUNCH(c, launch_vec_sqnorm(c, c->mu, c->dim, c->mu_norm2));
    // the split-fp16 filter works on centred instances, and its margin on their norms
    SOM_LAUNCH(c, launch_row_sqnorms(c, c->d_data, c->d_n, c->dim, uses_planes(c) ? c->mu : nullptr,
                                     c->xn32, nullptr, nullptr));
  } else {
    SOM_LAUNCH(c, launch_csr_row_sqnorms(c, c->d_indptr, c->d_values, c->d_n, c->xn32));
  }
  c->d_norms_valid = 1;
  return SOM_OK;
}

namespace som { int64_t choose_hot_columns(const std::vector<int32_t> &counts, std::vector<int32_t> &cols); }

static void free_hot(som_ctx *c) {
  dev_free(c->tail_start); dev_free(c->tail_indptr); dev_free(c->tail_indices); dev_free(c->tail_values);
  dev_free(c->hot_Xh); dev_free(c->hot_xscale); dev_free(c->hot_xn); dev_free(c->hot_P);
  c->hot_n_cap = 0;
  c->hot_nnz_cap = 0;
}

// Hot-column split of the registered sparse set (csr_hot.hip), examined once per registration: the column
// histogram, the choice of the columns (on the host: it waits for the stream), the tail as a CSR set of its
// own and the hot block as fp16 planes.  Leaves hot_on = 0 when the split is switched off, the columns are
// too few or too evenly used, or the table of partial sums would not be worth its memory.
static int registered_hot(som_ctx *c) {
  if (c->hot_valid) return SOM_OK;
  c->hot_valid = 1;
  c->hot_on = 0;
  const int64_t n = c->d_n, nnz = c->d_nnz;
  const int64_t kP = ((int64_t)c->k + 127) / 128 * 128;
  if (!c->hot_enabled || c->data_kind != 2 || c->dim < 4 * kHot || nnz < 1) return SOM_OK;
  if (n * kP * 4 > (8ll << 30)) return SOM_OK;
  if (!c->hot_counts) {
    const size_t halves = (size_t)kHot * 2;
    if (!(dev_alloc(&c->hot_counts, (size_t)c->dim) && dev_alloc(&c->hot_rank, (size_t)c->dim) &&
          dev_alloc(&c->hot_cols, (size_t)kHot) && dev_alloc(&c->hot_Wc, (size_t)c->k * kHot) &&
          dev_alloc(&c->hot_Wh, (size_t)c->k * halves) && dev_alloc(&c->hot_wscale, 1) &&
          dev_alloc(&c->hot_wmax_bits, 1))) {
      dev_free(c->hot_counts); dev_free(c->hot_rank); dev_free(c->hot_cols); dev_free(c->hot_Wc); dev_free(c->hot_Wh);
      dev_free(c->hot_wscale); dev_free(c->hot_wmax_bits);
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the hot-column tables");
    }
  }
  SOM_LAUNCH(c, launch_hot_histogram(c, c->d_indices, nnz, c->hot_counts));
  std::vector<int32_t> counts((size_t)c->dim), cols, rank((size_t)c->dim, -1);
  SOM_LAUNCH(c, hipMemcpyAsync(counts.data(), c->hot_counts, counts.size() * sizeof(int32_t), hipMemcpyDeviceToHost,
                               c->stream));
  SOM_LAUNCH(c, hipStreamSynchronize(c->stream));
  const int64_t held = choose_hot_columns(counts, cols);
  if ((int)cols.size() < kHot || (double)held < kHotMinShare * (double)nnz) return SOM_OK;
  for (int h = 0; h < kHot; ++h) rank[(size_t)cols[h]] = h;
  SOM_LAUNCH(c, hipMemcpyAsync(c->hot_rank, rank.data(), rank.size() * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
  SOM_LAUNCH(c, hipMemcpyAsync(c->hot_cols, cols.data(), cols.size() * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
  SOM_LAUNCH(c, hipStreamSynchronize(c->stream));          // the host vectors go out of scope
  const int64_t tail_cap = nnz;                            // the counters may include out-of-range indices the kernels clamp
  if (n > c->hot_n_cap || tail_cap > c->hot_nnz_cap) {
    free_hot(c);
    if (!(dev_alloc(&c->tail_start, (size_t)n + 1) && dev_alloc(&c->tail_indptr, (size_t)n + 1) &&
          dev_alloc(&c->tail_indices, (size_t)tail_cap) && dev_alloc(&c->tail_values, (size_t)tail_cap) &&
          dev_alloc(&c->hot_Xh, (size_t)n * kHot * 2) && dev_alloc(&c->hot_xscale, (size_t)n) &&
          dev_alloc(&c->hot_xn, (size_t)n) && dev_alloc(&c->hot_P, (size_t)(n * kP)))) {
      free_hot(c);
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the hot-column split of %lld rows", (long long)n);
    }
    c->hot_n_cap = n;
    c->hot_nnz_cap = tail_cap;
  }
  SOM_LAUNCH(c, launch_fill_zero_u32(c->stream, c->tail_start + n, 1));
  SOM_LAUNCH(c, launch_tail_lengths(c, c->d_indptr, c->d_indices, n, c->tail_start));
  SOM_LAUNCH(c, launch_scan_exclusive_i32(c, c->tail_start, c->tail_start, (int)(n + 1)));
  SOM_LAUNCH(c, launch_split_hot_tail(c, c->d_indptr, c->d_indices, c->d_values, n));
  int32_t total = 0;
  SOM_LAUNCH(c, hipMemcpyAsync(&total, c->tail_start + n, sizeof(total), hipMemcpyDeviceToHost, c->stream));
  SOM_LAUNCH(c, hipStreamSynchronize(c->stream));
  c->tail_nnz = total;
  c->hot_on = 1;
  return SOM_OK;
}

// Dense planes of the registered sparse set (som_set_sparse_dense_filter), examined once per registration:
// column means of the rows as the centring vector, then the rows are written out densely a batch at a time
// and go through the kernels that give dense data their norms and fp16 planes.  Leaves csrd_on = 0 when the
// mode is switched off, the filter does not use planes, or the rows are too long or too empty for the
// matrix cores to beat the gather sweep.
static int registered_csr_dense(som_ctx *c) {
  if (c->csrd_valid) return SOM_OK;
  c->csrd_valid = 1;
  c->csrd_on = 0;
  const int64_t n = c->d_n, nnz = c->d_nnz;
  if (!c->csrd_enabled || c->data_kind != 2 || !uses_planes(c) || c->dim > kCsrDenseMaxDim || nnz < 1) return SOM_OK;
  if ((double)nnz < kCsrDenseMinDensity * (double)n * (double)c->dim) return SOM_OK;
  int rc = ensure_rows(c, n, true);          // planes, centred code book (may reset csrd_valid: set again below)
  if (rc) return rc;
  c->csrd_valid = 1;
  if (n > c->csrd_n_cap || !c->csrd_mu) {
    dev_free(c->csrd_xn); dev_free(c->csrd_mu); dev_free(c->csrd_mu_norm2);
    c->csrd_n_cap = 0;
    if (!(dev_alloc(&c->csrd_xn, (size_t)n) && dev_alloc(&c->csrd_mu, (size_t)c->dim) && dev_alloc(&c->csrd_mu_norm2, 1))) {
      dev_free(c->csrd_xn); dev_free(c->csrd_mu); dev_free(c->csrd_mu_norm2);
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the norms of %lld centred rows", (long long)n);
    }
    c->csrd_n_cap = n;
  }
  SOM_LAUNCH(c, launch_csr_col_sums(c, c->d_indices, c->d_values, nnz, c->csrd_mu));
  SOM_LAUNCH(c, launch_scale_vector(c, c->csrd_mu, c->dim, 1.0f / (float)n));
  SOM_LAUNCH(c, launch_vec_sqnorm(c, c->csrd_mu, c->dim, c->csrd_mu_norm2));
  // batches of rows through a dense buffer of at most 1 GiB
  int64_t batch = (1ll << 28) / c->dim;
  if (batch > n) batch = n;
  if (batch < 1) batch = 1;
  float *dense = nullptr;
  if (!dev_alloc(&dense, (size_t)batch * c->dim)) return fail(c, SOM_ERR_ALLOC, "cannot allocate a batch of dense rows");
  const bool coarse = two_level_ready(c, n);
  const size_t row_halves = (size_t)((c->dim + 31) / 32) * 64, row_halves1 = (size_t)((c->dim + 63) / 64) * 64;
  int rcl = SOM_OK;
  for (int64_t r0 = 0; r0 < n && rcl == SOM_OK; r0 += batch) {
    const int64_t rows = n - r0 < batch ? n - r0 : batch;
    hipError_t e = launch_csr_densify(c, c->d_indptr, c->d_indices, c->d_values, r0, rows, dense);
    if (e == hipSuccess) e = launch_row_sqnorms(c, dense, rows, c->dim, c->csrd_mu, c->csrd_xn + r0, nullptr, nullptr);
    if (e == hipSuccess)
      e = launch_split_rows_f16(c, dense, rows, nullptr, c->csrd_mu, c->Xh + (size_t)r0 * row_halves, c->xscale + r0, 0,
                                coarse ? c->Xh1 + (size_t)r0 * row_halves1 : nullptr);
    if (e != hipSuccess) rcl = dev_fail(c, e, "dense planes of the sparse rows");
  }
  hipError_t es = hipStreamSynchronize(c->stream);     // the batch buffer is freed below
  dev_free(dense);
  if (rcl != SOM_OK) return rcl;
  if (es != hipSuccess) return dev_fail(c, es, "dense planes of the sparse rows");
  c->d_split_valid = 0;       // the planes do not belong to a registered dense set
  c->csrd_on = 1;
  return SOM_OK;
}

static bool is_registered_dense(const som_ctx *c, const float *data, int64_t n) {
  return c->data_kind == 1 && data == c->d_data && n == c->d_n;
}

static bool is_registered_csr(const som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                              int64_t n) {
  return c->data_kind == 2 && indptr == c->d_indptr && indices == c->d_indices && values == c->d_values &&
         n == c->d_n;
}

// ---------------------------------------------------------------- entry points
extern "C" {

int som_init(som_ctx **out, int rows, int cols, int dim, int map_type, int grid_type, float *codebook,
             uint64_t seed, void *hip_stream) {
  if (!out) return fail(nullptr, SOM_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  if (rows < 1 || cols < 1 || dim < 1) return fail(nullptr, SOM_ERR_INVALID_ARG, "rows, cols and dim must be >= 1");
  if (rows > 65535 || cols > 65535 || (int64_t)rows * cols > (1 << 24))
    return fail(nullptr, SOM_ERR_INVALID_ARG, "map too large (each side <= 65535, rows*cols <= 2^24)");
  if ((int64_t)rows * cols * dim >= (1ll << 40)) return fail(nullptr, SOM_ERR_INVALID_ARG, "code book too large");
  if (map_type != SOM_MAP_PLANAR && map_type != SOM_MAP_TOROID)
    return fail(nullptr, SOM_ERR_INVALID_ARG, "unknown map_type %d", map_type);
  if (grid_type != SOM_GRID_SQUARE && grid_type != SOM_GRID_HEXAGONAL)
    return fail(nullptr, SOM_ERR_INVALID_ARG, "unknown grid_type %d", grid_type);
  if (!codebook) return fail(nullptr, SOM_ERR_INVALID_ARG, "codebook is NULL");

  som_ctx *c = (som_ctx *)calloc(1, sizeof(som_ctx));
  if (!c) return fail(nullptr, SOM_ERR_ALLOC, "out of host memory");
  c->rows = rows; c->cols = cols; c->dim = dim; c->k = rows * cols;
  c->map_type = map_type; c->grid_type = grid_type;
  c->stream = (hipStream_t)hip_stream;
  csr_slice_geometry(c->k, &c->csr_acc, &c->csr_sweeps, &c->kpad);
  c->filter = SOM_FILTER_AUTO;
  c->scale_cooling = -1;
  c->hot_enabled = 1;
  c->csrd_enabled = 1;
  c->smooth_mfma_min = kSmoothMfmaMin;
  c->smooth_split_min = kSmoothSplitMin;

  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    free(c);
    return fail(nullptr, SOM_ERR_DEVICE, "no HIP device");
  }
  c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  (void)static_scratch(nullptr);      // so that a later som_bmu_distances_dense_static on this device has nothing left to set up

  const size_t K = (size_t)c->k;
  const size_t images = grid_type == SOM_GRID_HEXAGONAL ? 2 : 1;
  bool ok = dev_alloc(&c->wn32, (K + 127) / 128 * 128) && dev_alloc(&c->wn64, K) && dev_alloc(&c->wmax_bits, 2) &&
            dev_alloc(&c->counts, K + 1) && dev_alloc(&c->seg_off, K + 1) && dev_alloc(&c->chunk_off, K + 1) &&
            dev_alloc(&c->massD, K) && dev_alloc(&c->dist_partial, kDistBlocks) && dev_alloc(&c->cntT, 2 * K) && dev_alloc(&c->gx, 2 * (size_t)cols + 1) &&
            dev_alloc(&c->gy, (size_t)rows) && dev_alloc(&c->params, 1) && dev_alloc(&c->list_counts, kListWords) &&
            dev_alloc(&c->mu, (size_t)dim) && dev_alloc(&c->mu_partial, (size_t)64 * dim) &&
            dev_alloc(&c->zero16, 16) && dev_alloc(&c->mu_norm2, 1) && dev_alloc(&c->wscale, 1) &&
            dev_alloc(&c->S, K * dim) && dev_alloc(&c->T, images * K * dim) &&
            dev_alloc(&c->hit_x, K) && dev_alloc(&c->hit_n, (size_t)rows) && dev_alloc(&c->hit_rows, (size_t)rows + 1);
  if (ok && rows <= kSmoothMatMax && cols <= kSmoothMatMax) {
    const size_t par = grid_type == SOM_GRID_HEXAGONAL ? 2 : 1;
    c->xi_pad = ((cols + 31) / 32) * 32;
    c->e_pad = (int)(((((size_t)rows + par - 1) / par) + 31) / 32) * 32;
    ok = dev_alloc(&c->GxT, par * par * cols * c->xi_pad) && dev_alloc(&c->GyT, par * rows * c->e_pad);
  }
  if (!ok) {
    som_destroy(c);
    return fail(nullptr, SOM_ERR_ALLOC, "cannot allocate map scratch (%d nodes x %d)", c->k, dim);
  }
  hipError_t e = launch_fill_zero_u32(c->stream, c->list_counts, kListWords);
  if (e == hipSuccess) e = launch_fill_zero_u32(c->stream, c->zero16, 16);
  if (e == hipSuccess && K % 128 != 0) {       // the tail of the node constants past k stays +inf for good
    float inf[128];
    for (int i = 0; i < 128; ++i) inf[i] = INFINITY;
    e = hipMemcpyAsync(c->wn32 + K, inf, (128 - K % 128) * sizeof(float), hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  }
  if (e == hipSuccess && seed != 0) e = launch_fill_uniform(c, codebook, (int64_t)c->k * dim, seed);
  if (e != hipSuccess) {
    int rc = dev_fail(nullptr, e, "som_init");
    som_destroy(c);
    return rc;
  }
  *out = c;
  return SOM_OK;
}

void som_destroy(som_ctx *c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  free_row_scratch(c);
  dev_free(c->wn32); dev_free(c->wn64); dev_free(c->wmax_bits); dev_free(c->counts); dev_free(c->seg_off);
  dev_free(c->chunk_off); dev_free(c->massD); dev_free(c->dist_partial); dev_free(c->row_hash); dev_free(c->dedup_keys);
  dev_free(c->dedup_lowest); dev_free(c->cntT); dev_free(c->gx); dev_free(c->gy);
  dev_free(c->params); dev_free(c->list_counts); dev_free(c->unit_work); dev_free(c->vq); dev_free(c->S); dev_free(c->T); dev_free(c->Wt); dev_free(c->Wt32);
  dev_free(c->col_range); dev_free(c->qstep); dev_free(c->qstep_max_bits); dev_free(c->ct_partial); dev_free(c->H2);
  dev_free(c->GxT); dev_free(c->GyT); dev_free(c->hit_x); dev_free(c->hit_n); dev_free(c->hit_rows);
  dev_free(c->mu); dev_free(c->mu_partial); dev_free(c->Wc); dev_free(c->zero16); dev_free(c->mu_norm2);
  dev_free(c->Wh); dev_free(c->Wh1); dev_free(c->wscale);
  free_hot(c);
  dev_free(c->csrd_mu); dev_free(c->csrd_mu_norm2); dev_free(c->csrd_xn);
  dev_free(c->hot_counts); dev_free(c->hot_rank); dev_free(c->hot_cols); dev_free(c->hot_Wc); dev_free(c->hot_Wh);
  dev_free(c->hot_wscale); dev_free(c->hot_wmax_bits);
  for (int s = 0; s < SOM_PROFILE_STAGES; ++s) {
    if (!c->prof_ev[s]) continue;
    for (int e = 0; e < 2 * kProfMax; ++e) (void)hipEventDestroy(c->prof_ev[s][e]);
    free(c->prof_ev[s]);
  }
  free(c);
}

const char *som_last_error(const som_ctx *c) { return c ? c->err : g_init_error; }

int som_bmus_dense(som_ctx *c, const float *data, int64_t n, const float *codebook, int32_t *bmus) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!data || !codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  int rc = check_rows(c, n);
  if (!rc) rc = ensure_rows(c, n, true);
  bool reg = false;
  if (!rc && is_registered_dense(c, data, n)) { rc = registered_norms(c); reg = true; }
  if (rc) return rc;
  return bmu_search_dense(c, data, n, codebook, bmus, reg);
}

int som_bmus_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                 int64_t nnz, const float *codebook, int32_t *bmus) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  int rc = check_csr(c, indptr, indices, values, n, nnz);
  if (!rc) rc = ensure_rows(c, n, false);
  bool reg = false;
  if (!rc && is_registered_csr(c, indptr, indices, values, n)) {
    rc = registered_norms(c);
    if (!rc) rc = registered_csr_dense(c);
    if (!rc && !c->csrd_on) rc = registered_hot(c);
    reg = true;
  }
  if (rc) return rc;
  return bmu_search_csr(c, indptr, indices, values, n, nnz, codebook, bmus, reg);
}

int som_bmu_distances_dense(som_ctx *c, const float *data, int64_t n, const float *codebook, const int32_t *bmus,
                            float *distances, double *qerror) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!data || !codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  if (!distances && !qerror) return fail(c, SOM_ERR_INVALID_ARG, "distances and qerror are both NULL");
  const int rc = check_rows(c, n);
  if (rc) return rc;
  SOM_LAUNCH(c, launch_bmu_distances(c, data, nullptr, nullptr, nullptr, n, codebook, bmus, distances, qerror));
  return SOM_OK;
}

int som_bmu_distances_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                          int64_t nnz, const float *codebook, const int32_t *bmus, float *distances,
                          double *qerror) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  if (!distances && !qerror) return fail(c, SOM_ERR_INVALID_ARG, "distances and qerror are both NULL");
  const int rc = check_csr(c, indptr, indices, values, n, nnz);
  if (rc) return rc;
  SOM_LAUNCH(c, launch_bmu_distances(c, nullptr, indptr, indices, values, n, codebook, bmus, distances, qerror));
  return SOM_OK;
}

int som_bmu_distances_dense_static(const float *data, int64_t n, int dim, const float *codebook, int n_nodes,
                                   const int32_t *bmus, float *distances, double *qerror, void *hip_stream) {
  if (!data || !codebook || !bmus) return fail(nullptr, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  if (!distances && !qerror) return fail(nullptr, SOM_ERR_INVALID_ARG, "distances and qerror are both NULL");
  if (n < 1 || n >= (1ll << 31)) return fail(nullptr, SOM_ERR_INVALID_ARG, "n must be in [1, 2^31)");
  if (dim < 1 || n_nodes < 1 || n_nodes > (1 << 24) || (int64_t)n_nodes * dim >= (1ll << 40))
    return fail(nullptr, SOM_ERR_INVALID_ARG, "dim and n_nodes must be >= 1, n_nodes <= 2^24, n_nodes * dim < 2^40");
  hipError_t e = hipSuccess;
  double *partial = static_scratch(&e);
  if (!partial) return dev_fail(nullptr, e, "address of the static scratch");
  e = launch_bmu_distances_on((hipStream_t)hip_stream, data, nullptr, nullptr, nullptr, n, codebook, n_nodes, dim,
                              bmus, distances, qerror, partial);
  if (e != hipSuccess) return dev_fail(nullptr, e, "som_bmu_distances_dense_static");
  return SOM_OK;
}

int som_update_dense(som_ctx *c, const float *data, int64_t n, const int32_t *bmus, float *codebook,
                     float radius, float scale) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!data || !codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  int rc = check_rows(c, n);
  if (!rc) rc = check_epoch_scalars(c, radius, scale);
  if (!rc) rc = ensure_rows(c, n, true);
  if (rc) return rc;
  SOM_LAUNCH(c, launch_epoch_params(c, 0, 1, radius, radius, scale, scale, SOM_COOL_LINEAR));
  return update_dense(c, data, n, bmus, codebook);
}

int som_update_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                   int64_t nnz, const int32_t *bmus, float *codebook, float radius, float scale) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  int rc = check_csr(c, indptr, indices, values, n, nnz);
  if (!rc) rc = check_epoch_scalars(c, radius, scale);
  if (!rc) rc = ensure_rows(c, n, false);
  if (rc) return rc;
  SOM_LAUNCH(c, launch_epoch_params(c, 0, 1, radius, radius, scale, scale, SOM_COOL_LINEAR));
  return update_csr(c, indptr, indices, values, n, bmus, codebook);
}

int som_train_epoch_dense(som_ctx *c, const float *data, int64_t n, float *codebook, float radius, float scale,
                          int32_t *bmus) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!data || !codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  int rc = check_rows(c, n);
  if (!rc) rc = check_epoch_scalars(c, radius, scale);
  if (!rc) rc = ensure_rows(c, n, true);
  bool reg = false;
  if (!rc && is_registered_dense(c, data, n)) { rc = registered_norms(c); reg = true; }
  if (rc) return rc;
  SOM_LAUNCH(c, launch_epoch_params(c, 0, 1, radius, radius, scale, scale, SOM_COOL_LINEAR));
  rc = bmu_search_dense(c, data, n, codebook, bmus, reg);
  if (rc) return rc;
  return update_dense(c, data, n, bmus, codebook);
}

int som_train_epoch_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                        int64_t n, int64_t nnz, float *codebook, float radius, float scale, int32_t *bmus) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  int rc = check_csr(c, indptr, indices, values, n, nnz);
  if (!rc) rc = check_epoch_scalars(c, radius, scale);
  if (!rc) rc = ensure_rows(c, n, false);
  bool reg = false;
  if (!rc && is_registered_csr(c, indptr, indices, values, n)) {
    rc = registered_norms(c);
    if (!rc) rc = registered_csr_dense(c);
    if (!rc && !c->csrd_on) rc = registered_hot(c);
    reg = true;
  }
  if (rc) return rc;
  SOM_LAUNCH(c, launch_epoch_params(c, 0, 1, radius, radius, scale, scale, SOM_COOL_LINEAR));
  rc = bmu_search_csr(c, indptr, indices, values, n, nnz, codebook, bmus, reg);
  if (rc) return rc;
  return update_csr(c, indptr, indices, values, n, bmus, codebook);
}

int som_set_data_dense(som_ctx *c, const float *data, int64_t n) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!data) return fail(c, SOM_ERR_INVALID_ARG, "data is NULL");
  int rc = check_rows(c, n);
  if (rc) return rc;
  c->data_kind = 1; c->d_data = data; c->d_n = n; c->d_nnz = 0;
  c->d_indptr = nullptr; c->d_indices = nullptr; c->d_values = nullptr;
  c->d_norms_valid = 0;
  c->d_split_valid = 0;
  c->hot_valid = 0;
  c->hot_on = 0;
  c->csrd_valid = 0;
  c->csrd_on = 0;
  return SOM_OK;
}

int som_set_data_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                     int64_t nnz) {
  if (!c) return SOM_ERR_INVALID_ARG;
  int rc = check_csr(c, indptr, indices, values, n, nnz);
  if (rc) return rc;
  c->data_kind = 2; c->d_data = nullptr; c->d_n = n; c->d_nnz = nnz;
  c->d_indptr = indptr; c->d_indices = indices; c->d_values = values;
  c->d_norms_valid = 0;
  c->d_split_valid = 0;
  c->hot_valid = 0;
  c->hot_on = 0;
  c->csrd_valid = 0;
  c->csrd_on = 0;
  return SOM_OK;
}

static void schedule_defaults(const som_ctx *c, float &r0, float &rN, float &s0, float &sN) {
  if (!(r0 > 0.f)) {
    r0 = 0.5f * (float)(c->rows < c->cols ? c->rows : c->cols);
    if (r0 < 1.f) r0 = 1.f;
  }
  if (!(rN > 0.f)) rN = 1.f;
  if (!(s0 > 0.f)) s0 = 1.0f;
  if (!(sN > 0.f)) sN = 0.01f;
}

int som_train(som_ctx *c, int n_epochs, float radius0, float radiusN, float scale0, float scaleN, int cooling,
              float *codebook, int32_t *bmus) {
  return som_train_snapshots(c, n_epochs, radius0, radiusN, scale0, scaleN, cooling, codebook, bmus, 0, nullptr,
                             nullptr, nullptr);
}

int som_train_snapshots(som_ctx *c, int n_epochs, float radius0, float radiusN, float scale0, float scaleN,
                        int cooling, float *codebook, int32_t *bmus, int snapshots, float *umatrices,
                        float *codebooks, int32_t *bmus_all) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (snapshots < 0 || snapshots > 2) return fail(c, SOM_ERR_INVALID_ARG, "snapshots must be 0, 1 or 2");
  if (snapshots >= 1 && !umatrices) return fail(c, SOM_ERR_INVALID_ARG, "umatrices is NULL");
  if (snapshots == 2 && (!codebooks || !bmus_all)) return fail(c, SOM_ERR_INVALID_ARG, "codebooks/bmus_all is NULL");
  if (c->data_kind == 0) return fail(c, SOM_ERR_STATE, "no training data registered (som_set_data_*)");
  if (!codebook || !bmus) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  if (n_epochs < 1) return fail(c, SOM_ERR_INVALID_ARG, "n_epochs must be >= 1");
  if (cooling != SOM_COOL_LINEAR && cooling != SOM_COOL_EXPONENTIAL)
    return fail(c, SOM_ERR_INVALID_ARG, "unknown cooling %d", cooling);
  schedule_defaults(c, radius0, radiusN, scale0, scaleN);
  if (!isfinite(radius0) || !isfinite(radiusN)) return fail(c, SOM_ERR_INVALID_ARG, "radius not finite");
  if (scale0 > 1.f || scaleN > 1.f) return fail(c, SOM_ERR_INVALID_ARG, "scale must be in (0, 1]");
  const bool dense = c->data_kind == 1;
  int rc = ensure_rows(c, c->d_n, dense);
  if (rc) return rc;
  rc = registered_norms(c);
  if (!rc && !dense) rc = registered_csr_dense(c);
  if (!rc && !dense && !c->csrd_on) rc = registered_hot(c);
  if (rc) return rc;
  for (int e = 0; e < n_epochs; ++e) {
    SOM_LAUNCH(c, launch_epoch_params(c, e, n_epochs, radius0, radiusN, scale0, scaleN, cooling));
    if (dense) {
      rc = bmu_search_dense(c, c->d_data, c->d_n, codebook, bmus, true);
      if (!rc) rc = update_dense(c, c->d_data, c->d_n, bmus, codebook);
    } else {
      rc = bmu_search_csr(c, c->d_indptr, c->d_indices, c->d_values, c->d_n, c->d_nnz, codebook, bmus, true);
      if (!rc) rc = update_csr(c, c->d_indptr, c->d_indices, c->d_values, c->d_n, bmus, codebook);
    }
    if (rc) return rc;
    if (snapshots >= 1) SOM_LAUNCH(c, launch_umatrix(c, codebook, umatrices + (size_t)e * c->k));
    if (snapshots == 2) {
      SOM_LAUNCH(c, hipMemcpyAsync(codebooks + (size_t)e * c->k * c->dim, codebook,
                                   (size_t)c->k * c->dim * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
      SOM_LAUNCH(c, hipMemcpyAsync(bmus_all + (size_t)e * c->d_n, bmus, (size_t)c->d_n * sizeof(int32_t),
                                   hipMemcpyDeviceToDevice, c->stream));
    }
  }
  return SOM_OK;
}

int som_cool_schedule(som_ctx *c, int n_epochs, float radius0, float radiusN, float scale0, float scaleN,
                      int cooling, double *radius_out, double *scale_out) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (n_epochs < 1) return fail(c, SOM_ERR_INVALID_ARG, "n_epochs must be >= 1");
  if (cooling != SOM_COOL_LINEAR && cooling != SOM_COOL_EXPONENTIAL)
    return fail(c, SOM_ERR_INVALID_ARG, "unknown cooling %d", cooling);
  schedule_defaults(c, radius0, radiusN, scale0, scaleN);
  SOM_LAUNCH(c, launch_cool_schedule(c, n_epochs, radius0, radiusN, scale0, scaleN, cooling, radius_out,
                                     scale_out));
  return SOM_OK;
}

int som_umatrix(som_ctx *c, const float *codebook, float *umatrix) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!codebook || !umatrix) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  SOM_LAUNCH(c, launch_umatrix(c, codebook, umatrix));
  return SOM_OK;
}

int som_set_neighborhood(som_ctx *c, int function, int compact_support) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (function != SOM_NEIGHBORHOOD_GAUSSIAN && function != SOM_NEIGHBORHOOD_BUBBLE)
    return fail(c, SOM_ERR_INVALID_ARG, "unknown neighborhood function %d", function);
  const bool direct = function != SOM_NEIGHBORHOOD_GAUSSIAN || compact_support;
  if (direct && !c->H2) {
    const size_t width = (size_t)(c->map_type == SOM_MAP_TOROID ? c->cols : 2 * c->cols - 1) + 16;
    const size_t classes = c->grid_type == SOM_GRID_HEXAGONAL ? 3 : 1;
    if (!dev_alloc(&c->H2, classes * c->rows * width))
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the neighbourhood table");
  }
  if (function == SOM_NEIGHBORHOOD_BUBBLE && !c->row_hash) {
    // a bubble makes whole classes of nodes bit-identical: the searches take the duplicates out first
    int slots = 64;
    while (slots < 2 * c->k) slots *= 2;
    if (!(dev_alloc(&c->row_hash, (size_t)c->k) && dev_alloc(&c->dedup_keys, (size_t)slots) &&
          dev_alloc(&c->dedup_lowest, (size_t)slots))) {
      dev_free(c->row_hash); dev_free(c->dedup_keys); dev_free(c->dedup_lowest);
      return fail(c, SOM_ERR_ALLOC, "cannot allocate the duplicate-row table");
    }
    c->dedup_slots = slots;
  }
  c->nb_function = function;
  c->nb_compact = compact_support ? 1 : 0;
  return SOM_OK;
}

int som_set_scale_cooling(som_ctx *c, int cooling) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (cooling != SOM_COOL_AS_RADIUS && cooling != SOM_COOL_LINEAR && cooling != SOM_COOL_EXPONENTIAL)
    return fail(c, SOM_ERR_INVALID_ARG, "unknown cooling %d", cooling);
  c->scale_cooling = cooling;
  return SOM_OK;
}

int som_validate_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                     int64_t nnz) {
  if (!c) return SOM_ERR_INVALID_ARG;
  int rc = check_csr(c, indptr, indices, values, n, nnz);
  if (rc) return rc;
  int32_t *flag = c->list_counts + 3;
  int32_t bad = 0;
  SOM_LAUNCH(c, launch_fill_zero_u32(c->stream, flag, 1));
  SOM_LAUNCH(c, launch_validate_csr(c, indptr, indices, n, nnz, flag));
  SOM_LAUNCH(c, hipMemcpyAsync(&bad, flag, sizeof(bad), hipMemcpyDeviceToHost, c->stream));
  SOM_LAUNCH(c, hipStreamSynchronize(c->stream));
  switch (bad) {
    case 0: return SOM_OK;
    case kCsrBadFirst: return fail(c, SOM_ERR_INVALID_ARG, "CSR: indptr[0] is not 0");
    case kCsrBadLast: return fail(c, SOM_ERR_INVALID_ARG, "CSR: indptr[n] is not nnz");
    case kCsrBadOrder: return fail(c, SOM_ERR_INVALID_ARG, "CSR: indptr decreases or leaves [0, nnz]");
    case kCsrBadIndex: return fail(c, SOM_ERR_INVALID_ARG, "CSR: a column index is outside [0, dim)");
    default: return fail(c, SOM_ERR_INVALID_ARG, "CSR: column indices of a row are not strictly increasing");
  }
}

int som_set_sparse_hot_block(som_ctx *c, int enable) {
  if (!c) return SOM_ERR_INVALID_ARG;
  c->hot_enabled = enable ? 1 : 0;
  c->hot_valid = 0;          // examined again at the next use of the registered set
  c->hot_on = 0;
  return SOM_OK;
}

int som_sparse_hot_block_active(const som_ctx *c) { return c && c->hot_valid && c->hot_on ? 1 : 0; }

int som_set_sparse_dense_filter(som_ctx *c, int enable) {
  if (!c) return SOM_ERR_INVALID_ARG;
  c->csrd_enabled = enable ? 1 : 0;
  c->csrd_valid = 0;         // examined again at the next use of the registered set
  c->csrd_on = 0;
  return SOM_OK;
}

int som_sparse_dense_filter_active(const som_ctx *c) { return c && c->csrd_valid && c->csrd_on ? 1 : 0; }

int som_set_smoothing(som_ctx *c, int form) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (form != SOM_SMOOTH_AUTO && form != SOM_SMOOTH_VECTOR && form != SOM_SMOOTH_MATRIX && form != SOM_SMOOTH_MATRIX_SPLIT)
    return fail(c, SOM_ERR_INVALID_ARG, "unknown smoothing form %d", form);
  c->smooth_mfma_min = form == SOM_SMOOTH_AUTO ? kSmoothMfmaMin : (form == SOM_SMOOTH_VECTOR ? 0 : 1);
  c->smooth_split_min = form == SOM_SMOOTH_AUTO ? kSmoothSplitMin : (form == SOM_SMOOTH_MATRIX_SPLIT ? 1 : 0);
  return SOM_OK;
}

int som_set_filter(som_ctx *c, int filter) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (filter != SOM_FILTER_FP32 && filter != SOM_FILTER_SPLIT_F16 && filter != SOM_FILTER_TWO_LEVEL &&
      filter != SOM_FILTER_AUTO)
    return fail(c, SOM_ERR_INVALID_ARG, "unknown filter %d", filter);
  if (filter != c->filter) {           // norms and planes of a registered set belong to the filter they were made for
    c->d_norms_valid = 0;
    c->d_split_valid = 0;
    c->csrd_valid = 0;
  }
  c->filter = filter;
  return SOM_OK;
}

int som_debug_scores_dense(som_ctx *c, const float *data, int64_t n, const float *codebook, float *scores,
                           float *mu_out, double *margin_out) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!data || !codebook || !scores || !mu_out || !margin_out) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  int rc = check_rows(c, n);
  if (!rc) rc = ensure_rows(c, n, true);
  if (!rc) rc = ensure_candidates(c, n, true);
  if (!rc) rc = prepare_dense(c, data, n, codebook, false);
  if (rc) return rc;
  const bool split = uses_planes(c);
  const bool coarse = c->filter == SOM_FILTER_TWO_LEVEL && two_level_ready(c, n);    // asked for by name: its coarse scores
  if (coarse) SOM_LAUNCH(c, launch_bmu_coarse(c, n, scores));
  else if (split) SOM_LAUNCH(c, launch_bmu_dense_h(c, n, scores));
  else SOM_LAUNCH(c, launch_bmu_dense(c, data, n, scores));
  SOM_LAUNCH(c, launch_margins(c, n, coarse ? kCertifyCoarse : split ? kCertifySplit : kCertifyFp32, nullptr, margin_out));
  SOM_LAUNCH(c, hipMemcpyAsync(mu_out, c->mu, (size_t)c->dim * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
  return SOM_OK;
}

int som_debug_scores_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                         int64_t nnz, const float *codebook, float *scores, float *mu_out, double *margin_out) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!codebook || !scores || !mu_out || !margin_out) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  int rc = check_csr(c, indptr, indices, values, n, nnz);
  if (!rc) rc = ensure_rows(c, n, false);
  if (!rc) rc = prepare_csr(c, indptr, indices, values, n, nnz, codebook, false);
  if (rc) return rc;
  rc = codebook_for_sweep(c, codebook);
  if (rc) return rc;
  SOM_LAUNCH(c, launch_scale_values(c, indices, values, nnz));
  SOM_LAUNCH(c, launch_bmu_csr_sliced(c, indptr, indices, c->vq, n, false, scores));
  SOM_LAUNCH(c, launch_margins(c, n, kCertifyCsr, indptr, margin_out));
  SOM_LAUNCH(c, hipMemcpyAsync(mu_out, c->mu, (size_t)c->dim * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
  return SOM_OK;
}

int som_debug_mfma_f16(const uint16_t *a, const uint16_t *b, const float *c_in, float *d_out, int count,
                       void *hip_stream) {
  if (!a || !b || !c_in || !d_out || count < 1) return SOM_ERR_INVALID_ARG;
  return launch_probe_mfma_f16((hipStream_t)hip_stream, a, b, c_in, d_out, count) == hipSuccess ? SOM_OK
                                                                                                : SOM_ERR_DEVICE;
}

int som_debug_xcc_ids(int32_t *out, int n_blocks, void *hip_stream) {
  if (!out || n_blocks < 1 || n_blocks > (1 << 20)) return SOM_ERR_INVALID_ARG;
  return launch_probe_xcc((hipStream_t)hip_stream, out, n_blocks) == hipSuccess ? SOM_OK : SOM_ERR_DEVICE;
}

int som_get_stats(som_ctx *c, int64_t *out) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!out) return fail(c, SOM_ERR_INVALID_ARG, "out is NULL");
  int32_t h[3] = {0, 0, 0};
  hipError_t e = hipMemcpyAsync(h, c->list_counts, sizeof(h), hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return dev_fail(c, e, "som_get_stats");
  out[0] = h[0];
  out[1] = h[1];
  out[2] = h[2];
  return SOM_OK;
}

int som_two_level_stats(som_ctx *c, int64_t *out) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!out) return fail(c, SOM_ERR_INVALID_ARG, "out is NULL");
  out[0] = out[1] = 0;
  if (c->two_level_n <= 0) return SOM_OK;
  const int64_t tiles = (c->two_level_n + 127) / 128;
  std::vector<int32_t> h((size_t)tiles);
  hipError_t e = hipMemcpyAsync(h.data(), c->tile_cnt, (size_t)tiles * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return dev_fail(c, e, "som_two_level_stats");
  for (int32_t v : h) out[0] += v;
  out[1] = tiles * (int64_t)((c->k + 127) / 128);
  return SOM_OK;
}

int som_profile_enable(som_ctx *c, int on) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (on) {
    for (int s = 0; s < SOM_PROFILE_STAGES; ++s) {
      if (c->prof_ev[s]) continue;
      hipEvent_t *ev = (hipEvent_t *)calloc(2 * kProfMax, sizeof(hipEvent_t));
      if (!ev) return fail(c, SOM_ERR_ALLOC, "out of host memory");
      for (int e = 0; e < 2 * kProfMax; ++e) {
        hipError_t err = hipEventCreate(&ev[e]);
        if (err != hipSuccess) {
          for (int d = 0; d < e; ++d) (void)hipEventDestroy(ev[d]);
          free(ev);
          return dev_fail(c, err, "hipEventCreate");
        }
      }
      c->prof_ev[s] = ev;
    }
  }
  c->prof_on = on ? 1 : 0;
  return SOM_OK;
}

int som_profile_read(som_ctx *c, double *total_ms, int64_t *launches) {
  if (!c) return SOM_ERR_INVALID_ARG;
  if (!total_ms || !launches) return fail(c, SOM_ERR_INVALID_ARG, "NULL pointer argument");
  hipError_t e = hipStreamSynchronize(c->stream);
  if (e != hipSuccess) return dev_fail(c, e, "som_profile_read");
  for (int s = 0; s < SOM_PROFILE_STAGES; ++s) {
    double sum = 0.0;
    for (int b = 0; b < c->prof_used[s]; ++b) {
      float ms = 0.f;
      e = hipEventElapsedTime(&ms, c->prof_ev[s][2 * b], c->prof_ev[s][2 * b + 1]);
      if (e != hipSuccess) return dev_fail(c, e, "hipEventElapsedTime");
      sum += ms;
    }
    total_ms[s] = sum;
    launches[s] = c->prof_used[s];
    c->prof_used[s] = 0;
  }
  return SOM_OK;
}

}  // extern "C"
