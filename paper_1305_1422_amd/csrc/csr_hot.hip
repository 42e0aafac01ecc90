// Sparse best-matching-unit search: the frequent columns as a dense block (paper: sparse kernel;
// BMU equation; "Parallelism": distances through linear algebra).
//
// The column frequencies of a text-like vector space are heavily skewed: on the stated sparse
// workload the 256 most frequent of 50,000 columns hold 48 % of the nonzeros.  A gather sweep
// (bmu_csr.hip) pays for every (nonzero, node) pair with a 2-byte load through L2, a conversion and a
// multiply-add on the vector units, however often the same code-book rows are asked for.  For a
// REGISTERED sparse training set the library therefore splits the columns once:
//   - the kHot most frequent columns become a dense block X_hot [n][kHot], kept as the fp16 hi/lo
//     planes of the dense filter (split_f16.hip); every epoch the same columns of the centred code
//     book are gathered into planes of their own, and the dot products x_hot . w'_hot of ALL
//     (instance, node) pairs are one split-fp16 matrix-core contraction (bmu_dense_h.hip, partial
//     mode) that leaves them in a table P [blocks of 128 nodes][n][128];
//   - the other columns stay a CSR set (the "tail": same rows, fewer nonzeros), and the gather sweep
//     runs over the tail only, starting its per-node sums from P instead of 0.
// The exact stage is untouched: it evaluates distances on the caller's full rows.  The hot block is
// fp32-grade (22-bit operands), so it adds only a rounding term to the margin and takes its columns'
// share out of the 16-bit quantisation term (bmu_exact.hip).
// The split is used only if it pays: at least kHotMinShare of the nonzeros in the hot columns.
//
// Everything here except the choice of the columns runs on the device; the choice itself (the kHot
// largest of dim counters) is made on the host from a copy of the counters, once per registration.
#include "som_internal.hpp"

#include <math.h>

#include <algorithm>
#include <vector>

namespace som {

__global__ __launch_bounds__(256) void k_hot_histogram(const int32_t *__restrict__ indices, int64_t nnz, int dim,
                                                       int32_t *__restrict__ counts) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
    const int c = indices[p];
    if (c >= 0 && c < dim) atomicAdd(&counts[c], 1);
  }
}

// Nonzeros of every row outside the hot columns (rank < 0).  One wavefront per row.
__global__ __launch_bounds__(256) void k_tail_lengths(const int64_t *__restrict__ indptr,
                                                      const int32_t *__restrict__ indices, int64_t n, int dim,
                                                      const int32_t *__restrict__ rank, int32_t *__restrict__ len) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  for (int64_t j = wave; j < n; j += nwaves) {
    int cnt = 0;
    for (int64_t p = indptr[j] + lane; p < indptr[j + 1]; p += 64) {
      int c = indices[p];
      c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
      cnt += rank[c] < 0 ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o, 64);
    if (lane == 0) len[j] = cnt;
  }
}

// Tail rows (order of the nonzeros kept) and the hot part of every row as fp16 hi/lo planes with a
// power-of-two scale per row, in the layout of split_f16.hip: chunk t of a row = 32 hi halves of
// columns 32 t .., then their 32 lo halves.  Also |x_hot|^2 per row.  One wavefront per row; the dense
// hot row is assembled in LDS.
__global__ __launch_bounds__(256) void k_split_hot_tail(const int64_t *__restrict__ indptr,
                                                        const int32_t *__restrict__ indices,
                                                        const float *__restrict__ values, int64_t n, int dim,
                                                        const int32_t *__restrict__ rank,
                                                        const int32_t *__restrict__ tail_start,
                                                        int64_t *__restrict__ tail_indptr,
                                                        int32_t *__restrict__ tail_indices,
                                                        float *__restrict__ tail_values,
                                                        _Float16 *__restrict__ planes, float *__restrict__ xscale,
                                                        float *__restrict__ xn_hot) {
  __shared__ float row[4][kHot];
  const int lane = threadIdx.x & 63;
  const int w = threadIdx.x >> 6;
  const int64_t wave = (int64_t)blockIdx.x * 4 + w;
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  for (int64_t j = wave; j < n; j += nwaves) {
    for (int h = lane; h < kHot; h += 64) row[w][h] = 0.f;
    __builtin_amdgcn_wave_barrier();
    const int64_t s = indptr[j], e = indptr[j + 1];
    int64_t out = tail_start[j];
    if (lane == 0) tail_indptr[j] = out;
    for (int64_t p0 = s; p0 < e; p0 += 64) {
      const int64_t p = p0 + lane;
      int c = 0, r = 0;
      float v = 0.f;
      bool tail = false;
      if (p < e) {
        c = indices[p];
        c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
        v = values[p];
        r = rank[c];
        tail = r < 0;
        if (!tail) row[w][r] = v;          // columns are unique within a row: no two lanes share a slot
      }
      const unsigned long long m = __ballot(tail);
      if (tail) {
        const int64_t at = out + __popcll(m & ((1ull << lane) - 1ull));
        tail_indices[at] = c;
        tail_values[at] = v;
      }
      out += __popcll(m);
    }
    __builtin_amdgcn_wave_barrier();
    float mx = 0.f;
    double nn = 0.0;
    for (int h = lane; h < kHot; h += 64) {
      const float v = row[w][h];
      mx = fmaxf(mx, fabsf(v));
      nn += (double)v * (double)v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    nn = wave_sum(nn);
    int ex = 0;
    if (mx > 0.f && mx < INFINITY) {
      (void)frexpf(mx, &ex);               // mx = f * 2^ex, f in [0.5, 1): 2^ex is a power of two above mx
      ex = ex < -100 ? -100 : (ex > 127 ? 127 : ex);
    }
    const float inv = ldexpf(1.f, -ex);
    if (lane == 0) {
      xscale[j] = ldexpf(1.f, ex);
      xn_hot[j] = (float)nn;
    }
    _Float16 *o = planes + j * (int64_t)(kHot * 2);
    for (int h = lane; h < kHot; h += 64) {
      const float v = row[w][h] * inv;
      const _Float16 hi = (_Float16)v;
      const _Float16 lo = (_Float16)(v - (float)hi);
      const int at = (h >> 5) * 64 + (h & 31);
      o[at] = hi;
      o[at + 32] = lo;
    }
    __builtin_amdgcn_wave_barrier();
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) tail_indptr[n] = tail_start[n];
}

// Hot columns of the centred code book, [k][kHot] fp32, and the largest magnitude among them
// (bit pattern, atomic maximum): the operand the split kernel turns into planes.
__global__ __launch_bounds__(256) void k_gather_hot_codebook(const float *__restrict__ W, const float *__restrict__ mu,
                                                             const int32_t *__restrict__ hot_cols, int k, int dim,
                                                             float *__restrict__ out, unsigned *__restrict__ max_bits) {
  float amax = 0.f;
  for (int h = threadIdx.x; h < kHot; h += 256) {
    const int c = hot_cols[h];
    const float m = mu[c];
    for (int i = blockIdx.x; i < k; i += gridDim.x) {
      const float t = W[(int64_t)i * dim + c] - m;
      out[(int64_t)i * kHot + h] = t;
      amax = fmaxf(amax, fabsf(t));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o, 64));
  if ((threadIdx.x & 63) == 0 && amax > 0.f) atomicMax(max_bits, __float_as_uint(amax));
}

// ---- dense planes of a registered sparse set of modest dimension (som_set_sparse_dense_filter)
// Column sums of the nonzeros (fp32 atomics: the result is only used as a centring vector, any vector
// serves) and rows written out densely, zeros included, for the kernels that split dense rows into planes.
__global__ __launch_bounds__(256) void k_csr_col_sums(const int32_t *__restrict__ indices, const float *__restrict__ values,
                                                      int64_t nnz, int dim, float *__restrict__ sums) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
    const int c = indices[p];
    if (c >= 0 && c < dim) unsafeAtomicAdd(&sums[c], values[p]);
  }
}

__global__ __launch_bounds__(256) void k_scale_vector(float *__restrict__ v, int len, float factor) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < len) v[i] *= factor;
}

// One workgroup per row: clear, then add the nonzeros in (indices outside [0, dim) are clamped as everywhere;
// a column listed twice counts twice, as in the sweep).
__global__ __launch_bounds__(256) void k_csr_densify(const int64_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                     const float *__restrict__ values, int64_t row0, int64_t nrows,
                                                     int dim, float *__restrict__ out) {
  for (int64_t r = blockIdx.x; r < nrows; r += gridDim.x) {
    float *o = out + r * dim;
    for (int c = threadIdx.x; c < dim; c += 256) o[c] = 0.f;
    __syncthreads();
    for (int64_t p = indptr[row0 + r] + threadIdx.x; p < indptr[row0 + r + 1]; p += 256) {
      int c = indices[p];
      c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
      unsafeAtomicAdd(&o[c], values[p]);
    }
    __syncthreads();
  }
}

hipError_t launch_csr_col_sums(som_ctx *c, const int32_t *indices, const float *values, int64_t nnz, float *sums) {
  hipError_t e = launch_fill_zero_u32(c->stream, sums, c->dim);
  if (e != hipSuccess || nnz < 1) return e;
  int64_t blocks = (nnz + 255) / 256;
  if (blocks > (int64_t)c->n_cu * 8) blocks = (int64_t)c->n_cu * 8;
  hipLaunchKernelGGL(k_csr_col_sums, dim3((unsigned)blocks), dim3(256), 0, c->stream, indices, values, nnz, c->dim, sums);
  return hipGetLastError();
}

hipError_t launch_scale_vector(som_ctx *c, float *v, int len, float factor) {
  hipLaunchKernelGGL(k_scale_vector, dim3((len + 255) / 256), dim3(256), 0, c->stream, v, len, factor);
  return hipGetLastError();
}

hipError_t launch_csr_densify(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                              int64_t row0, int64_t nrows, float *out) {
  int64_t blocks = nrows < (int64_t)c->n_cu * 16 ? nrows : (int64_t)c->n_cu * 16;
  if (blocks < 1) return hipSuccess;
  hipLaunchKernelGGL(k_csr_densify, dim3((unsigned)blocks), dim3(256), 0, c->stream, indptr, indices, values, row0,
                     nrows, c->dim, out);
  return hipGetLastError();
}

static_assert(kHot % 256 == 0, "k_gather_hot_codebook deals the hot columns to 256 threads");

hipError_t launch_hot_histogram(som_ctx *c, const int32_t *indices, int64_t nnz, int32_t *counts) {
  hipError_t e = launch_fill_zero_u32(c->stream, counts, c->dim);
  if (e != hipSuccess || nnz < 1) return e;
  int64_t blocks = (nnz + 255) / 256;
  if (blocks > (int64_t)c->n_cu * 8) blocks = (int64_t)c->n_cu * 8;
  hipLaunchKernelGGL(k_hot_histogram, dim3((unsigned)blocks), dim3(256), 0, c->stream, indices, nnz, c->dim, counts);
  return hipGetLastError();
}

// The kHot columns with the most nonzeros (ties: lower column first), ascending by column; returns the
// number of nonzeros they hold.  Host code: a selection among dim counters, once per registration.
int64_t choose_hot_columns(const std::vector<int32_t> &counts, std::vector<int32_t> &cols) {
  const int dim = (int)counts.size();
  std::vector<int32_t> order(dim);
  for (int i = 0; i < dim; ++i) order[i] = i;
  const int take = dim < kHot ? dim : kHot;
  std::partial_sort(order.begin(), order.begin() + take, order.end(), [&](int32_t a, int32_t b) {
    return counts[a] != counts[b] ? counts[a] > counts[b] : a < b;
  });
  cols.assign(order.begin(), order.begin() + take);
  std::sort(cols.begin(), cols.end());
  int64_t held = 0;
  for (int32_t col : cols) held += counts[col];
  return held;
}

hipError_t launch_tail_lengths(som_ctx *c, const int64_t *indptr, const int32_t *indices, int64_t n, int32_t *len) {
  int64_t blocks = (n + 3) / 4;
  if (blocks > (int64_t)c->n_cu * 16) blocks = (int64_t)c->n_cu * 16;
  hipLaunchKernelGGL(k_tail_lengths, dim3((unsigned)blocks), dim3(256), 0, c->stream, indptr, indices, n, c->dim,
                     c->hot_rank, len);
  return hipGetLastError();
}

hipError_t launch_split_hot_tail(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                                 int64_t n) {
  int64_t blocks = (n + 3) / 4;
  if (blocks > (int64_t)c->n_cu * 16) blocks = (int64_t)c->n_cu * 16;
  hipLaunchKernelGGL(k_split_hot_tail, dim3((unsigned)blocks), dim3(256), 0, c->stream, indptr, indices, values, n,
                     c->dim, c->hot_rank, c->tail_start, c->tail_indptr, c->tail_indices, c->tail_values, c->hot_Xh,
                     c->hot_xscale, c->hot_xn);
  return hipGetLastError();
}

hipError_t launch_gather_hot_codebook(som_ctx *c, const float *W) {
  hipError_t e = launch_fill_zero_u32(c->stream, c->hot_wmax_bits, 1);
  if (e != hipSuccess) return e;
  const int blocks = c->k < c->n_cu * 4 ? c->k : c->n_cu * 4;
  hipLaunchKernelGGL(k_gather_hot_codebook, dim3(blocks), dim3(256), 0, c->stream, W, c->mu, c->hot_cols, c->k,
                     c->dim, c->hot_Wc, c->hot_wmax_bits);
  return hipGetLastError();
}

}  // namespace som
