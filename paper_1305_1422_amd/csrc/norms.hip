// Squared Euclidean norms of matrix rows (code-book nodes, dense instances, CSR instances).
//
// The BMU search ranks nodes by |w|^2 - 2 x.w (paper, "Parallelism": the GPU variant
// evaluates Euclidean distances through linear algebra); |w|^2 is recomputed every epoch,
// |x|^2 only bounds the rounding error of the fp32 scores.  One wavefront per row, fp64
// accumulation, so each fp32 result carries a single rounding.
#include "som_internal.hpp"

namespace som {

__global__ __launch_bounds__(256) void k_row_sqnorms(const float *__restrict__ A, int64_t nrows, int dim,
                                                     float *__restrict__ out32, double *__restrict__ out64,
                                                     unsigned *__restrict__ max_bits) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x / kWave);
  for (int64_t r = wave; r < nrows; r += nwaves) {
    const float *a = A + r * dim;
    double s = 0.0;
    for (int c = lane; c < dim; c += kWave) {
      double v = (double)a[c];
      s += v * v;
    }
    s = wave_sum(s);
    if (lane == 0) {
      float f = (float)s;
      out32[r] = f;
      if (out64) out64[r] = s;
      if (max_bits) atomicMax(max_bits, __float_as_uint(f));
    }
  }
}

__global__ __launch_bounds__(256) void k_csr_row_sqnorms(const int64_t *__restrict__ indptr,
                                                         const float *__restrict__ values, int64_t n,
                                                         float *__restrict__ out32) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x / kWave);
  for (int64_t r = wave; r < n; r += nwaves) {
    double s = 0.0;
    for (int64_t p = indptr[r] + lane; p < indptr[r + 1]; p += kWave) {
      double v = (double)values[p];
      s += v * v;
    }
    s = wave_sum(s);
    if (lane == 0) out32[r] = (float)s;
  }
}

__global__ void k_zero_u32(unsigned *p, int64_t count) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) p[i] = 0u;
}

static int grid_for_waves(const som_ctx *c, int64_t nrows) {
  int64_t blocks = (nrows + 3) / 4;
  int64_t cap = (int64_t)c->n_cu * 32;
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

hipError_t launch_fill_zero_u32(hipStream_t s, void *p, int64_t count_u32) {
  if (count_u32 <= 0) return hipSuccess;
  int64_t blocks = (count_u32 + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(k_zero_u32, dim3((unsigned)blocks), dim3(256), 0, s, (unsigned *)p, count_u32);
  return hipGetLastError();
}

hipError_t launch_row_sqnorms(som_ctx *c, const float *A, int64_t nrows, int dim, float *out32,
                              double *out64, unsigned *max_bits) {
  if (max_bits) {
    hipError_t e = launch_fill_zero_u32(c->stream, max_bits, 1);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k_row_sqnorms, dim3(grid_for_waves(c, nrows)), dim3(256), 0, c->stream, A, nrows, dim,
                     out32, out64, max_bits);
  return hipGetLastError();
}

hipError_t launch_csr_row_sqnorms(som_ctx *c, const int64_t *indptr, const float *values, int64_t n,
                                  float *out32) {
  hipLaunchKernelGGL(k_csr_row_sqnorms, dim3(grid_for_waves(c, n)), dim3(256), 0, c->stream, indptr,
                     values, n, out32);
  return hipGetLastError();
}

}  // namespace som
