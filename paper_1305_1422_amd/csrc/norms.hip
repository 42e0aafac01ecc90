// Squared Euclidean norms of matrix rows (code-book nodes, dense instances, CSR instances) and
// the centring vector of the dense BMU search.
//
// The BMU search ranks nodes by |w|^2 - 2 x.w (paper, "Parallelism": the GPU variant
// evaluates Euclidean distances through linear algebra).  Distances do not change when the
// same vector mu is subtracted from instances and nodes, and
//     |x - w|^2 - |x - mu|^2 = |w'|^2 + 2 mu.w' - 2 x.w',   w' = w - mu,
// so the dense path multiplies the raw instances with the CENTRED code book: the rounding
// error of the fp32 scores then scales with |x| |w - mu| instead of |x| |w|.  mu is the mean
// of a sample of the instances.  Every epoch k_center_codebook writes w' = fl(w - mu) and the
// per-node constants c_i = |w'_i|^2 + 2 mu.w'_i (of the rounded w', in fp64, rounded once).
// The split-fp16 filter reads the instances from planes of the library's own, which hold
// x' = fl(x - mu): there the scores are |w'_i|^2 - 2 x'.w'_i and their error scales with |x - mu|.
// |x|^2 and |mu|^2 only bound the rounding error.  One wavefront per row, fp64 accumulation.
#include "som_internal.hpp"

namespace som {

__global__ __launch_bounds__(256) void k_row_sqnorms(const float *__restrict__ A, int64_t nrows, int dim,
                                                     const float *__restrict__ mu, float *__restrict__ out32,
                                                     double *__restrict__ out64,
                                                     unsigned *__restrict__ max_bits) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t wave = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x / kWave);
  for (int64_t r = wave; r < nrows; r += nwaves) {
    const float *a = A + r * dim;
    double s = 0.0;
    if (mu) {
      for (int c = lane; c < dim; c += kWave) {
        const float t = a[c] - mu[c];          // fp32 difference, as staged by the BMU kernel
        s += (double)t * (double)t;
      }
    } else {
      for (int c = lane; c < dim; c += kWave) {
        double v = (double)a[c];
        s += v * v;
      }
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

// Sum of three doubles over a 256-thread workgroup, in a fixed order; result valid in thread 0.
__device__ __forceinline__ void block_sum3(double &a, double &b, double &c, double (*scratch)[3]) {
  a = wave_sum(a);
  b = wave_sum(b);
  c = wave_sum(c);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  if (lane == 0) { scratch[wave][0] = a; scratch[wave][1] = b; scratch[wave][2] = c; }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = (scratch[0][0] + scratch[1][0]) + (scratch[2][0] + scratch[3][0]);
    b = (scratch[0][1] + scratch[1][1]) + (scratch[2][1] + scratch[3][1]);
    c = (scratch[0][2] + scratch[1][2]) + (scratch[2][2] + scratch[3][2]);
  }
  __syncthreads();
}

// w' = fl(w - mu) (stored if Wc is given), c_i = |w'_i|^2 + 2 mu.w'_i, the maximum of |w'_i|^2
// over the nodes, and optionally |w_i|^2 of the uncentred rows in fp64.  kTeam threads per node:
// a wavefront for short rows, the whole workgroup for long ones.  Every writer thread keeps its
// own running maximum and issues one atomic at the end.
template <int kTeam>
__global__ __launch_bounds__(256) void k_center_codebook(const float *__restrict__ W, int k, int dim,
                                                         const float *__restrict__ mu, float *__restrict__ Wc,
                                                         float *__restrict__ cn, unsigned *__restrict__ max_bits,
                                                         double *__restrict__ wn64,
                                                         unsigned *__restrict__ wabs_bits, int x_centered) {
  __shared__ double scratch[4][3];
  constexpr int kTeams = 256 / kTeam;
  const int tl = threadIdx.x % kTeam, team = threadIdx.x / kTeam;
  float vmax = 0.f;
  float amax = 0.f;                  // largest |w'| element this thread has seen
  for (int i = blockIdx.x * kTeams + team; i < k; i += gridDim.x * kTeams) {
    const float *w = W + (int64_t)i * dim;
    float *wc = Wc ? Wc + (int64_t)i * dim : nullptr;
    double s2 = 0.0, sm = 0.0, sw = 0.0;
    int c = tl;
    for (; c + 3 * kTeam < dim; c += 4 * kTeam) {        // four independent loads in flight per thread
      float m[4], x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { m[u] = mu[c + u * kTeam]; x[u] = w[c + u * kTeam]; }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float t = x[u] - m[u];
        if (Wc) wc[c + u * kTeam] = t;
        amax = fmaxf(amax, fabsf(t));
        s2 += (double)t * (double)t;
        sm += (double)m[u] * (double)t;
        sw += (double)x[u] * (double)x[u];
      }
    }
    for (; c < dim; c += kTeam) {
      const float m = mu[c];
      const float x = w[c];
      const float t = x - m;
      if (Wc) wc[c] = t;
      amax = fmaxf(amax, fabsf(t));
      s2 += (double)t * (double)t;
      sm += (double)m * (double)t;
      sw += (double)x * (double)x;
    }
    if (kTeam == 256) {
      block_sum3(s2, sm, sw, scratch);     // i depends on the block only: every thread gets here
    } else {
      s2 = wave_sum(s2);
      sm = wave_sum(sm);
      sw = wave_sum(sw);
    }
    if (tl == 0) {
      cn[i] = (float)(x_centered ? s2 : s2 + 2.0 * sm);      // instances centred too: |w'|^2 - 2 x'.w' ranks alike
      vmax = fmaxf(vmax, (float)s2);
      if (wn64) wn64[i] = sw;
    }
  }
  // one pair of atomics per workgroup: thousands of atomics on one address would cost more than
  // the rest of the kernel
  __shared__ float smax[2][4];
  if (tl != 0) vmax = 0.f;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    vmax = fmaxf(vmax, __shfl_xor(vmax, o, 64));
    amax = fmaxf(amax, __shfl_xor(amax, o, 64));
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { smax[0][threadIdx.x >> 6] = vmax; smax[1][threadIdx.x >> 6] = amax; }
  __syncthreads();
  if (threadIdx.x == 0) {
    vmax = fmaxf(fmaxf(smax[0][0], smax[0][1]), fmaxf(smax[0][2], smax[0][3]));
    amax = fmaxf(fmaxf(smax[1][0], smax[1][1]), fmaxf(smax[1][2], smax[1][3]));
    if (vmax > 0.f) atomicMax(max_bits, __float_as_uint(vmax));
    if (wabs_bits && amax > 0.f) atomicMax(wabs_bits, __float_as_uint(amax));
  }
}

// |v|^2 of one vector, one workgroup of 1024 threads, fixed summation order.
__global__ __launch_bounds__(1024) void k_vec_sqnorm(const float *__restrict__ v, int dim, float *__restrict__ out) {
  __shared__ double part[16];
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  int c = threadIdx.x;
  for (; c + 3072 < dim; c += 4096) {
    const float a = v[c], b = v[c + 1024], d = v[c + 2048], e = v[c + 3072];
    s0 += (double)a * (double)a;
    s1 += (double)b * (double)b;
    s2 += (double)d * (double)d;
    s3 += (double)e * (double)e;
  }
  for (; c < dim; c += 1024) s0 += (double)v[c] * (double)v[c];
  const double s = wave_sum((s0 + s1) + (s2 + s3));
  if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int w = 0; w < 16; ++w) t += part[w];
    *out = (float)t;
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

// Column means of a strided sample of the rows, in two steps: kMeanSlabs partial sums per column,
// then their total.  Any mu is valid for the search (the error bound uses the norms actually
// obtained), so a sample of up to 8192 rows is enough.  fp64 sums in a fixed order: deterministic.
constexpr int kMeanSlabs = 64;
constexpr int kMeanRowsPerSlab = 128;

// With `range` the slab minima and maxima of every column are recorded too ([2][slabs][dim]).
constexpr int kColBlock = 256;      // columns per workgroup: a kilobyte of every row it visits

__global__ __launch_bounds__(kColBlock) void k_sample_col_sums(const float *__restrict__ A, int64_t nsample,
                                                        int64_t stride, int dim, double *__restrict__ partial,
                                                        float *__restrict__ range) {
  const int c = blockIdx.x * kColBlock + threadIdx.x;
  if (c >= dim) return;
  const int64_t per = (nsample + kMeanSlabs - 1) / kMeanSlabs;
  const int64_t t0 = blockIdx.y * per;
  const int64_t t1 = t0 + per < nsample ? t0 + per : nsample;
  double s = 0.0;
  float lo = INFINITY, hi = -INFINITY;
  int64_t t = t0;
  for (; t + 4 <= t1; t += 4) {                 // four rows in flight per thread
    float a[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) a[u] = A[(t + u) * stride * dim + c];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      s += (double)a[u];
      lo = fminf(lo, a[u]);
      hi = fmaxf(hi, a[u]);
    }
  }
  for (; t < t1; ++t) {
    const float a = A[t * stride * dim + c];
    s += (double)a;
    lo = fminf(lo, a);
    hi = fmaxf(hi, a);
  }
  partial[(int64_t)blockIdx.y * dim + c] = s;
  if (range) {
    range[(int64_t)blockIdx.y * dim + c] = lo;
    range[((int64_t)kMeanSlabs + blockIdx.y) * dim + c] = hi;
  }
}

// Column means; with `range` (which must then cover ALL rows) also the 16-bit quantisation step of
// every column of the centred matrix: step_c = max_i |a_ic - mu_c| / 32767 with a little slack, so
// that a_ic - mu_c, rounded to fp32, divided by the step and rounded to an integer fits an int16;
// and the largest step (atomic maximum on the bit pattern).
__global__ __launch_bounds__(64) void k_finish_col_means(const double *__restrict__ partial, int64_t nsample,
                                                         int dim, float *__restrict__ mu,
                                                         const float *__restrict__ range, float *__restrict__ qstep,
                                                         unsigned *__restrict__ qstep_max_bits) {
  const int c = blockIdx.x * 64 + threadIdx.x;
  float step = 0.f;
  if (c < dim) {
    double s = 0.0;
    for (int b = 0; b < kMeanSlabs; ++b) s += partial[(int64_t)b * dim + c];
    const float m = (float)(s / (double)nsample);
    mu[c] = m;
    if (range) {
      float lo = INFINITY, hi = -INFINITY;
      for (int b = 0; b < kMeanSlabs; ++b) {
        lo = fminf(lo, range[(int64_t)b * dim + c]);
        hi = fmaxf(hi, range[((int64_t)kMeanSlabs + b) * dim + c]);
      }
      const double amax = fmax((double)hi - (double)m, (double)m - (double)lo);
      step = amax > 0.0 && amax < 1e300 ? (float)(amax * (1.0 + 1e-6) / 32767.0) : 0.f;
      if (!(step > 0.f)) step = 1e-30f;          // constant column (or no rows): every quotient is 0, and the
                                                 // column must not weigh on the quantisation term of the margin
      qstep[c] = step;
    }
  }
  if (range) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) step = fmaxf(step, __shfl_xor(step, o, 64));
    if (threadIdx.x == 0 && step > 0.f) atomicMax(qstep_max_bits, __float_as_uint(step));
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

hipError_t launch_sample_col_means(som_ctx *c, const float *A, int64_t nrows, int dim, float *mu) {
  const int64_t cap = (int64_t)kMeanSlabs * kMeanRowsPerSlab;
  const int64_t nsample = nrows < cap ? nrows : cap;
  const int64_t stride = nrows / nsample;
  hipLaunchKernelGGL(k_sample_col_sums, dim3((dim + kColBlock - 1) / kColBlock, kMeanSlabs), dim3(kColBlock), 0, c->stream, A, nsample,
                     stride, dim, c->mu_partial, (float *)nullptr);
  hipLaunchKernelGGL(k_finish_col_means, dim3((dim + 63) / 64), dim3(64), 0, c->stream, c->mu_partial, nsample,
                     dim, mu, (const float *)nullptr, (float *)nullptr, (unsigned *)nullptr);
  return hipGetLastError();
}

// Means of ALL rows of the code book (at most kMeanSlabs * kMeanRowsPerSlab of them) plus the
// quantisation steps of its centred columns: c->mu, c->qstep, c->qstep_max_bits.
hipError_t launch_codebook_means_and_steps(som_ctx *c, const float *W) {
  hipError_t e = launch_fill_zero_u32(c->stream, c->qstep_max_bits, 1);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_sample_col_sums, dim3((c->dim + kColBlock - 1) / kColBlock, kMeanSlabs), dim3(kColBlock), 0, c->stream, W,
                     (int64_t)c->k, (int64_t)1, c->dim, c->mu_partial, c->col_range);
  hipLaunchKernelGGL(k_finish_col_means, dim3((c->dim + 63) / 64), dim3(64), 0, c->stream, c->mu_partial,
                     (int64_t)c->k, c->dim, c->mu, c->col_range, c->qstep, c->qstep_max_bits);
  return hipGetLastError();
}

hipError_t launch_vec_sqnorm(som_ctx *c, const float *v, int dim, float *out) {
  hipLaunchKernelGGL(k_vec_sqnorm, dim3(1), dim3(1024), 0, c->stream, v, dim, out);
  return hipGetLastError();
}

hipError_t launch_center_codebook(som_ctx *c, const float *W, bool store_centered, bool want_wn64, bool x_centered) {
  hipError_t e = launch_fill_zero_u32(c->stream, c->wmax_bits, 2);     // wmax_bits and wabs_bits are neighbours
  if (e != hipSuccess) return e;
  float *wc = store_centered ? c->Wc : nullptr;
  unsigned *wabs = store_centered ? c->wmax_bits + 1 : nullptr;
  double *wn64 = want_wn64 ? c->wn64 : nullptr;
  const int cap = c->n_cu * 2;
  if (c->dim <= 2048) {
    const int need = (c->k + 3) / 4;
    hipLaunchKernelGGL(k_center_codebook<64>, dim3(need < cap ? need : cap), dim3(256), 0, c->stream, W, c->k, c->dim,
                       c->mu, wc, c->wn32, c->wmax_bits, wn64, wabs, x_centered ? 1 : 0);
  } else {
    const int cap_long = c->n_cu * 8;       // long rows: more workgroups in flight, still few atomics
    hipLaunchKernelGGL(k_center_codebook<256>, dim3(c->k < cap_long ? c->k : cap_long), dim3(256), 0, c->stream, W, c->k, c->dim,
                       c->mu, wc, c->wn32, c->wmax_bits, wn64, wabs, x_centered ? 1 : 0);
  }
  return hipGetLastError();
}

hipError_t launch_row_sqnorms(som_ctx *c, const float *A, int64_t nrows, int dim, const float *mu, float *out32,
                              double *out64, unsigned *max_bits) {
  if (max_bits) {
    hipError_t e = launch_fill_zero_u32(c->stream, max_bits, 1);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k_row_sqnorms, dim3(grid_for_waves(c, nrows)), dim3(256), 0, c->stream, A, nrows, dim,
                     mu, out32, out64, max_bits);
  return hipGetLastError();
}

hipError_t launch_csr_row_sqnorms(som_ctx *c, const int64_t *indptr, const float *values, int64_t n,
                                  float *out32) {
  hipLaunchKernelGGL(k_csr_row_sqnorms, dim3(grid_for_waves(c, n)), dim3(256), 0, c->stream, indptr,
                     values, n, out32);
  return hipGetLastError();
}

}  // namespace som
