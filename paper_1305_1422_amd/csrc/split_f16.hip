// fp32 rows as two fp16 planes, for the BMU filter that runs on the fp16 matrix cores
// (paper: BMU equation; "Parallelism": distances through linear algebra).
//
// A row v is divided by a power of two s > max|v_c| (so |v/s| < 1: no fp16 overflow, and the
// division is exact), then every element is written as hi + lo with
//     hi = fp16(v/s),   lo = fp16(v/s - hi)     (both round-to-nearest; the subtraction is exact)
// which leaves |v/s - hi - lo| <= max(2^-22 |v/s|, 2^-25): fp16 keeps 11 significant bits and its
// subnormals end at 2^-24 (the matrix cores honour subnormal inputs).  The product of two such
// numbers is hi*hi' + hi*lo' + lo*hi' up to 3 * 2^-22 relative: three fp16 MFMAs give an fp32-grade
// dot product at a third of the fp16 rate, which is still more than five times the fp32 MFMA rate.
//
// Storage: rows are padded to whole chunks of 32 columns, and chunk t of a row is 128 bytes:
// the 32 hi halves of columns 32 t .. 32 t + 31, then their 32 lo halves.  That is exactly the
// shape of one LDS tile row of the filter kernel (bmu_dense_h.hip).  Padding columns are zero.
// The coarse pass of the two-level search reads the hi halves alone: a second copy, rows padded to
// whole chunks of 64 columns, 128 bytes per chunk again.
#include "som_internal.hpp"

#include <math.h>

namespace som {

// Power of two strictly above m (1 for m = 0 or a non-finite m), exponent kept inside fp32's range.
__device__ __forceinline__ float pow2_above(float m, float *inverse) {
  int e = 0;
  if (m > 0.f && m < INFINITY) {
    (void)frexpf(m, &e);          // m = f * 2^e, f in [0.5, 1)
    e = e < -100 ? -100 : (e > 127 ? 127 : e);
  }
  *inverse = ldexpf(1.f, -e);
  return ldexpf(1.f, e);
}

// kTeam threads per row (a wavefront for short rows, the workgroup for long ones).  With
// `global_max_bits` every row uses the same scale (the code book: one factor for all nodes, so
// that the scores of an instance stay comparable without a per-node multiplication) and the
// scale is also written to *scale_out; without it each row gets its own scale in scale_out[row].
// With `mu` the rows are centred first, a_c - mu_c in fp32 (the instances of the dense search: their
// scores then carry |x - mu| instead of |x| in the rounding bound).
template <int kTeam>
__global__ __launch_bounds__(256) void k_split_rows_f16(const float *__restrict__ A, int64_t nrows, int dim, int nK,
                                                        const unsigned *__restrict__ global_max_bits,
                                                        const float *__restrict__ mu,
                                                        _Float16 *__restrict__ out, float *__restrict__ scale_out,
                                                        _Float16 *__restrict__ out_hi) {
  __shared__ float smax[4];
  constexpr int kTeams = 256 / kTeam;
  const int tl = threadIdx.x % kTeam, team = threadIdx.x / kTeam;
  const int padded = nK * 32;
  const int padded_hi = (nK + 1) / 2 * 64;
  for (int64_t r = (int64_t)blockIdx.x * kTeams + team; r < nrows; r += (int64_t)gridDim.x * kTeams) {
    const float *a = A + r * dim;
    float m;
    if (global_max_bits) {
      m = __uint_as_float(*global_max_bits);
    } else {
      m = 0.f;
      for (int c = tl; c < dim; c += kTeam) m = fmaxf(m, fabsf(mu ? a[c] - mu[c] : a[c]));
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
      if (kTeam == 256) {          // r depends on the block only: every thread gets here
        __syncthreads();
        if ((threadIdx.x & 63) == 0) smax[threadIdx.x >> 6] = m;
        __syncthreads();
        m = fmaxf(fmaxf(smax[0], smax[1]), fmaxf(smax[2], smax[3]));
      }
    }
    float inv;
    const float s = pow2_above(m, &inv);
    if (tl == 0) {
      if (global_max_bits) { if (r == 0) *scale_out = s; }
      else scale_out[r] = s;
    }
    _Float16 *o = out + r * (int64_t)nK * 64;
    for (int c = tl; c < padded; c += kTeam) {
      const float v = c < dim ? (mu ? a[c] - mu[c] : a[c]) * inv : 0.f;
      const _Float16 hi = (_Float16)v;
      const _Float16 lo = (_Float16)(v - (float)hi);
      const int at = (c >> 5) * 64 + (c & 31);
      o[at] = hi;
      o[at + 32] = lo;
      if (out_hi) out_hi[r * (int64_t)padded_hi + c] = hi;
    }
    if (out_hi && padded_hi > padded) {
      for (int c = padded + tl; c < padded_hi; c += kTeam) out_hi[r * (int64_t)padded_hi + c] = (_Float16)0.f;
    }
  }
}

hipError_t launch_split_rows_f16(som_ctx *c, const float *A, int64_t nrows, const unsigned *global_max_bits,
                                 const float *mu, _Float16 *out, float *scale_out, int dim, _Float16 *out_hi) {
  if (dim <= 0) dim = c->dim;
  const int nK = (dim + 31) / 32;
  const int64_t cap = (int64_t)c->n_cu * 16;
  if (dim <= 2048) {
    int64_t blocks = (nrows + 3) / 4;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(k_split_rows_f16<64>, dim3((unsigned)blocks), dim3(256), 0, c->stream, A, nrows, dim, nK,
                       global_max_bits, mu, out, scale_out, out_hi);
  } else {
    int64_t blocks = nrows < cap ? nrows : cap;
    hipLaunchKernelGGL(k_split_rows_f16<256>, dim3((unsigned)blocks), dim3(256), 0, c->stream, A, nrows, dim, nK,
                       global_max_bits, mu, out, scale_out, out_hi);
  }
  return hipGetLastError();
}

// One v_mfma_f32_32x32x16_f16 on caller-given operands: D = A B^T + C with A [32][16] and
// B [32][16] fp16 bit patterns, C and D [32][32] fp32.  Exists so that a test can check the
// rounding behaviour that the error bound of the filter assumes of this instruction.
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(64) void k_probe_mfma_f16(const _Float16 *__restrict__ A, const _Float16 *__restrict__ B,
                                                       const float *__restrict__ C, float *__restrict__ D,
                                                       int count) {
  const int l = threadIdx.x;
  for (int t = blockIdx.x; t < count; t += gridDim.x) {
    const _Float16 *a = A + (int64_t)t * 512, *b = B + (int64_t)t * 512;
    const float *cc = C + (int64_t)t * 1024;
    float *d = D + (int64_t)t * 1024;
    f16x8_t av, bv;
#pragma unroll
    for (int v = 0; v < 8; ++v) {
      av[v] = a[(l & 31) * 16 + (l >> 5) * 8 + v];
      bv[v] = b[(l & 31) * 16 + (l >> 5) * 8 + v];
    }
    f32x16_t acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = cc[(8 * (v >> 2) + 4 * (l >> 5) + (v & 3)) * 32 + (l & 31)];
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, acc, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 16; ++v) d[(8 * (v >> 2) + 4 * (l >> 5) + (v & 3)) * 32 + (l & 31)] = acc[v];
  }
}

hipError_t launch_probe_mfma_f16(hipStream_t stream, const uint16_t *A, const uint16_t *B, const float *C, float *D,
                                 int count) {
  hipLaunchKernelGGL(k_probe_mfma_f16, dim3((unsigned)(count < 1024 ? count : 1024)), dim3(64), 0, stream,
                     reinterpret_cast<const _Float16 *>(A), reinterpret_cast<const _Float16 *>(B), C, D, count);
  return hipGetLastError();
}

}  // namespace som
