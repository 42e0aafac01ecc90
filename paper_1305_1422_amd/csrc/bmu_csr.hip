// Sparse best-matching-unit search, fp32 pass (paper: sparse kernel - the code book stays
// dense while the data are index:value lists; BMU equation).
//
// As in the dense path the nodes are ranked by s_i = c_i - 2 x.w'_i with w' = w - mu and
// c_i = |w'_i|^2 + 2 mu.w'_i (identical ranking to |x - w_i|^2, smaller rounding error); x stays
// sparse, so x.w'_i = sum_nz v * w'_i[c].  mu is the mean of the code-book rows here.  The
// centred code book is written transposed, Wt[dim][kpad], so that one nonzero (c, v) touches
// one contiguous row of Wt: a workgroup owns an instance, its 256 threads own nodes t, t+256,
// ... and every nonzero is one coalesced sweep over the node range with v broadcast from LDS.
// The scores of an instance never leave registers.
//
// The fp32 scores only filter: the workgroup finds the minimum, then the nodes whose score
// lies within the rounding-error bound of it.  One such node: decided.  Up to kCand: handed to
// the exact refine pass.  Up to kListCap: stored as a collected list for the exact list pass.
// More: the instance is rescanned exactly.
#include "som_internal.hpp"

#include <math.h>

namespace som {

constexpr int kCsrUnroll = 4;      // nonzeros whose gathers are in flight together

// ---------------------------------------------------------------- transpose with centring
__global__ __launch_bounds__(256) void k_transpose_centered(const float *__restrict__ W,
                                                            const float *__restrict__ mu, int k, int dim, int kpad,
                                                            float *__restrict__ Wt) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
  const int c0 = blockIdx.x * 32, i0 = blockIdx.y * 32;
  for (int r = ty; r < 32; r += 8) {
    const int i = i0 + r, c = c0 + tx;
    tile[r][tx] = (i < k && c < dim) ? W[(int64_t)i * dim + c] - mu[c] : 0.f;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int c = c0 + r, i = i0 + tx;
    if (c < dim && i < kpad) Wt[(int64_t)c * kpad + i] = tile[tx][r];
  }
}

// The same transposition for the sliced kernel: entries as int16 multiples of the column's
// quantisation step, q = round((w - mu_c) / step_c), |q| <= 32767 by the choice of the step.
__global__ __launch_bounds__(256) void k_transpose_centered_q16(const float *__restrict__ W,
                                                                const float *__restrict__ mu,
                                                                const float *__restrict__ qstep, int k, int dim,
                                                                int kpad, int16_t *__restrict__ Wt) {
  __shared__ float tile[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
  const int c0 = blockIdx.x * 32, i0 = blockIdx.y * 32;
  for (int r = ty; r < 32; r += 8) {
    const int i = i0 + r, c = c0 + tx;
    float q = 0.f;
    if (i < k && c < dim) {
      q = rintf((W[(int64_t)i * dim + c] - mu[c]) / qstep[c]);
      q = fminf(fmaxf(q, -32767.f), 32767.f);
    }
    tile[r][tx] = q;
  }
  __syncthreads();
  for (int r = ty; r < 32; r += 8) {
    const int c = c0 + r, i = i0 + tx;
    if (c < dim && i < kpad) Wt[(int64_t)c * kpad + i] = (int16_t)tile[tx][r];
  }
}

// Error bound of one sparse fp32 score (see bmu_exact.hip): FMA chain of len terms, g = len.
__device__ __forceinline__ double csr_margin(double len, double xnorm2, double wmax2, double munorm2) {
  const double u = 5.9604644775390625e-08;   // 2^-24
  const double xn = sqrt(xnorm2 * (1.0 + 1.2e-7));
  const double wm = sqrt(wmax2 * (1.0 + 1.2e-7));
  const double mn = sqrt(munorm2 * (1.0 + 1.2e-7));
  const double g = len < 1.0 ? 1.0 : len;
  return 2.125 * u * ((2.0 * g + 4.0) * xn * wm + 4.0 * wm * wm + 6.0 * mn * wm);
}

struct CsrBmuOut {
  int32_t *bmus;
  int32_t *cand_idx, *cand_n, *refine_list;
  int32_t *collect_rows, *collect_cnt, *collect_list;
  int32_t *rescan_list;
  int32_t *list_counts;
};

template <int ACC>
__global__ __launch_bounds__(256) void k_bmu_csr(const int64_t *__restrict__ indptr,
                                                 const int32_t *__restrict__ indices,
                                                 const float *__restrict__ values, const float *__restrict__ Wt,
                                                 int kpad, const float *__restrict__ cn32,
                                                 const float *__restrict__ xn32,
                                                 const unsigned *__restrict__ wmax_bits,
                                                 const float *__restrict__ mu_norm2, int64_t n, int k, int dim,
                                                 CsrBmuOut out) {
  __shared__ int64_t s_off[256];
  __shared__ float s_val[256];
  __shared__ float s_min[4];
  __shared__ int s_cnt;
  __shared__ int s_list[kListCap];
  __shared__ int s_slot;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int span = 256 * ACC;                       // nodes covered by one sweep
  const int nsweep = (k + span - 1) / span;
  const float wmax2 = __uint_as_float(*wmax_bits);
  const float mu2 = *mu_norm2;

  for (int64_t j = blockIdx.x; j < n; j += gridDim.x) {
    const int64_t rs = indptr[j];
    const int len = (int)(indptr[j + 1] - rs);
    float sc[ACC];
    float lmin = INFINITY;
    float thr = 0.f;
    // phase 0 finds the minimum score, phase 1 collects the nodes within the margin of it;
    // with a single sweep the scores of phase 0 are still in registers for phase 1.
    for (int phase = 0; phase < 2; ++phase) {
      for (int sw = 0; sw < nsweep; ++sw) {
        const int node_base = sw * span + tid;
        if (phase == 0 || nsweep > 1) {
          float acc[ACC];
#pragma unroll
          for (int a = 0; a < ACC; ++a) acc[a] = 0.f;
          for (int p0 = 0; p0 < len; p0 += 256) {
            __syncthreads();
            if (p0 + tid < len) {
              int c = indices[rs + p0 + tid];
              c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
              s_off[tid] = (int64_t)c * kpad;
              s_val[tid] = values[rs + p0 + tid];
            }
            __syncthreads();
            const int m = min(256, len - p0);
            // four nonzeros per step: all their loads are issued before the first use, so that
            // enough bytes are in flight to cover the latency of the gathers
            int q = 0;
            for (; q + kCsrUnroll <= m; q += kCsrUnroll) {
              float w[kCsrUnroll][ACC];
#pragma unroll
              for (int u = 0; u < kCsrUnroll; ++u) {
                const float *wrow = Wt + s_off[q + u] + node_base;
#pragma unroll
                for (int a = 0; a < ACC; ++a) w[u][a] = (sw * span + a * 256 < kpad) ? wrow[a * 256] : 0.f;
              }
#pragma unroll
              for (int u = 0; u < kCsrUnroll; ++u) {
                const float v = s_val[q + u];
#pragma unroll
                for (int a = 0; a < ACC; ++a) acc[a] = fmaf(v, w[u][a], acc[a]);
              }
            }
            for (; q < m; ++q) {
              const float v = s_val[q];
              const float *wrow = Wt + s_off[q] + node_base;
#pragma unroll
              for (int a = 0; a < ACC; ++a)
                if (sw * span + a * 256 < kpad) acc[a] = fmaf(v, wrow[a * 256], acc[a]);
            }
          }
#pragma unroll
          for (int a = 0; a < ACC; ++a) {
            const int node = node_base + a * 256;
            sc[a] = node < k ? fmaf(-2.f, acc[a], cn32[node]) : INFINITY;
          }
        }
        if (phase == 0) {
#pragma unroll
          for (int a = 0; a < ACC; ++a) lmin = fminf(lmin, sc[a]);
        } else {
#pragma unroll
          for (int a = 0; a < ACC; ++a)
            if (sc[a] <= thr) {
              const int pos = atomicAdd(&s_cnt, 1);
              if (pos < kListCap) s_list[pos] = node_base + a * 256;
            }
        }
      }
      if (phase == 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) lmin = fminf(lmin, __shfl_xor(lmin, o, 64));
        __syncthreads();
        if (lane == 0) s_min[wave] = lmin;
        if (tid == 0) s_cnt = 0;
        __syncthreads();
        const float smin = fminf(fminf(s_min[0], s_min[1]), fminf(s_min[2], s_min[3]));
        const double t = (double)smin + csr_margin((double)len, (double)xn32[j], (double)wmax2, (double)mu2);
        // round the threshold up to fp32 so that no score inside the margin is lost
        thr = (float)t;
        if ((double)thr < t) thr = nextafterf(thr, INFINITY);
      }
    }
    __syncthreads();
    const int cnt = s_cnt;
    if (cnt == 1) {
      if (tid == 0) out.bmus[j] = s_list[0];
    } else if (cnt >= 2 && cnt <= kCand) {
      if (tid < cnt) out.cand_idx[j * kCand + tid] = s_list[tid];
      if (tid == 0) {
        out.cand_n[j] = cnt;
        out.refine_list[atomicAdd(&out.list_counts[0], 1)] = (int32_t)j;
      }
    } else if (cnt > kCand && cnt <= kListCap) {
      if (tid == 0) {
        s_slot = atomicAdd(&out.list_counts[1], 1);
        out.collect_rows[s_slot] = (int32_t)j;
        out.collect_cnt[s_slot] = cnt;
      }
      __syncthreads();
      if (tid < cnt) out.collect_list[(int64_t)s_slot * kListCap + tid] = s_list[tid];
    } else {
      if (tid == 0) out.rescan_list[atomicAdd(&out.list_counts[2], 1)] = (int32_t)j;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- node slices, one per XCD
// What bounds the kernel above is the traffic its gathers send past L2: a nonzero touches a whole
// row of Wt (4 kpad bytes), the popular columns of a Zipf-distributed vocabulary are few, and a 4 MB
// L2 holds only some hundred rows.  MI355X has eight L2s, one per XCD, and hands workgroup b to
// XCD b mod 8.  So the nodes are cut into eight slices and workgroup b only ever scores slice
// b mod 8: an XCD then touches an eighth of every row of Wt, its L2 holds eight times as many
// columns, and the instances are walked once per slice (their 8 bytes per nonzero are small
// change next to the 4 kpad / 8 bytes of the gather).
//
// A wavefront owns one (instance, slice) pair; lane l owns nodes slice0 + l + 64 a.  The nonzeros of
// the row are read 64 at a time, one per lane, and handed round with v_readlane: column and value
// of the current nonzero live in scalar registers, so the gathers are "scalar base + lane offset"
// loads and the multiply-adds take the value as a scalar operand - no LDS, no workgroup barrier.
// Wt holds 16-bit integers here (k_transpose_centered_q16): half the bytes per gather, twice the
// columns per L2; the value of a nonzero is multiplied by its column's step once, and a gathered
// entry costs one conversion before its multiply-add.  The quantisation moves the dot product of
// a row by at most 0.51 sum_nz |v_c| step_c; that sum falls out of the products the lanes hold
// anyway and is stored per instance (row_q) for the margin of k_certify.
// Output per pair: the two best nodes and the smallest score dropped, in the candidate arrays of
// the dense path ([slice][instance][kCand]); k_certify merges the eight slices.  In collect mode
// the wavefront appends every node under the instance's threshold to its list instead.
__device__ __forceinline__ void wave_argmin(float &v, int &i) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(v, o, 64);
    const int oi = __shfl_xor(i, o, 64);
    const bool take = ov < v || (ov == v && (unsigned)oi < (unsigned)i);
    v = take ? ov : v;
    i = take ? oi : i;
  }
}

template <int ACC, bool kCollect>
__global__ __launch_bounds__(256) void k_bmu_csr_sliced(const int64_t *__restrict__ indptr,
                                                        const int32_t *__restrict__ indices,
                                                        const float *__restrict__ values,
                                                        const int16_t *__restrict__ Wt, int kpad,
                                                        const float *__restrict__ qstep,
                                                        const float *__restrict__ cn32, int64_t n, int k, int dim,
                                                        CandView out, float *__restrict__ row_q,
                                                        const int32_t *__restrict__ rows,
                                                        const int32_t *__restrict__ n_slots,
                                                        const float *__restrict__ thr, int32_t *__restrict__ cnt,
                                                        int32_t *__restrict__ list) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int slice = blockIdx.x & 7;
  const int slice0 = slice * (kpad >> 3);               // kpad is a multiple of 512: ACC * 64 nodes per slice
  const int64_t pairs = kCollect ? (int64_t)*n_slots : n;
  const int64_t stride = (int64_t)(gridDim.x >> 3) * 4;
  float cnode[ACC];
#pragma unroll
  for (int a = 0; a < ACC; ++a) {
    const int node = slice0 + lane + 64 * a;
    cnode[a] = node < k ? cn32[node] : INFINITY;
  }
  for (int64_t p = (int64_t)(blockIdx.x >> 3) * 4 + wave; p < pairs; p += stride) {
    const int64_t j = kCollect ? (int64_t)rows[p] : p;
    const int64_t rs = indptr[j];
    const int len = (int)(indptr[j + 1] - rs);
    float acc[ACC];
#pragma unroll
    for (int a = 0; a < ACC; ++a) acc[a] = 0.f;
    float vq_abs = 0.f;                                  // this lane's share of sum |v_c| step_c
    for (int p0 = 0; p0 < len; p0 += 64) {
      int c = 0;
      float v = 0.f;
      if (p0 + lane < len) {
        c = indices[rs + p0 + lane];
        c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
        v = values[rs + p0 + lane] * qstep[c];
        vq_abs += fabsf(v);
      }
      const int m = min(64, len - p0);
      int q = 0;
      // four nonzeros per step: all their gathers are issued before the first use
      for (; q + kCsrUnroll <= m; q += kCsrUnroll) {
        int w[kCsrUnroll][ACC];
        float vs[kCsrUnroll];
#pragma unroll
        for (int u = 0; u < kCsrUnroll; ++u) {
          const int cs = __builtin_amdgcn_readlane(c, q + u);
          vs[u] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), q + u));
          const int16_t *wrow = Wt + (int64_t)cs * kpad + slice0 + lane;
#pragma unroll
          for (int a = 0; a < ACC; ++a) w[u][a] = wrow[64 * a];
        }
#pragma unroll
        for (int u = 0; u < kCsrUnroll; ++u)
#pragma unroll
          for (int a = 0; a < ACC; ++a) acc[a] = fmaf(vs[u], (float)w[u][a], acc[a]);
      }
      for (; q < m; ++q) {
        const int cs = __builtin_amdgcn_readlane(c, q);
        const float vq = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), q));
        const int16_t *wrow = Wt + (int64_t)cs * kpad + slice0 + lane;
#pragma unroll
        for (int a = 0; a < ACC; ++a) acc[a] = fmaf(vq, (float)wrow[64 * a], acc[a]);
      }
    }
    float sc[ACC];
#pragma unroll
    for (int a = 0; a < ACC; ++a) sc[a] = fmaf(-2.f, acc[a], cnode[a]);      // +inf for nodes past k

    if (kCollect) {
      const float lim = thr[p];
#pragma unroll
      for (int a = 0; a < ACC; ++a) {
        const int node = slice0 + lane + 64 * a;
        if (sc[a] <= lim && node < k) {
          const int pos = atomicAdd(&cnt[p], 1);
          if (pos < kListCap) list[p * kListCap + pos] = node;
        }
      }
    } else {
      // two best nodes of the slice and the smallest score after them
      float best[3];
      int arg[2];
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        float v = INFINITY;
        int i = 0x7fffffff;
#pragma unroll
        for (int a = 0; a < ACC; ++a) {
          const int node = slice0 + lane + 64 * a;
          const bool take = sc[a] < v;                   // nodes ascend with a: strict keeps the lower index
          v = take ? sc[a] : v;
          i = take ? node : i;
        }
        wave_argmin(v, i);
        best[t] = v;
        if (t < 2) {
          arg[t] = i;
#pragma unroll
          for (int a = 0; a < ACC; ++a)
            if (slice0 + lane + 64 * a == i) sc[a] = INFINITY;
        }
      }
      if (slice == 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) vq_abs += __shfl_xor(vq_abs, o, 64);
        if (lane == 0) row_q[j] = vq_abs;
      }
      if (lane == 0) {
        const int64_t o = (int64_t)slice * n + j;
        out.val[o * kCand + 0] = best[0];
        out.idx[o * kCand + 0] = best[0] < INFINITY ? arg[0] : -1;
        out.val[o * kCand + 1] = best[1];
        out.idx[o * kCand + 1] = best[1] < INFINITY ? arg[1] : -1;
#pragma unroll
        for (int t = 2; t < kCand; ++t) { out.val[o * kCand + t] = INFINITY; out.idx[o * kCand + t] = -1; }
        out.over[o] = best[2];
      }
    }
  }
}

constexpr int kCsrSlices = 8;
constexpr int kCsrSlicedMaxAcc = 16;       // the sliced kernel keeps kpad / 8 / 64 scores per lane

bool bmu_csr_sliced_ok(const som_ctx *c) { return c->kpad / (kCsrSlices * 64) <= kCsrSlicedMaxAcc; }

template <bool kCollect>
static void launch_sliced(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n) {
  const int acc = c->kpad / (kCsrSlices * 64);
  int64_t groups = (n + 3) / 4;                                   // workgroups per slice
  const int64_t cap = (int64_t)c->n_cu;                           // 8 slices x n_cu = 8 workgroups per CU
  if (groups > cap) groups = cap;
  const dim3 grid((unsigned)(groups * kCsrSlices));
  CandView out{c->cand_val, c->cand_idx, c->cand_over};
#define SOM_SLICED(A)                                                                                              \
  hipLaunchKernelGGL((k_bmu_csr_sliced<A, kCollect>), grid, dim3(256), 0, c->stream, indptr, indices, values,        \
                     reinterpret_cast<const int16_t *>(c->Wt), c->kpad, c->qstep, c->wn32, n, c->k, c->dim, out,    \
                     c->row_q, c->collect_rows, c->list_counts + 1, c->collect_thr, c->collect_cnt, c->collect_list)
  switch (acc) {
    case 1: SOM_SLICED(1); break;
    case 2: SOM_SLICED(2); break;
    case 3: SOM_SLICED(3); break;
    case 4: SOM_SLICED(4); break;
    case 5: SOM_SLICED(5); break;
    case 6: SOM_SLICED(6); break;
    case 7: SOM_SLICED(7); break;
    case 8: SOM_SLICED(8); break;
    case 9: SOM_SLICED(9); break;
    case 10: SOM_SLICED(10); break;
    case 11: SOM_SLICED(11); break;
    case 12: SOM_SLICED(12); break;
    case 13: SOM_SLICED(13); break;
    case 14: SOM_SLICED(14); break;
    case 15: SOM_SLICED(15); break;
    default: SOM_SLICED(16); break;
  }
#undef SOM_SLICED
}

hipError_t launch_bmu_csr_sliced(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                                 int64_t n, bool collect) {
  if (collect) launch_sliced<true>(c, indptr, indices, values, n);
  else launch_sliced<false>(c, indptr, indices, values, n);
  return hipGetLastError();
}

hipError_t launch_transpose_codebook(som_ctx *c, const float *W) {
  dim3 grid((c->dim + 31) / 32, (c->kpad + 31) / 32);
  if (bmu_csr_sliced_ok(c))
    hipLaunchKernelGGL(k_transpose_centered_q16, grid, dim3(256), 0, c->stream, W, c->mu, c->qstep, c->k, c->dim,
                       c->kpad, reinterpret_cast<int16_t *>(c->Wt));
  else
    hipLaunchKernelGGL(k_transpose_centered, grid, dim3(256), 0, c->stream, W, c->mu, c->k, c->dim, c->kpad, c->Wt);
  return hipGetLastError();
}

template <int ACC>
static void launch_bmu_csr_acc(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                               int64_t n, int32_t *bmus) {
  int64_t blocks = (int64_t)c->n_cu * 8;
  if (blocks > n) blocks = n;
  CsrBmuOut out{bmus, c->cand_idx, c->cand_n, c->refine_list, c->collect_rows, c->collect_cnt, c->collect_list,
                c->rescan_list, c->list_counts};
  hipLaunchKernelGGL(k_bmu_csr<ACC>, dim3((unsigned)blocks), dim3(256), 0, c->stream, indptr, indices, values,
                     c->Wt, c->kpad, c->wn32, c->xn32, c->wmax_bits, c->mu_norm2, n, c->k, c->dim, out);
}

hipError_t launch_bmu_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                          int64_t n, int32_t *bmus) {
  const int need = (c->k + 255) / 256;
  if (need <= 1) launch_bmu_csr_acc<1>(c, indptr, indices, values, n, bmus);
  else if (need <= 2) launch_bmu_csr_acc<2>(c, indptr, indices, values, n, bmus);
  else if (need <= 4) launch_bmu_csr_acc<4>(c, indptr, indices, values, n, bmus);
  else if (need <= 6) launch_bmu_csr_acc<6>(c, indptr, indices, values, n, bmus);
  else if (need <= 8) launch_bmu_csr_acc<8>(c, indptr, indices, values, n, bmus);
  else if (need <= 10) launch_bmu_csr_acc<10>(c, indptr, indices, values, n, bmus);
  else if (need <= 12) launch_bmu_csr_acc<12>(c, indptr, indices, values, n, bmus);
  else launch_bmu_csr_acc<16>(c, indptr, indices, values, n, bmus);
  return hipGetLastError();
}

}  // namespace som
