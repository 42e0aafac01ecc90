// Sparse best-matching-unit search, filter pass (paper: sparse kernel - the code book stays
// dense while the data are index:value lists; BMU equation).
//
// As in the dense path the nodes are ranked by s_i = c_i - 2 x.w'_i with w' = w - mu and
// c_i = |w'_i|^2 + 2 mu.w'_i (identical ranking to |x - w_i|^2, smaller rounding error); x stays
// sparse, so x.w'_i = sum_nz v * w'_i[c].  mu is the mean of the code-book rows here.  The
// centred code book is written transposed, Wt[dim][kpad], so that one nonzero (c, v) touches one
// contiguous row of Wt.
//
// What bounds this kernel is the traffic its gathers send past L2: a nonzero touches a whole row
// of Wt, the popular columns of a Zipf-distributed vocabulary are few, and a 4 MB L2 holds only
// some hundred fp32 rows of a 50 x 50 map.  Two things make the caches hold more columns:
//
//   One node slice per XCD.  MI355X has eight L2s, one per XCD, and hands workgroup b to XCD
//   b mod 8.  The nodes are cut into eight slices and workgroup b only ever scores slice b mod 8:
//   an XCD then touches an eighth of every row of Wt, and the instances are walked once per slice
//   (their 8 bytes per nonzero are small change next to the gather).
//
//   16-bit entries.  Wt holds int16 multiples of a per-column step (k_finish_col_means); the value
//   of a nonzero is multiplied by its column's step once, and a gathered entry costs one conversion
//   before its multiply-add.  The quantisation moves the dot product of a row by at most
//   0.51 sum_nz |v_c| step_c; that sum falls out of the products the lanes hold anyway and is stored
//   per instance (row_q) for the margin of k_certify.
//
// A slice is cut into `sweeps` ranges of 64 ACC nodes (kpad = 512 ACC sweeps, so every range is
// full), and a wavefront owns one (instance, slice, range) unit: lane l owns nodes
// slice0 + 64 ACC s + l + 64 a, a < ACC.  The
// nonzeros of the row are read 64 at a time, one per lane, and handed round with v_readlane: column
// and value of the current nonzero live in scalar registers, so the gathers are "scalar base + lane
// offset" loads and the multiply-adds take the value as a scalar operand - no LDS, no workgroup
// barrier.  Output per unit: the two best nodes and the smallest score after them, in the candidate
// arrays of the dense path ([slice * sweeps + range][instance][kCand]); k_certify merges the 8 sweeps
// groups.  In collect mode the wavefront appends every node under the instance's threshold to its
// list instead.
#include "som_internal.hpp"

#include <math.h>

namespace som {

constexpr int kCsrUnroll = 4;      // nonzeros whose gathers are in flight together
constexpr int kCsrSlices = 8;      // one per XCD
constexpr int kCsrMaxAcc = 16;     // scores a lane holds per sweep

// Slice geometry for k nodes: sweeps per slice, scores per lane and sweep, padded node count.
void csr_slice_geometry(int k, int *acc, int *sweeps, int *kpad) {
  const int s64 = (k + 64 * kCsrSlices - 1) / (64 * kCsrSlices);      // 64-node groups per slice
  const int ns = (s64 + kCsrMaxAcc - 1) / kCsrMaxAcc;
  const int a = (s64 + ns - 1) / ns;
  *acc = a;
  *sweeps = ns;
  *kpad = 64 * kCsrSlices * a * ns;
}

// ---------------------------------------------------------------- centring, node constants and transpose in one pass
// One pass over the code book does what the sparse search needs of it every epoch: w' = fl(w - mu), the
// node constants c_i = |w'_i|^2 + 2 mu.w'_i and |w_i|^2 (fp64 sums in a fixed order: the exact stage
// relies on bit-identical rows having bit-identical norms), the largest |w'_i|^2, and the transposed
// 16-bit code book: entries q = round(w' / step_c) as int16, |q| <= 32767 by the choice of the step; nodes
// past k are zeros.  A workgroup owns 64 nodes and a slab of the columns, which it walks in tiles of 64:
// a thread reads four nodes (two pairs of neighbours) x four columns per tile (16-byte loads along the
// rows), the quantised tile turns in LDS, and every column leaves as 128 contiguous bytes.  The row sums of a slab go to
// `partial` [slab][node][3]; k_finish_node_constants adds the slabs in order.
constexpr int kCtNodes = 64;
constexpr int kCtCols = 64;

__global__ __launch_bounds__(256) void k_center_transpose_q16(const float *__restrict__ W, const float *__restrict__ mu,
                                                              const float *__restrict__ qstep, int k, int dim,
                                                              int kpad, int cols_per_slab, int16_t *__restrict__ Wt,
                                                              double *__restrict__ partial) {
  // the tile turned: [column][pair of neighbouring nodes] as 32-bit words (two int16), so that a thread
  // writes one word per two entries and the columns leave through 16-byte reads; 33 words per row keep
  // the column-wise writes of a wavefront on different banks
  __shared__ uint32_t tile[kCtCols][kCtNodes / 2 + 1];
  const int tid = threadIdx.x;
  const int q4 = tid & 15;                      // column quad within the tile
  const int p0 = tid >> 4;                      // first of this thread's two node pairs (p0 + 16 j): rows 2 p, 2 p + 1
  const int i0 = blockIdx.x * kCtNodes;
  const int slab = blockIdx.y;
  const int c_begin = slab * cols_per_slab;
  const int c_end = min(dim, c_begin + cols_per_slab);
  const bool vec = (dim & 3) == 0 && (reinterpret_cast<uintptr_t>(W) & 15) == 0;
  double s2[4] = {0, 0, 0, 0}, sm[4] = {0, 0, 0, 0}, sw[4] = {0, 0, 0, 0};      // rows 2 (p0 + 16 j) + h at [2 j + h]
  // this thread's four rows x four columns of a tile; entries past the slab or the map come out as mu (w' = 0).
  // The next tile is loaded while the current one goes through LDS.
  auto load_tile = [&](int c0, float (&x)[4][4]) {
    const int c = c0 + 4 * q4;
#pragma unroll
    for (int jh = 0; jh < 4; ++jh) {
      const int i = i0 + 2 * (p0 + 16 * (jh >> 1)) + (jh & 1);
      if (i < k && vec && c + 3 < c_end) {
        const float4 v = *reinterpret_cast<const float4 *>(W + (int64_t)i * dim + c);
        x[jh][0] = v.x; x[jh][1] = v.y; x[jh][2] = v.z; x[jh][3] = v.w;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool on = i < k && c + e < c_end;
          x[jh][e] = on ? W[(int64_t)i * dim + c + e] : (c + e < c_end ? mu[c + e] : 0.f);
        }
      }
    }
  };
  float xn[4][4];
  load_tile(c_begin, xn);
  for (int c0 = c_begin; c0 < c_end; c0 += kCtCols) {
    const int c = c0 + 4 * q4;
    float xc[4][4];
#pragma unroll
    for (int jh = 0; jh < 4; ++jh)
#pragma unroll
      for (int e = 0; e < 4; ++e) xc[jh][e] = xn[jh][e];
    if (c0 + kCtCols < c_end) load_tile(c0 + kCtCols, xn);
    float m[4], inv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool on = c + e < c_end;
      m[e] = on ? mu[c + e] : 0.f;
      inv[e] = on ? qstep[c + e] : 1.f;
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int pr = p0 + 16 * j;
      uint32_t word[4] = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int i = i0 + 2 * pr + h;
        const float (&x)[4] = xc[2 * j + h];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float t = x[e] - m[e];
          if (i < k && c + e < c_end) {
            s2[2 * j + h] += (double)t * (double)t;
            sm[2 * j + h] += (double)m[e] * (double)t;
            sw[2 * j + h] += (double)x[e] * (double)x[e];
          }
          float q = rintf(t / inv[e]);
          q = fminf(fmaxf(q, -32767.f), 32767.f);
          word[e] |= ((uint32_t)(uint16_t)(int16_t)q) << (16 * h);
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) tile[4 * q4 + e][pr] = word[e];
    }
    __syncthreads();
    {   // column tid / 4 of the tile, nodes 16 (tid % 4) .. + 15: 32 contiguous bytes of one row of Wt
      const int col = tid >> 2, g = tid & 3;
      if (c0 + col < c_end && i0 + 16 * g < kpad) {
        uint32_t out[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e] = tile[col][8 * g + e];
        uint4 *dst = reinterpret_cast<uint4 *>(Wt + (int64_t)(c0 + col) * kpad + i0 + 16 * g);
        dst[0] = make_uint4(out[0], out[1], out[2], out[3]);
        dst[1] = make_uint4(out[4], out[5], out[6], out[7]);
      }
    }
    __syncthreads();
  }
  // the four rows' sums over this slab: the 16 threads of a row pair sit in consecutive lanes
#pragma unroll
  for (int jh = 0; jh < 4; ++jh) {
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {
      s2[jh] += __shfl_xor(s2[jh], o, 64);
      sm[jh] += __shfl_xor(sm[jh], o, 64);
      sw[jh] += __shfl_xor(sw[jh], o, 64);
    }
    const int i = i0 + 2 * (p0 + 16 * (jh >> 1)) + (jh & 1);
    if (q4 == 0 && i < k) {
      double *dst = partial + ((int64_t)slab * k + i) * 3;
      dst[0] = s2[jh]; dst[1] = sm[jh]; dst[2] = sw[jh];
    }
  }
}

__global__ __launch_bounds__(256) void k_finish_node_constants(const double *__restrict__ partial, int slabs, int k,
                                                               float *__restrict__ cn, double *__restrict__ wn64,
                                                               unsigned *__restrict__ max_bits) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  float vmax = 0.f;
  if (i < k) {
    double s2 = 0.0, sm = 0.0, sw = 0.0;
    for (int s = 0; s < slabs; ++s) {
      const double *p = partial + ((int64_t)s * k + i) * 3;
      s2 += p[0]; sm += p[1]; sw += p[2];
    }
    cn[i] = (float)(s2 + 2.0 * sm);
    wn64[i] = sw;
    vmax = (float)s2;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, o, 64));
  if ((threadIdx.x & 63) == 0 && vmax > 0.f) atomicMax(max_bits, __float_as_uint(vmax));
}

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
                                                        const int16_t *__restrict__ Wt, int kpad, int sweeps,
                                                        const float *__restrict__ qstep,
                                                        const float *__restrict__ cn32, int64_t n, int k, int dim,
                                                        CandView out, float *__restrict__ row_q,
                                                        const int32_t *__restrict__ rows,
                                                        UnitWork work,
                                                        const float *__restrict__ thr, int32_t *__restrict__ cnt,
                                                        int32_t *__restrict__ list, float *__restrict__ dump,
                                                        const float *__restrict__ phot,
                                                        const float *__restrict__ hot_xscale) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int slice = blockIdx.x & 7;
  const int slice0 = slice * (kpad >> 3);
  // the range is the slow index: the wavefronts an XCD runs together gather from the same 64 ACC
  // columns of Wt, a working set its L2 and the memory-side cache can hold for the frequent features
  // Second sweep: the units come from this slice's work list instead.
  const int64_t units = kCollect ? (int64_t)work.counts[slice] : n * sweeps;
  const int64_t stride = (int64_t)(gridDim.x >> 3) * 4;
  for (int64_t unit = (int64_t)(blockIdx.x >> 3) * 4 + wave; unit < units; unit += stride) {
    int sw;
    int64_t p;
    if (kCollect) {
      const int64_t e = work.units[(int64_t)slice * work.cap + unit];
      p = e / sweeps;
      sw = (int)(e - p * sweeps);
    } else {
      sw = (int)(unit / n);
      p = unit - (int64_t)sw * n;
    }
    const int64_t j = kCollect ? (int64_t)rows[p] : p;
    const int64_t rs = indptr[j];
    const int len = (int)(indptr[j + 1] - rs);
    const int base = slice0 + sw * (64 * ACC) + lane;    // this lane's first node
    float vq_abs = 0.f;                                  // this lane's share of sum |v_c| step_c
    float acc[ACC];
    if (phot) {
      // the rows are the tail of a registered set: the dot products of its frequent columns come from the
      // matrix-core pass (csr_hot.hip), 64 consecutive nodes = 256 contiguous bytes per load
      // (the table is [block of 128 nodes][instance][128]: a lane set of 64 nodes never straddles a block)
      const float xs = hot_xscale[j];
#pragma unroll
      for (int a = 0; a < ACC; ++a) {
        const int node = base + 64 * a;
        acc[a] = node < k ? xs * phot[((int64_t)(node >> 7) * n + j) * 128 + (node & 127)] : 0.f;
      }
    } else {
#pragma unroll
      for (int a = 0; a < ACC; ++a) acc[a] = 0.f;
    }
    for (int p0 = 0; p0 < len; p0 += 64) {
      int c = 0;
      float v = 0.f;
      if (p0 + lane < len) {
        c = indices[rs + p0 + lane];
        c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
        v = qstep ? values[rs + p0 + lane] * qstep[c] : values[rs + p0 + lane];
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
          const int16_t *wrow = Wt + (int64_t)cs * kpad + base;
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
        const int16_t *wrow = Wt + (int64_t)cs * kpad + base;
#pragma unroll
        for (int a = 0; a < ACC; ++a) acc[a] = fmaf(vq, (float)wrow[64 * a], acc[a]);
      }
    }
    float sc[ACC];
#pragma unroll
    for (int a = 0; a < ACC; ++a) {
      const int node = base + 64 * a;
      sc[a] = node < k ? fmaf(-2.f, acc[a], cn32[node]) : INFINITY;
    }

    if (kCollect) {
      const float lim = thr[p];
#pragma unroll
      for (int a = 0; a < ACC; ++a) {
        const int node = base + 64 * a;
        if (sc[a] <= lim && node < k) {
          const int pos = atomicAdd(&cnt[p], 1);
          if (pos < kListCap) list[p * kListCap + pos] = node;
        }
      }
    } else {
      if (dump) {                                        // test hook: every score of the unit
#pragma unroll
        for (int a = 0; a < ACC; ++a)
          if (base + 64 * a < k) dump[j * k + base + 64 * a] = sc[a];
      }
      // two best nodes of the range and the smallest score after them
      float best[3];
      int arg[2];
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        float v = INFINITY;
        int i = 0x7fffffff;
#pragma unroll
        for (int a = 0; a < ACC; ++a) {
          const bool take = sc[a] < v;                   // nodes ascend with a: strict keeps the lower index
          v = take ? sc[a] : v;
          i = take ? base + 64 * a : i;
        }
        wave_argmin(v, i);
        best[t] = v;
        if (t < 2) {
          arg[t] = i;
#pragma unroll
          for (int a = 0; a < ACC; ++a)
            if (base + 64 * a == i) sc[a] = INFINITY;
        }
      }
      if (slice == 0 && sw == 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) vq_abs += __shfl_xor(vq_abs, o, 64);
        if (lane == 0) row_q[j] = vq_abs;
      }
      if (lane == 0) {
        const int64_t o = (int64_t)(slice * sweeps + sw) * n + j;
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

template <bool kCollect>
static void launch_sliced(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values, int64_t n,
                          float *dump, bool hot) {
  const float *phot = hot ? c->hot_P : nullptr;
  int64_t groups = (n * c->csr_sweeps + 3) / 4;                   // workgroups per slice
  const int64_t cap = (int64_t)c->n_cu;                           // 8 slices x n_cu = 8 workgroups per CU
  if (groups > cap) groups = cap;
  const dim3 grid((unsigned)(groups * kCsrSlices));
  CandView out{c->cand_val, c->cand_idx, c->cand_over};
  const UnitWork work{c->csr_sweeps, c->unit_cap, c->unit_work, c->list_counts + kUnitCounts, c->collect_list};
#define SOM_SLICED(A)                                                                                              \
  hipLaunchKernelGGL((k_bmu_csr_sliced<A, kCollect>), grid, dim3(256), 0, c->stream, indptr, indices, values,        \
                     reinterpret_cast<const int16_t *>(c->Wt), c->kpad, c->csr_sweeps, nullptr, c->wn32, n, c->k,   \
                     c->dim, out, c->row_q, c->collect_rows, work, c->collect_thr, c->collect_cnt,    \
                     c->collect_list, dump, phot, c->hot_xscale)
  switch (c->csr_acc) {
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

// Values of the nonzeros times the quantisation step of their column: once per search instead of once
// per node range and slice.
__global__ __launch_bounds__(256) void k_scale_values(const int32_t *__restrict__ indices,
                                                      const float *__restrict__ values, int64_t nnz, int dim,
                                                      const float *__restrict__ qstep, float *__restrict__ out) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < nnz; p += stride) {
    int c = indices[p];
    c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
    out[p] = values[p] * qstep[c];
  }
}

hipError_t launch_scale_values(som_ctx *c, const int32_t *indices, const float *values, int64_t nnz) {
  if (nnz < 1) return hipSuccess;                       // every row empty: nothing to scale (and no buffer yet)
  if (!c->vq || c->vq_cap < nnz) return hipErrorInvalidValue;
  int64_t cb = (nnz + 255) / 256;
  if (cb > (int64_t)c->n_cu * 16) cb = (int64_t)c->n_cu * 16;
  hipLaunchKernelGGL(k_scale_values, dim3((unsigned)cb), dim3(256), 0, c->stream, indices, values, nnz, c->dim,
                     c->qstep, c->vq);
  return hipGetLastError();
}

// ---------------------------------------------------------------- structure check (debug pass)
// The sparse format of the paper's command line: per row, zero-based index:value pairs.  The searches
// assume indptr[0] = 0, indptr non-decreasing up to indptr[n] = nnz, and within a row strictly
// increasing column indices in [0, dim).  One wavefront per row; the largest violation code found is
// left in *flag (0 = none).  A row whose bounds are not inside [0, nnz] is reported and not read.
__global__ __launch_bounds__(256) void k_validate_csr(const int64_t *__restrict__ indptr,
                                                      const int32_t *__restrict__ indices, int64_t n, int64_t nnz,
                                                      int dim, int32_t *__restrict__ flag) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  int bad = 0;
  if (wave == 0 && lane == 0) {
    if (indptr[n] != nnz) bad = kCsrBadLast;
    if (indptr[0] != 0) bad = kCsrBadFirst;
  }
  for (int64_t j = wave; j < n; j += nwaves) {
    const int64_t s = indptr[j], e = indptr[j + 1];
    if (s > e || s < 0 || e > nnz) {
      bad = max(bad, (int)kCsrBadOrder);
      continue;
    }
    for (int64_t p = s + lane; p < e; p += 64) {
      const int c = indices[p];
      if (c < 0 || c >= dim) bad = max(bad, (int)kCsrBadIndex);
      else if (p > s && indices[p - 1] >= c) bad = max(bad, (int)kCsrBadSorted);
    }
  }
  if (bad) atomicMax(flag, bad);
}

hipError_t launch_validate_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, int64_t n, int64_t nnz,
                               int32_t *flag) {
  int64_t blocks = (n + 3) / 4;
  if (blocks > (int64_t)c->n_cu * 16) blocks = (int64_t)c->n_cu * 16;
  hipLaunchKernelGGL(k_validate_csr, dim3((unsigned)blocks), dim3(256), 0, c->stream, indptr, indices, n, nnz, c->dim,
                     flag);
  return hipGetLastError();
}

hipError_t launch_bmu_csr_sliced(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                                 int64_t n, bool collect, float *dump, bool hot) {
  if (collect) launch_sliced<true>(c, indptr, indices, values, n, nullptr, hot);
  else launch_sliced<false>(c, indptr, indices, values, n, dump, hot);
  return hipGetLastError();
}

// Centred transposed 16-bit code book, node constants (wn32 = c_i), |w_i|^2 (wn64) and the largest |w'_i|^2
// (wmax_bits), from mu and qstep: one pass over W.
hipError_t launch_center_transpose_codebook(som_ctx *c, const float *W) {
  hipError_t e = launch_fill_zero_u32(c->stream, c->wmax_bits, 2);
  if (e != hipSuccess) return e;
  const int tiles = c->kpad / kCtNodes;                       // kpad is a multiple of 512
  // enough workgroups for twelve per CU: a workgroup walks its slab one tile after the other and waits for
  // every tile's loads, so the memory system is kept busy by their number (two per CU: 2.3 TB/s)
  int slabs = (12 * c->n_cu + tiles - 1) / tiles;
  const int max_slabs = (c->dim + kCtCols - 1) / kCtCols;
  if (slabs > max_slabs) slabs = max_slabs;
  if (slabs > kCtMaxSlabs) slabs = kCtMaxSlabs;
  if (slabs < 1) slabs = 1;
  int cols_per_slab = (c->dim + slabs - 1) / slabs;
  cols_per_slab = (cols_per_slab + kCtCols - 1) / kCtCols * kCtCols;
  slabs = (c->dim + cols_per_slab - 1) / cols_per_slab;
  hipLaunchKernelGGL(k_center_transpose_q16, dim3((unsigned)tiles, (unsigned)slabs), dim3(256), 0, c->stream, W, c->mu,
                     c->qstep, c->k, c->dim, c->kpad, cols_per_slab, reinterpret_cast<int16_t *>(c->Wt), c->ct_partial);
  hipLaunchKernelGGL(k_finish_node_constants, dim3((c->k + 255) / 256), dim3(256), 0, c->stream, c->ct_partial, slabs,
                     c->k, c->wn32, c->wn64, c->wmax_bits);
  return hipGetLastError();
}

}  // namespace som
