// Exact stage of the best-matching-unit search (paper: BMU equation, d = Euclidean distance).
//
// The fp32 pass leaves, per instance, a few candidate nodes with their scores
// s = |w'|^2 - 2 x'.w' (x' = x - mu, w' = w - mu) and the smallest score it dropped.  Here:
//   certify  - bounds the rounding error of those scores; an instance whose best score beats
//              everything else by more than twice the bound is decided on the spot;
//   refine   - otherwise the candidates inside the bound are compared by their squared
//              distances sum_c (x_c - w_c)^2 evaluated in fp64 on the original (uncentred)
//              vectors, lowest node index on exact ties (sparse rows: a regrouped sum over the
//              nonzeros, and the plain sum over all coordinates where that one would cancel);
//   collect  - if a dropped score lies inside the bound too, the fp32 sweep is repeated for
//              that instance and every node under the threshold is listed (bmu_dense.hip),
//              then the list is compared exactly;
//   rescan   - if even that list overflows, all nodes are compared exactly.
// The instance lists are built with atomic counters, so their order varies between runs;
// every instance is decided independently, so the BMUs do not.
//
// (The split-fp16 pass multiplies centred instances x' = fl(x - mu): there X = |x'| and the terms in M
// fall away.)
// Error bound of one dense fp32 score s = c_i - 2 x.w'_i (u = 2^-24, g = roundings a product term
// can suffer, X = |x|, M = |mu|, Wm = max |w'| over the nodes, w' = fl(w - mu)):
//   |s_fp32 - s_exact| <= u [ (2 g + 4) X Wm + 4 Wm^2 + 6 M Wm ]
// made of: the dot product, g u sum|x_c w'_c| <= g u X Wm, doubled by the factor -2; the rounding
// of the stored c_i, u (Wm^2 + 2 M Wm); the final multiply-add, u (Wm^2 + 2 M Wm + 2 X Wm); and the
// rounding of w - mu itself, which moves a squared distance by at most 2 u (X + M + Wm) Wm.
// MFMA pass with two-level accumulation: g = block + ceil(dim / block) + 2.
// Sparse scores |w|^2 - 2 x.w from an FMA chain of len terms, no centring: g = len,
//   |s_fp32 - s_exact| <= u [ (2 g + 2) X Wm + 2 Wm^2 ].
#include "margin.hpp"

namespace som {

// `groups` candidate lists per instance (one per node group of the fp32 pass), stored
// [group][instance][kCand]; the kept candidates are written back into group 0's slots.
__global__ __launch_bounds__(256) void k_certify(CandView cand, int groups, const float *__restrict__ xn32,
                                                 const unsigned *__restrict__ wmax_bits,
                                                 const float *__restrict__ mu_norm2, MarginModel mm, int64_t n, int k,
                                                 int32_t *__restrict__ bmus, int32_t *__restrict__ cand_n,
                                                 int32_t *__restrict__ refine_list,
                                                 int32_t *__restrict__ collect_rows,
                                                 float *__restrict__ collect_thr,
                                                 int32_t *__restrict__ collect_cnt,
                                                 int32_t *__restrict__ list_counts, UnitWork work,
                                                 const int32_t *__restrict__ order) {
  // with `order` the instances are visited in that order, so that neighbours in it are appended to the
  // lists together: the second sweep's tiles then hold instances with similar block sets (two-level
  // search).  List slots are reserved per workgroup - one atomic per list and workgroup, the positions
  // inside from ballots - because a million instances' worth of wavefront-wide atomics on one counter
  // (16,000 of them) were what this kernel spent its time on.
  __shared__ int s_wave_cnt[2][4], s_base[2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool live = p < n;
  const int64_t j = live ? (order ? (int64_t)order[p] : p) : 0;
  static_assert(kCand == 4, "the candidate lists are read as 16-byte vectors");
  const float4 *val4 = reinterpret_cast<const float4 *>(cand.val);
  const int4 *idx4 = reinterpret_cast<const int4 *>(cand.idx);
  float smin = INFINITY, omin = INFINITY;
  double thr = 0.0;
  int keep[kCand] = {0, 0, 0, 0};
  int cnt = 0;
  if (live) {
    for (int q = 0; q < groups; ++q) {
      const float4 v = val4[(int64_t)q * n + j];
      const int4 id = idx4[(int64_t)q * n + j];
      if ((unsigned)id.x < (unsigned)k) smin = fminf(smin, v.x);
      if ((unsigned)id.y < (unsigned)k) smin = fminf(smin, v.y);
      if ((unsigned)id.z < (unsigned)k) smin = fminf(smin, v.z);
      if ((unsigned)id.w < (unsigned)k) smin = fminf(smin, v.w);
      omin = fminf(omin, cand.over[(int64_t)q * n + j]);
    }
    const double margin = score_margin(mm, j, (double)xn32[j], (double)__uint_as_float(*wmax_bits), (double)*mu_norm2);
    thr = (double)smin + margin;
    for (int q = 0; q < groups; ++q) {
      const float4 v4 = val4[(int64_t)q * n + j];
      const int4 id4 = idx4[(int64_t)q * n + j];
      const float v[kCand] = {v4.x, v4.y, v4.z, v4.w};
      const int id[kCand] = {id4.x, id4.y, id4.z, id4.w};
#pragma unroll
      for (int t = 0; t < kCand; ++t) {
        if ((unsigned)id[t] < (unsigned)k && (double)v[t] <= thr) {
          if (cnt < kCand) keep[cnt] = id[t];
          ++cnt;
        }
      }
    }
  }
  const bool overflow = (double)omin <= thr || cnt > kCand;
  const bool to_collect = live && (overflow || cnt == 0);
  const bool to_refine = live && !to_collect && cnt > 1;
  // slots: [0] refine list, [1] collect list
  const unsigned long long bal_r = __ballot(to_refine), bal_c = __ballot(to_collect);
  if (lane == 0) {
    s_wave_cnt[0][wave] = __popcll(bal_r);
    s_wave_cnt[1][wave] = __popcll(bal_c);
  }
  __syncthreads();
  if (threadIdx.x < 2) {
    const int total = s_wave_cnt[threadIdx.x][0] + s_wave_cnt[threadIdx.x][1] + s_wave_cnt[threadIdx.x][2] +
                      s_wave_cnt[threadIdx.x][3];
    s_base[threadIdx.x] = total ? atomicAdd(&list_counts[threadIdx.x], total) : 0;
  }
  __syncthreads();
  const unsigned long long below = (1ull << lane) - 1ull;
  int before_r = s_base[0], before_c = s_base[1];
  for (int w = 0; w < wave; ++w) {
    before_r += s_wave_cnt[0][w];
    before_c += s_wave_cnt[1][w];
  }
  if (to_collect) {
    const int slot = before_c + __popcll(bal_c & below);
    collect_rows[slot] = (int32_t)j;
    float t32 = (float)thr;                     // round the threshold up: no score inside the margin is lost
    if ((double)t32 < thr) t32 = nextafterf(t32, INFINITY);
    collect_thr[slot] = cnt == 0 ? INFINITY : t32;
    int filled = 0;
    if (work.sweeps > 0) {
      // sparse search: only the node ranges whose third-best score is inside the threshold have to be
      // swept again; the others are known completely through their two best nodes, listed here
      const double lim = cnt == 0 ? (double)INFINITY : thr;
      for (int q = 0; q < groups; ++q) {
        if ((double)cand.over[(int64_t)q * n + j] <= lim) {
          const int slice = q / work.sweeps;
          const int pos = atomicAdd(&work.counts[slice], 1);
          work.units[(int64_t)slice * work.cap + pos] = (int64_t)slot * work.sweeps + (q - slice * work.sweeps);
        } else {
          const int64_t base = ((int64_t)q * n + j) * kCand;
#pragma unroll
          for (int t = 0; t < kCand; ++t) {
            const int id = cand.idx[base + t];
            if ((unsigned)id < (unsigned)k && (double)cand.val[base + t] <= lim) {
              if (filled < kListCap) work.list[(int64_t)slot * kListCap + filled] = id;
              ++filled;
            }
          }
        }
      }
    }
    collect_cnt[slot] = filled;
  } else if (to_refine) {
    for (int t = 0; t < cnt; ++t) cand.idx[j * kCand + t] = keep[t];
    cand_n[j] = cnt;
    refine_list[before_r + __popcll(bal_r & below)] = (int32_t)j;
  } else if (live) {
    bmus[j] = keep[0];
  }
}

// sum_c (x_c - w_c)^2 in fp64, columns dealt to lanes round-robin, butterfly reduction: the
// same order for every node, so identical weight vectors give bit-identical results.
__device__ __forceinline__ double sqdist_dense_wave(const float *__restrict__ x, const float *__restrict__ w,
                                                    int dim, int lane) {
  double s = 0.0;
  for (int c = lane; c < dim; c += kWave) {
    const double d = (double)x[c] - (double)w[c];
    s += d * d;
  }
  return wave_sum(s);
}

// Four such distances at once, each with the summation order of sqdist_dense_wave (same bits).
__device__ __forceinline__ void sqdist_dense_wave4(const float *__restrict__ x, const float *__restrict__ W,
                                                   const int (&id)[4], int dim, int lane, double (&out)[4]) {
  const float *w0 = W + (int64_t)id[0] * dim, *w1 = W + (int64_t)id[1] * dim;
  const float *w2 = W + (int64_t)id[2] * dim, *w3 = W + (int64_t)id[3] * dim;
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  for (int c = lane; c < dim; c += kWave) {
    const double xv = (double)x[c];
    const double d0 = xv - (double)w0[c], d1 = xv - (double)w1[c];
    const double d2 = xv - (double)w2[c], d3 = xv - (double)w3[c];
    s0 += d0 * d0;
    s1 += d1 * d1;
    s2 += d2 * d2;
    s3 += d3 * d3;
  }
  out[0] = wave_sum(s0);
  out[1] = wave_sum(s1);
  out[2] = wave_sum(s2);
  out[3] = wave_sum(s3);
}

// The same distance for a sparse row with implicit zeros, regrouped so that only the nonzeros are
// visited: |w|^2 + sum_nz ((v - w_c)^2 - w_c^2).  Equal to the plain sum in exact arithmetic; in fp64
// its absolute error is about (dim + len) 2^-53 (|w|^2 + |x|^2), which is harmless unless the
// distance itself is that small (sqdist_csr_wave below).
__device__ __forceinline__ double sqdist_csr_regrouped_wave(const int32_t *__restrict__ idx,
                                                            const float *__restrict__ val, int len,
                                                            const float *__restrict__ w, double wn, int dim,
                                                            int lane) {
  double s = 0.0;
  for (int p = lane; p < len; p += kWave) {
    int c = idx[p];
    c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
    const double wc = (double)w[c];
    const double d = (double)val[p] - wc;
    s += d * d - wc * wc;
  }
  return wn + wave_sum(s);
}

// The BMU equation's sum as it is printed: every coordinate once, an unlisted one as zero, all
// terms non-negative, so nothing cancels and an instance that coincides with the weight vector
// is at distance exactly 0.  Lanes take the coordinates round-robin; each keeps a cursor into the
// row's (sorted) column list, which only ever moves forward.  dim loads: the rare path.
__device__ __forceinline__ double sqdist_csr_plain_wave(const int32_t *__restrict__ idx,
                                                        const float *__restrict__ val, int len,
                                                        const float *__restrict__ w, int dim, int lane) {
  double s = 0.0;
  int p = 0;
  for (int c = lane; c < dim; c += kWave) {
    while (p < len && idx[p] < c) ++p;
    const double x = (p < len && idx[p] == c) ? (double)val[p] : 0.0;
    const double d = x - (double)w[c];
    s += d * d;
  }
  return wave_sum(s);
}

// Squared norm of a sparse row in fp64 (every lane gets the sum).
__device__ __forceinline__ double csr_row_sqnorm_wave(const float *__restrict__ val, int len, int lane) {
  double s = 0.0;
  for (int p = lane; p < len; p += kWave) s += (double)val[p] * (double)val[p];
  return wave_sum(s);
}

// Exact distance of a sparse row: the regrouped sum wherever its rounding is at least 2^23 times
// smaller than the result (relative error below 1.2e-7, a hundredth of the tolerance band of the
// decision), the plain sum otherwise.  wn = |w|^2, xn = |x|^2.  Every lane holds the same bits of
// the regrouped value, so the branch is uniform over the wavefront; bit-identical weight vectors
// take the same branch and get the same bits.
__device__ __forceinline__ double sqdist_csr_wave(const int32_t *__restrict__ idx, const float *__restrict__ val,
                                                  int len, const float *__restrict__ w, double wn, double xn,
                                                  int dim, int lane) {
  const double d2 = sqdist_csr_regrouped_wave(idx, val, len, w, wn, dim, lane);
  const double noise = ((double)dim + (double)len + 2.0) * 1.862645149230957e-09 * (wn + xn);   // 2^-29 = 2^-52 * 2^23
  if (d2 < noise) return sqdist_csr_plain_wave(idx, val, len, w, dim, lane);
  return d2;
}

__global__ __launch_bounds__(256) void k_refine_dense(const float *__restrict__ X, const float *__restrict__ W,
                                                      int dim, const int32_t *__restrict__ cand_idx,
                                                      const int32_t *__restrict__ cand_n,
                                                      const int32_t *__restrict__ refine_list,
                                                      const int32_t *__restrict__ list_counts,
                                                      int32_t *__restrict__ bmus) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int nwaves = gridDim.x * (blockDim.x / kWave);
  const int count = list_counts[0];
  for (int e = wave; e < count; e += nwaves) {
    const int64_t j = refine_list[e];
    const int cn = cand_n[j];
    double best = INFINITY;
    int arg = 0x7fffffff;
    for (int t = 0; t < cn; ++t) {
      const int i = cand_idx[j * kCand + t];
      const double d2 = sqdist_dense_wave(X + j * dim, W + (int64_t)i * dim, dim, lane);
      if (d2 < best || (d2 == best && i < arg)) { best = d2; arg = i; }
    }
    if (lane == 0) bmus[j] = arg == 0x7fffffff ? 0 : arg;      // no finite distance (non-finite input): node 0, as a plain scan gives
  }
}

// Next entry of a work list for this wavefront.  The lists differ in length by two orders of magnitude (2 to
// 256 nodes), and a fixed assignment of entries to wavefronts left most of the chip idle behind the wavefronts
// that had drawn the long ones (5 resident wavefronts per CU on average, out of 32); so entries are handed out
// from counters that the search zeroes with the list lengths.  One counter serialises: an atomic on one address
// takes about 10 ns whoever issues it, more than the comparison of a list of 128-feature rows.  Hence eight
// counters in different memory channels: workgroup b draws from counter b mod 8, which hands out the entries
// e = b mod 8 (mod 8).
__device__ inline int next_entry(int32_t *list_counts, int lane) {
  const int slice = blockIdx.x & (kListTickets - 1);
  int t = 0;
  if (lane == 0) t = atomicAdd(list_counts + kListCounts + slice * kListTicketStride, 1);
  return __builtin_amdgcn_readfirstlane(t) * kListTickets + slice;
}

// Exact comparison of the collected lists: one wavefront per listed instance.  A list that
// overflowed its capacity sends the instance on to the full rescan.
__global__ __launch_bounds__(256) void k_refine_lists_dense(const float *__restrict__ X, const float *__restrict__ W,
                                                            int dim, int k, const int32_t *__restrict__ collect_rows,
                                                            const int32_t *__restrict__ collect_cnt,
                                                            const int32_t *__restrict__ collect_list,
                                                            int32_t *__restrict__ rescan_list,
                                                            int32_t *__restrict__ list_counts,
                                                            int32_t *__restrict__ bmus) {
  const int lane = threadIdx.x & (kWave - 1);
  const int count = list_counts[1];
  for (int e = next_entry(list_counts, lane); e < count; e = next_entry(list_counts, lane)) {
    const int64_t j = collect_rows[e];
    const int cn = collect_cnt[e];
    if (cn > kListCap || cn == 0) {
      if (lane == 0) rescan_list[atomicAdd(&list_counts[2], 1)] = (int32_t)j;
      continue;
    }
    const int32_t *lst = collect_list + (int64_t)e * kListCap;
    double best = INFINITY;
    int arg = 0x7fffffff;
    // four listed nodes at a time: their rows stream together and the instance is read once for the four
    // (a list can be long, and one distance at a time left the kernel waiting on its own loads); every
    // distance is still summed in the order of sqdist_dense_wave
    int t = 0;
    for (; t + 4 <= cn; t += 4) {
      int id[4];
      double d2[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) id[u] = min(max(lst[t + u], 0), k - 1);   // lists only ever hold valid nodes; never trust memory
      sqdist_dense_wave4(X + j * dim, W, id, dim, lane, d2);
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (d2[u] < best || (d2[u] == best && id[u] < arg)) { best = d2[u]; arg = id[u]; }
    }
    for (; t < cn; ++t) {
      const int i = min(max(lst[t], 0), k - 1);
      const double d2 = sqdist_dense_wave(X + j * dim, W + (int64_t)i * dim, dim, lane);
      if (d2 < best || (d2 == best && i < arg)) { best = d2; arg = i; }
    }
    if (lane == 0) bmus[j] = arg == 0x7fffffff ? 0 : arg;      // no finite distance (non-finite input): node 0, as a plain scan gives
  }
}

__global__ __launch_bounds__(256) void k_rescan_dense(const float *__restrict__ X, const float *__restrict__ W,
                                                      int dim, int k, const int32_t *__restrict__ rescan_list,
                                                      const int32_t *__restrict__ list_counts,
                                                      int32_t *__restrict__ bmus) {
  __shared__ double s_best[4];
  __shared__ int s_arg[4];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int count = list_counts[2];
  for (int e = blockIdx.x; e < count; e += gridDim.x) {
    const int64_t j = rescan_list[e];
    const float *x = X + j * dim;
    double best = INFINITY;
    int arg = 0x7fffffff;
    for (int i = wave; i < k; i += 4) {           // ascending within a wave: strict < keeps the lowest index
      const double d2 = sqdist_dense_wave(x, W + (int64_t)i * dim, dim, lane);
      if (d2 < best) { best = d2; arg = i; }
    }
    if (lane == 0) { s_best[wave] = best; s_arg[wave] = arg; }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = 1; w < 4; ++w)
        if (s_best[w] < best || (s_best[w] == best && s_arg[w] < arg)) { best = s_best[w]; arg = s_arg[w]; }
      bmus[j] = arg == 0x7fffffff ? 0 : arg;
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void k_refine_csr(const int64_t *__restrict__ indptr,
                                                    const int32_t *__restrict__ indices,
                                                    const float *__restrict__ values,
                                                    const float *__restrict__ W, const double *__restrict__ wn64,
                                                    int dim, const int32_t *__restrict__ cand_idx,
                                                    const int32_t *__restrict__ cand_n,
                                                    const int32_t *__restrict__ refine_list,
                                                    const int32_t *__restrict__ list_counts,
                                                    int32_t *__restrict__ bmus) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int nwaves = gridDim.x * (blockDim.x / kWave);
  const int count = list_counts[0];
  for (int e = wave; e < count; e += nwaves) {
    const int64_t j = refine_list[e];
    const int64_t s = indptr[j];
    const int len = (int)(indptr[j + 1] - s);
    const int cn = cand_n[j];
    const double xn = csr_row_sqnorm_wave(values + s, len, lane);
    double best = INFINITY;
    int arg = 0x7fffffff;
    for (int t = 0; t < cn; ++t) {
      const int i = cand_idx[j * kCand + t];
      const double d2 = sqdist_csr_wave(indices + s, values + s, len, W + (int64_t)i * dim, wn64[i], xn, dim, lane);
      if (d2 < best || (d2 == best && i < arg)) { best = d2; arg = i; }
    }
    if (lane == 0) bmus[j] = arg == 0x7fffffff ? 0 : arg;      // no finite distance (non-finite input): node 0, as a plain scan gives
  }
}

__global__ __launch_bounds__(256) void k_refine_lists_csr(const int64_t *__restrict__ indptr,
                                                          const int32_t *__restrict__ indices,
                                                          const float *__restrict__ values,
                                                          const float *__restrict__ W,
                                                          const double *__restrict__ wn64, int dim, int k,
                                                          const int32_t *__restrict__ collect_rows,
                                                          const int32_t *__restrict__ collect_cnt,
                                                          const int32_t *__restrict__ collect_list,
                                                          int32_t *__restrict__ rescan_list,
                                                          int32_t *__restrict__ list_counts, int scan_above,
                                                          int32_t *__restrict__ bmus) {
  const int lane = threadIdx.x & (kWave - 1);
  const int count = list_counts[1];
  for (int e = next_entry(list_counts, lane); e < count; e = next_entry(list_counts, lane)) {
    const int64_t j = collect_rows[e];
    const int64_t s = indptr[j];
    const int len = (int)(indptr[j + 1] - s);
    // overflowed (or empty) list: exact scan of all nodes; so is a list longer than scan_above, for which that scan
    // is the cheaper of the two
    if (collect_cnt[e] > min(kListCap, scan_above) || collect_cnt[e] < 1) {
      if (lane == 0) rescan_list[atomicAdd(&list_counts[2], 1)] = (int32_t)j;
      continue;
    }
    const int cn = min(collect_cnt[e], kListCap);
    const int32_t *lst = collect_list + (int64_t)e * kListCap;
    const double xn = csr_row_sqnorm_wave(values + s, len, lane);
    double best = INFINITY;
    int arg = 0x7fffffff;
    for (int t = 0; t < cn; ++t) {
      const int i = min(max(lst[t], 0), k - 1);
      const double d2 = sqdist_csr_wave(indices + s, values + s, len, W + (int64_t)i * dim, wn64[i], xn, dim, lane);
      if (d2 < best || (d2 == best && i < arg)) { best = d2; arg = i; }
    }
    if (lane == 0) bmus[j] = arg == 0x7fffffff ? 0 : arg;
  }
}

// Exact scan of all nodes for one sparse row from the row-major code book: wavefront w takes the nodes
// w, w + 4, ...; (best, arg) of this wavefront, ties to the lowest index.
__device__ __forceinline__ void rescan_row_major(const int32_t *__restrict__ idx, const float *__restrict__ val,
                                                 int len, const float *__restrict__ W,
                                                 const double *__restrict__ wn64, double xn, int dim, int k,
                                                 int lane, int wave, double &best, int &arg) {
  best = INFINITY;
  arg = 0x7fffffff;
  for (int i = wave; i < k; i += 4) {             // ascending within a wave: strict < keeps the lowest index
    const double d2 = sqdist_csr_wave(idx, val, len, W + (int64_t)i * dim, wn64[i], xn, dim, lane);
    if (d2 < best) { best = d2; arg = i; }
  }
}

__global__ __launch_bounds__(256) void k_rescan_csr(const int64_t *__restrict__ indptr,
                                                    const int32_t *__restrict__ indices,
                                                    const float *__restrict__ values,
                                                    const float *__restrict__ W, const double *__restrict__ wn64,
                                                    int dim, int k, const int32_t *__restrict__ rescan_list,
                                                    const int32_t *__restrict__ list_counts,
                                                    int32_t *__restrict__ bmus) {
  __shared__ double s_best[4];
  __shared__ int s_arg[4];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int count = list_counts[2];
  for (int e = blockIdx.x; e < count; e += gridDim.x) {
    const int64_t j = rescan_list[e];
    const int64_t s = indptr[j];
    const int len = (int)(indptr[j + 1] - s);
    const double xn = csr_row_sqnorm_wave(values + s, len, lane);
    double best;
    int arg;
    rescan_row_major(indices + s, values + s, len, W, wn64, xn, dim, k, lane, wave, best, arg);
    if (lane == 0) { s_best[wave] = best; s_arg[wave] = arg; }
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = 1; w < 4; ++w)
        if (s_best[w] < best || (s_best[w] == best && s_arg[w] < arg)) { best = s_best[w]; arg = s_arg[w]; }
      bmus[j] = arg == 0x7fffffff ? 0 : arg;
    }
    __syncthreads();
  }
}

// The same scan from a transposed fp32 copy of the code book, Wt[c][i] with row stride kt.  A scan from the
// row-major code book reads one 4-byte weight per node and nonzero, each from a row of its own: a memory
// transaction per weight.  From the transposed copy the weights of one column and 64 consecutive nodes are
// one 256-byte read, and a thread adds up one node's terms over the row's nonzeros:
//     d2_i = |w_i|^2 + sum_nz ((v - w_ic)^2 - w_ic^2)
// (the regrouped sum of sqdist_csr_regrouped_wave, its terms added in the order of the row instead of
// across a wavefront).  A node for which that sum is all rounding noise needs the plain sum over every
// coordinate, which has to walk the node's row of W: if any node of the scan is that close to the instance,
// the whole scan is done again from the row-major code book, as k_rescan_csr does it (an instance that
// coincides with a weight vector: rare).
// The copy is written by k_transpose_for_rescan, and only when the list of instances to scan is not empty.
constexpr int kRescanChunk = 512;        // nonzeros staged in LDS at a time
constexpr int kRescanNodes = 2;          // nodes per thread and round

__global__ __launch_bounds__(256) void k_transpose_for_rescan(const float *__restrict__ W, int k, int dim, int64_t kt,
                                                              const int32_t *__restrict__ list_counts,
                                                              float *__restrict__ Wt) {
  if (list_counts[2] == 0) return;
  __shared__ float tile[64][65];
  const int tc = (dim + 63) / 64, ti = (k + 63) / 64;
  const int x = threadIdx.x & 63, y = threadIdx.x >> 6;
  for (int64_t t = blockIdx.x; t < (int64_t)tc * ti; t += gridDim.x) {
    const int i0 = (int)(t / tc) * 64, c0 = (int)(t % tc) * 64;
    for (int r = y; r < 64; r += 4) {
      const int i = i0 + r, c = c0 + x;
      tile[r][x] = (i < k && c < dim) ? W[(int64_t)i * dim + c] : 0.f;
    }
    __syncthreads();
    for (int r = y; r < 64; r += 4) {
      const int c = c0 + r, i = i0 + x;
      if (c < dim && i < kt) Wt[(int64_t)c * kt + i] = tile[x][r];
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void k_rescan_csr_t(const int64_t *__restrict__ indptr,
                                                      const int32_t *__restrict__ indices,
                                                      const float *__restrict__ values,
                                                      const float *__restrict__ W, const float *__restrict__ Wt,
                                                      int64_t kt, const double *__restrict__ wn64, int dim, int k,
                                                      const int32_t *__restrict__ rescan_list,
                                                      const int32_t *__restrict__ list_counts,
                                                      int32_t *__restrict__ bmus) {
  __shared__ int32_t s_col[kRescanChunk];
  __shared__ float s_val[kRescanChunk];
  __shared__ double s_best[4];
  __shared__ int s_arg[4];
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  const int count = list_counts[2];
  for (int e = blockIdx.x; e < count; e += gridDim.x) {
    const int64_t j = rescan_list[e];
    const int64_t s = indptr[j];
    const int len = (int)(indptr[j + 1] - s);
    const double xn = csr_row_sqnorm_wave(values + s, len, lane);
    const double noise_scale = ((double)dim + (double)len + 2.0) * 1.862645149230957e-09;      // as in sqdist_csr_wave
    const bool fits = len <= kRescanChunk;
    if (fits) {
      for (int p = tid; p < len; p += 256) {
        s_col[p] = min(max(indices[s + p], 0), dim - 1);
        s_val[p] = values[s + p];
      }
      __syncthreads();
    }
    double best = INFINITY;
    int arg = 0x7fffffff;
    bool in_noise = false;
    for (int i0 = 0; i0 < k; i0 += 256 * kRescanNodes) {
      double acc[kRescanNodes];
      int node[kRescanNodes];
#pragma unroll
      for (int r = 0; r < kRescanNodes; ++r) {
        acc[r] = 0.0;
        node[r] = min(i0 + r * 256 + tid, k - 1);       // a thread beyond the last node reads node k - 1 and drops the result
      }
      for (int p0 = 0; p0 < len; p0 += kRescanChunk) {
        const int cn = min(kRescanChunk, len - p0);
        if (!fits) {
          __syncthreads();
          for (int p = tid; p < cn; p += 256) {
            s_col[p] = min(max(indices[s + p0 + p], 0), dim - 1);
            s_val[p] = values[s + p0 + p];
          }
          __syncthreads();
        }
#pragma unroll 4
        for (int p = 0; p < cn; ++p) {
          const float *row = Wt + (int64_t)s_col[p] * kt;
          const double v = (double)s_val[p];
#pragma unroll
          for (int r = 0; r < kRescanNodes; ++r) {
            const double wc = (double)row[node[r]];
            const double d = v - wc;
            acc[r] += d * d - wc * wc;
          }
        }
      }
#pragma unroll
      for (int r = 0; r < kRescanNodes; ++r) {
        const int i = i0 + r * 256 + tid;
        if (i < k) {                                    // ascending per thread: strict < keeps the lowest index
          const double wn = wn64[i];
          const double d2 = wn + acc[r];
          if (d2 < noise_scale * (wn + xn)) in_noise = true;
          if (d2 < best) { best = d2; arg = i; }
        }
      }
    }
    if (__syncthreads_or(in_noise)) {
      rescan_row_major(indices + s, values + s, len, W, wn64, xn, dim, k, lane, wave, best, arg);
    } else {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const double ob = __shfl_xor(best, o, kWave);
        const int oa = __shfl_xor(arg, o, kWave);
        if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
      }
    }
    if (lane == 0) { s_best[wave] = best; s_arg[wave] = arg; }
    __syncthreads();
    if (tid == 0) {
      for (int w = 1; w < 4; ++w)
        if (s_best[w] < best || (s_best[w] == best && s_arg[w] < arg)) { best = s_best[w]; arg = s_arg[w]; }
      bmus[j] = arg == 0x7fffffff ? 0 : arg;
    }
    __syncthreads();
  }
}

static int persistent_blocks(const som_ctx *c, int64_t upper) {
  int64_t b = (int64_t)c->n_cu * 8;
  if (b > upper) b = upper;
  if (b < 1) b = 1;
  return (int)b;
}

// Roundings a product term can suffer in the fp32 MFMA pass: the accumulator is flushed into a
// second one every kDenseAccumBlock features.
static double fp32_pass_roundings(int dim) {
  return (double)kDenseAccumBlock + (double)((dim + kDenseAccumBlock - 1) / kDenseAccumBlock) + 2.0;
}

// The same for the split-fp16 pass, in units of u relative to sum |x_c w'_c|.  Measured
// behaviour of v_mfma_f32_32x32x16_f16 on gfx950 (checked by a test through som_debug_mfma_f16):
// the 16 products are aligned to the largest of them and truncated 25 bits below its leading bit,
// their sum joins the accumulator with an error of at most 2 u of the result.  Priced here at
// 9 u max|product| + 2.5 u (|C| + sum|products|) per instruction: over a flush interval of f chunks
// of 32 features (6 f instructions) that is 2.5 * 6 f + 9; every flush adds one rounding, and a
// wavefront flushes at most ceil(dim / (32 f)) + 1 times per node block.
static double split_pass_roundings(int dim) {
  const int chunks = split_flush_chunks(dim);
  return 2.5 * 6.0 * chunks + 9.0 + (double)((dim + 32 * chunks - 1) / (32 * chunks)) + 2.0;
}

// The rounding model of the filter that produced the scores (mode = kCertify*).
// Roundings of the split-fp16 pass over `dim` features (see split_pass_roundings).
static double split_roundings_for(int dim) {
  const int chunks = split_flush_chunks(dim);
  return 2.5 * 6.0 * chunks + 9.0 + (double)((dim + 32 * chunks - 1) / (32 * chunks)) + 2.0;
}

MarginModel margin_model(const som_ctx *c, int mode, const int64_t *indptr, bool hot) {
  MarginModel mm{2.0 * fp32_pass_roundings(c->dim) + 4.0, 0.0, nullptr, nullptr, 0, nullptr, nullptr, 0.0, nullptr, nullptr, nullptr};
  if (mode == kCertifyCsr) {
    mm.indptr = indptr;
    mm.row_q = c->row_q;
    if (hot) {
      // the hot block's dot product: accumulation + 12 u of the split, doubled by the factor -2 of the score;
      // its product then joins the chain of the tail (one more rounding, inside the tail's own + 6)
      mm.coef_hot = 2.0 * split_roundings_for(kHot) + 24.0;
      mm.hot_xn = c->hot_xn;
      mm.hot_xscale = c->hot_xscale;
      mm.hot_wscale = c->hot_wscale;
    }
  }
  if (mode == kCertifyCoarse) {
    // One fp16 product per feature pair on the hi halves alone (coarse pass of the two-level search).  An
    // operand element v / scale is rounded to 11 significant bits, |dv| <= 2^-11 |v| + 2^-25 scale, so by
    // Cauchy-Schwarz the dot product of the rounded rows is off by at most
    //   |dx| |w'| + |hi_x| |dw| <= (2 + 2^-11) 2^-11 X Wm + floor terms = (2^14 + 8) u X Wm + ...,
    // doubled by the factor -2 of the score.  Accumulation: one chain of ceil(dim / 16) matrix instructions
    // per score, never flushed, priced per instruction like the split pass (2.5 u of the running sum each,
    // 9 u of the largest product once, + 2).  The stored c_i, the final multiply-add and the roundings of
    // w - mu and x - mu as in the split model.
    const double chain = 2.5 * (double)((c->dim + 15) / 16) + 9.0 + 2.0;
    mm.coef_xw = 2.0 * (16384.0 + 8.0) + 2.0 * chain + 4.0 + 2.0;
    mm.coef_floor = sqrt((double)c->dim);        // 2^-25 per element and operand, doubled = u
    mm.xscale = c->xscale;
    mm.wscale = c->wscale;
    mm.x_centered = 1;
  }
  if (mode == kCertifySplit) {
    // dot product: accumulation + 3 * 2^-22 of the split (= 12 u) ; both doubled by the factor -2;
    // + 4 for the stored c_i, the final multiply-add and the rounding of w - mu, + 2 for the rounding
    // of x - mu (its part that does not depend on the node cancels in every comparison).  Never
    // below the fp32 coefficient.
    const double split = 2.0 * split_pass_roundings(c->dim) + 24.0 + 4.0 + 2.0;
    if (split > mm.coef_xw) mm.coef_xw = split;
    mm.coef_floor = sqrt((double)c->dim);        // 2 * 2^-25 per element = u, |v|_1 <= sqrt(dim) |v|_2
    mm.xscale = c->xscale;
    mm.wscale = c->wscale;
    mm.x_centered = 1;
  }
  return mm;
}

hipError_t launch_certify(som_ctx *c, int64_t n, int groups, int mode, const int64_t *indptr, int32_t *bmus, bool hot,
                          const int32_t *order) {
  CandView cand{c->cand_val, c->cand_idx, c->cand_over};
  const MarginModel mm = margin_model(c, mode, indptr, hot);
  UnitWork work{0, 0, nullptr, nullptr, nullptr};
  if (mode == kCertifyCsr)
    work = UnitWork{c->csr_sweeps, c->unit_cap, c->unit_work, c->list_counts + kUnitCounts, c->collect_list};
  hipLaunchKernelGGL(k_certify, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, cand, groups, c->xn32,
                     c->wmax_bits, c->mu_norm2, mm, n, c->k, bmus, c->cand_n, c->refine_list, c->collect_rows,
                     c->collect_thr, c->collect_cnt, c->list_counts, work, order);
  return hipGetLastError();
}

// Test hook: the margin k_certify applies to every instance (the same function, the same inputs).
__global__ __launch_bounds__(256) void k_margins(const float *__restrict__ xn32, const unsigned *__restrict__ wmax_bits,
                                                 const float *__restrict__ mu_norm2, MarginModel mm, int64_t n,
                                                 double *__restrict__ out) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) out[j] = score_margin(mm, j, (double)xn32[j], (double)__uint_as_float(*wmax_bits), (double)*mu_norm2);
}

hipError_t launch_margins(som_ctx *c, int64_t n, int mode, const int64_t *indptr, double *out, bool hot) {
  hipLaunchKernelGGL(k_margins, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, c->xn32, c->wmax_bits,
                     c->mu_norm2, margin_model(c, mode, indptr, hot), n, out);
  return hipGetLastError();
}

hipError_t launch_refine_lists_dense(som_ctx *c, const float *X, const float *W, int32_t *bmus) {
  hipLaunchKernelGGL(k_refine_lists_dense, dim3(persistent_blocks(c, 1 << 20)), dim3(256), 0, c->stream, X, W,
                     c->dim, c->k, c->collect_rows, c->collect_cnt, c->collect_list, c->rescan_list, c->list_counts, bmus);
  return hipGetLastError();
}

hipError_t launch_refine_dense(som_ctx *c, const float *X, const float *W, int32_t *bmus) {
  hipLaunchKernelGGL(k_refine_dense, dim3(persistent_blocks(c, 1 << 20)), dim3(256), 0, c->stream, X, W, c->dim,
                     c->cand_idx, c->cand_n, c->refine_list, c->list_counts, bmus);
  return hipGetLastError();
}

hipError_t launch_rescan_dense(som_ctx *c, const float *X, const float *W, int32_t *bmus) {
  hipLaunchKernelGGL(k_rescan_dense, dim3(persistent_blocks(c, 1 << 20)), dim3(256), 0, c->stream, X, W, c->dim,
                     c->k, c->rescan_list, c->list_counts, bmus);
  return hipGetLastError();
}

hipError_t launch_refine_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                             const float *W, int32_t *bmus) {
  hipLaunchKernelGGL(k_refine_csr, dim3(persistent_blocks(c, 1 << 20)), dim3(256), 0, c->stream, indptr, indices,
                     values, W, c->wn64, c->dim, c->cand_idx, c->cand_n, c->refine_list, c->list_counts, bmus);
  return hipGetLastError();
}

hipError_t launch_refine_lists_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                                   const float *W, int32_t *bmus) {
  // A listed node costs a memory transaction per nonzero (its weights lie in a row of their own); the scan of all
  // nodes from the transposed copy reads the same weights 16 to a transaction, and measured 24 times cheaper per
  // (instance, node) pair on a 50 x 50 map: beyond k / 24 listed nodes the scan of everything wins.
  const int scan_above = c->Wt32 ? (c->k / 24 > 16 ? c->k / 24 : 16) : kListCap;
  hipLaunchKernelGGL(k_refine_lists_csr, dim3(persistent_blocks(c, 1 << 20)), dim3(256), 0, c->stream, indptr,
                     indices, values, W, c->wn64, c->dim, c->k, c->collect_rows, c->collect_cnt, c->collect_list,
                     c->rescan_list, c->list_counts, scan_above, bmus);
  return hipGetLastError();
}

// ---------------------------------------------------------------- distances to the BMUs
// Post-training output: Euclidean distance between every instance and the weight vector of
// the node it is mapped to, in fp64, and the mean of those distances (quantisation error).
// A wavefront per instance; a workgroup owns a contiguous block of instances and leaves one
// partial sum, the partial sums are added in index order by k_mean_of_partials: the result
// does not depend on the schedule.  A node index outside [0, k) yields NaN.

template <bool kCsr>
__global__ __launch_bounds__(256) void k_bmu_distances(const float *__restrict__ X,
                                                       const int64_t *__restrict__ indptr,
                                                       const int32_t *__restrict__ indices,
                                                       const float *__restrict__ values,
                                                       const float *__restrict__ W, int64_t n, int k, int dim,
                                                       const int32_t *__restrict__ bmus, float *__restrict__ dist,
                                                       double *__restrict__ partial) {
  __shared__ double wave_total[4];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t per_block = (n + gridDim.x - 1) / gridDim.x;
  const int64_t j0 = (int64_t)blockIdx.x * per_block;
  const int64_t j1 = j0 + per_block < n ? j0 + per_block : n;
  double total = 0.0;
  for (int64_t j = j0 + wave; j < j1; j += 4) {
    const int b = bmus[j];
    double d = NAN;
    if ((unsigned)b < (unsigned)k) {
      const float *w = W + (int64_t)b * dim;
      double d2;
      if (kCsr) {
        double wn = 0.0;
        for (int c = lane; c < dim; c += kWave) wn += (double)w[c] * (double)w[c];
        wn = wave_sum(wn);
        const int64_t rs = indptr[j];
        const int len = (int)(indptr[j + 1] - rs);
        d2 = sqdist_csr_wave(indices + rs, values + rs, len, w, wn, csr_row_sqnorm_wave(values + rs, len, lane), dim,
                             lane);
      } else {
        d2 = sqdist_dense_wave(X + j * dim, w, dim, lane);
      }
      d = sqrt(d2);
    }
    if (dist && lane == 0) dist[j] = (float)d;
    total += d;
  }
  if (lane == 0) wave_total[wave] = total;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (wave_total[0] + wave_total[1]) + (wave_total[2] + wave_total[3]);
}

__global__ __launch_bounds__(64) void k_mean_of_partials(const double *__restrict__ partial, int count, int64_t n,
                                                         double *__restrict__ out) {
  double s = 0.0;
  for (int i = threadIdx.x; i < count; i += kWave) s += partial[i];
  s = wave_sum(s);
  if (threadIdx.x == 0) *out = n > 0 ? s / (double)n : 0.0;
}

hipError_t launch_bmu_distances_on(hipStream_t stream, const float *X, const int64_t *indptr, const int32_t *indices,
                                   const float *values, int64_t n, const float *W, int k, int dim,
                                   const int32_t *bmus, float *dist, double *qerror, double *partial) {
  int blocks = (int)((n + 3) / 4);
  if (blocks > kDistBlocks) blocks = kDistBlocks;
  if (blocks < 1) blocks = 1;
  if (X)
    hipLaunchKernelGGL(k_bmu_distances<false>, dim3(blocks), dim3(256), 0, stream, X, nullptr, nullptr, nullptr, W,
                       n, k, dim, bmus, dist, partial);
  else
    hipLaunchKernelGGL(k_bmu_distances<true>, dim3(blocks), dim3(256), 0, stream, nullptr, indptr, indices, values,
                       W, n, k, dim, bmus, dist, partial);
  if (qerror)
    hipLaunchKernelGGL(k_mean_of_partials, dim3(1), dim3(64), 0, stream, partial, blocks, n, qerror);
  return hipGetLastError();
}

hipError_t launch_bmu_distances(som_ctx *c, const float *X, const int64_t *indptr, const int32_t *indices,
                                const float *values, int64_t n, const float *W, const int32_t *bmus, float *dist,
                                double *qerror) {
  return launch_bmu_distances_on(c->stream, X, indptr, indices, values, n, W, c->k, c->dim, bmus, dist, qerror,
                                 c->dist_partial);
}

hipError_t launch_rescan_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices, const float *values,
                             const float *W, int32_t *bmus) {
  if (c->Wt32) {
    hipLaunchKernelGGL(k_transpose_for_rescan, dim3(persistent_blocks(c, 1 << 20)), dim3(256), 0, c->stream, W, c->k,
                       c->dim, c->kt32, c->list_counts, c->Wt32);
    hipLaunchKernelGGL(k_rescan_csr_t, dim3(persistent_blocks(c, 1 << 20)), dim3(256), 0, c->stream, indptr, indices,
                       values, W, c->Wt32, c->kt32, c->wn64, c->dim, c->k, c->rescan_list, c->list_counts, bmus);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(k_rescan_csr, dim3(persistent_blocks(c, 1 << 20)), dim3(256), 0, c->stream, indptr, indices,
                     values, W, c->wn64, c->dim, c->k, c->rescan_list, c->list_counts, bmus);
  return hipGetLastError();
}

}  // namespace som
