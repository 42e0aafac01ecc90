// Dense best-matching-unit search, fp32 pass (paper: BMU equation; "Parallelism": distances
// between every instance and every node through the linear-algebra form of the Euclidean
// distance).
//
// For instance x and node i the ranking score is s = c_i - 2 x.w'_i (see bmu_dense_common.hpp).
// The x.w' contraction runs on the fp32 matrix cores (v_mfma_f32_32x32x2_f32); the n x k score
// matrix is never stored.  The MFMA "M" side carries nodes and the "N" side instances, so each
// lane owns one instance column of a 32x32 block and 16 of its node rows: the running minimum
// over nodes needs no cross-lane traffic until the very end.
//
// fp32 scores cannot decide the BMU on their own: the rounding error of a long dot product is
// of the order of the gap between the two best nodes.  The kernel is therefore a filter with
// two modes.
//   filter:  per instance it emits the kCand smallest scores with their nodes plus the
//            smallest score it dropped; bmu_exact.hip decides among the candidates that lie
//            within a proven error bound of the minimum.
//   collect: for the instances where a dropped score lies inside the bound too, the same
//            sweep is repeated over just those instances (row indirection) and every node
//            whose score is below the instance's threshold is appended to a list.
// To keep the bound small the MFMA accumulator is flushed into a second fp32 accumulator every
// kDenseAccumBlock columns (two-level summation).
//
// Work decomposition: one 256-thread workgroup owns kTI = 128 instances and sweeps one group of
// node blocks of kTN = 128 nodes each; 2 x 2 wavefronts, each a 64 x 64 patch = 2 x 2 MFMA
// blocks.  The node groups (grid y) exist for load balance only: with few, long workgroups the
// last round of workgroups leaves most compute units idle.  Workgroups that run at the same
// time share a node group, so its weight vectors stay in every L2.
//
// This file holds the general variant: tiles of both operands ([row][k], k contiguous, exactly
// the layout of X and W in memory) go global -> registers -> LDS in chunks of kBK = 32 columns,
// double-buffered, with bounds checks per element, so any dim and any alignment work.  The
// faster variant for dim % 4 == 0 is in bmu_dense_dl.hip; the launchers at the end choose.
#include "bmu_dense_common.hpp"

namespace som {

constexpr int kLS = kBK + 4;      // LDS row stride in floats: 16-byte aligned, conflict-free b128 reads

// Four consecutive columns c..c+3 of one row, zero outside the matrix.
__device__ __forceinline__ f32x4 load_row4(const float *__restrict__ base, int64_t row, bool row_ok, int dim, int c) {
  f32x4 r = {0.f, 0.f, 0.f, 0.f};
  if (row_ok) {
    const float *p = base + row * dim + c;
    if (c + 0 < dim) r[0] = p[0];
    if (c + 1 < dim) r[1] = p[1];
    if (c + 2 < dim) r[2] = p[2];
    if (c + 3 < dim) r[3] = p[3];
  }
  return r;
}

// kCollect == false: instances are rows inst0 .. of X; output = candidate lists (CandView).
// kCollect == true : instances are X[rows[slot]] for slot < *n_slots; output = every node with
//                    score <= thr[slot], appended to list[slot][..kListCap) with count cnt[slot].
// Wc = centred code book w', wc = the per-node constants c_i.
template <bool kCollect>
__global__ __launch_bounds__(256, 2) void k_bmu_dense(const float *__restrict__ X, const float *__restrict__ Wc,
                                                      const float *__restrict__ wc, int64_t n, int k, int dim,
                                                      CandView out, const int32_t *__restrict__ rows,
                                                      const int32_t *__restrict__ n_slots,
                                                      const float *__restrict__ thr, int32_t *__restrict__ cnt,
                                                      int32_t *__restrict__ list, float *__restrict__ dump) {
  __shared__ __attribute__((aligned(16))) float sW[2][kTN * kLS];
  __shared__ __attribute__((aligned(16))) float sX[2][kTI * kLS];
  __shared__ float sWn[2][kTN];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave >> 1;          // which 64-node half of the tile
  const int wi = wave & 1;           // which 64-instance half of the tile
  const int l32 = lane & 31;
  const int lhi = lane >> 5;
  const int64_t inst0 = (int64_t)blockIdx.x * kTI;
  const int64_t n_inst = kCollect ? (int64_t)*n_slots : n;
  if (inst0 >= n_inst) return;       // uniform over the workgroup

  // node blocks swept by this workgroup: the blockIdx.y-th share of them (node group)
  const int nK = (dim + kBK - 1) / kBK;
  const int nNB_all = (k + kTN - 1) / kTN;
  const int nb_per = (nNB_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int nb_first = (int)blockIdx.y * nb_per;
  const int nNB = min(nb_per, nNB_all - nb_first);
  if (nNB <= 0) return;              // uniform over the workgroup
  const int total = nK * nNB;

  // loader coordinates: 4 float4 per operand per thread and chunk
  const int ld_row = tid >> 3;       // + 32 p
  const int ld_c4 = (tid & 7) * 4;

  int64_t xrow[4];
  bool xok[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int64_t slot = inst0 + ld_row + 32 * p;
    xok[p] = slot < n_inst;
    xrow[p] = kCollect ? (xok[p] ? (int64_t)rows[slot] : 0) : slot;
  }

  f32x4 rw[4], rx[4];
  auto fetch = [&](int t) {
    const int nb = nb_first + t / nK, kc = t % nK;
    const int c = kc * kBK + ld_c4;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int64_t node = (int64_t)nb * kTN + ld_row + 32 * p;
      rw[p] = load_row4(Wc, node, node < k, dim, c);
      rx[p] = load_row4(X, xrow[p], xok[p], dim, c);
    }
  };
  auto stage = [&](int t) {
    const int buf = t & 1;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      *reinterpret_cast<f32x4 *>(&sW[buf][(ld_row + 32 * p) * kLS + ld_c4]) = rw[p];
      *reinterpret_cast<f32x4 *>(&sX[buf][(ld_row + 32 * p) * kLS + ld_c4]) = rx[p];
    }
    const int nb = nb_first + t / nK;
    if (t % nK == 0 && tid < kTN) {
      const int node = nb * kTN + tid;
      sWn[nb & 1][tid] = node < k ? wc[node] : INFINITY;    // padded nodes can never win
    }
  };

  const float kMinusTwo[2] = {-2.f, -2.f};
  Top2 top[2];
  float lim[2];                       // collect mode: per-instance threshold
  int64_t slot_of[2];
#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    top2_init(top[ni]);
    slot_of[ni] = inst0 + wi * 64 + ni * 32 + l32;
    lim[ni] = (kCollect && slot_of[ni] < n_inst) ? thr[slot_of[ni]] : -INFINITY;
  }

  f32x16 acc[2][2], tot[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) { acc[mi][ni][v] = 0.f; tot[mi][ni][v] = 0.f; }

  fetch(0);
  stage(0);
  __syncthreads();

  const int a_off = (wm * 64 + l32) * kLS + lhi * 4;
  const int b_off = (wi * 64 + l32) * kLS + lhi * 4;

  for (int t = 0; t < total; ++t) {
    const int nb = nb_first + t / nK, kc = t % nK;
    if (t + 1 < total) fetch(t + 1);

    const float *pw = &sW[t & 1][a_off];
    const float *px = &sX[t & 1][b_off];
#pragma unroll
    for (int kk = 0; kk < kBK; kk += 8) {
      const f32x4 a0 = *reinterpret_cast<const f32x4 *>(pw + kk);
      const f32x4 a1 = *reinterpret_cast<const f32x4 *>(pw + 32 * kLS + kk);
      const f32x4 b0 = *reinterpret_cast<const f32x4 *>(px + kk);
      const f32x4 b1 = *reinterpret_cast<const f32x4 *>(px + 32 * kLS + kk);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[s], b0[s], acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[s], b1[s], acc[0][1], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s], b0[s], acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[s], b1[s], acc[1][1], 0, 0, 0);
      }
    }

    const bool last_k = (kc == nK - 1);
    if (last_k || (kc % kFlushChunks) == kFlushChunks - 1) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
          for (int v = 0; v < 16; ++v) { tot[mi][ni][v] += acc[mi][ni][v]; acc[mi][ni][v] = 0.f; }
    }
    if (last_k) consume_scores<kCollect>(tot, sWn[nb & 1], nb * kTN, k, wm, lhi, kMinusTwo, top, lim, slot_of, cnt, list, dump, n);

    if (t + 1 < total) stage(t + 1);
    __syncthreads();
  }
  if (kCollect) return;
  merge_and_store<kTI>(top, &sW[0][0], reinterpret_cast<int *>(&sX[0][0]), tid, wm, wi, l32, lhi, inst0, n, blockIdx.y,
                  out);
}

// ---------------------------------------------------------------- launchers (both variants)
static bool direct_loads_ok(const som_ctx *c, const float *X) {
  return (c->dim % 4 == 0) && (((uintptr_t)X | (uintptr_t)c->Wc) % 16 == 0);
}

// Number of node groups for n instances: enough workgroups for about twelve rounds over the chip
// (measured: 8 rounds lose 3 % to the ragged last round, more than 16 gain nothing).
int bmu_dense_groups(const som_ctx *c, int64_t n) {
  const int64_t tiles = (n + kTI - 1) / kTI;
  const int nNB = (c->k + kTN - 1) / kTN;
  const int64_t slots = 2ll * c->n_cu;
  int64_t want = (12 * slots + tiles - 1) / tiles;
  if (want > nNB) want = nNB;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  const int nb_per = (int)((nNB + want - 1) / want);
  return (nNB + nb_per - 1) / nb_per;
}

hipError_t launch_bmu_dense(som_ctx *c, const float *X, int64_t n, float *dump) {
  CandView out{c->cand_val, c->cand_idx, c->cand_over};
  const dim3 grid((unsigned)((n + kTI - 1) / kTI), (unsigned)bmu_dense_groups(c, n));
  if (direct_loads_ok(c, X)) return launch_bmu_dense_dl(c, X, n, grid, false, dump);
  hipLaunchKernelGGL((k_bmu_dense<false>), grid, dim3(256), 0, c->stream, X, c->Wc, c->wn32, n, c->k, c->dim, out,
                     nullptr, nullptr, nullptr, nullptr, nullptr, dump);
  return hipGetLastError();
}

// Repeats the sweep for the instances in c->collect_rows (their number is only known on the
// device: the grid covers the worst case and surplus workgroups leave at once).  Usually only
// a few instance tiles are live, so the node blocks are shared out over up to 16 workgroups.
hipError_t launch_bmu_dense_collect(som_ctx *c, const float *X, int64_t n) {
  CandView out{nullptr, nullptr, nullptr};
  const int nNB = (c->k + kTN - 1) / kTN;
  const dim3 grid((unsigned)((n + kTI - 1) / kTI), (unsigned)(nNB < 16 ? nNB : 16));
  if (direct_loads_ok(c, X)) return launch_bmu_dense_dl(c, X, n, grid, true, nullptr);
  hipLaunchKernelGGL((k_bmu_dense<true>), grid, dim3(256), 0, c->stream, X, c->Wc, c->wn32, n, c->k, c->dim, out,
                     c->collect_rows, c->list_counts + 1, c->collect_thr, c->collect_cnt, c->collect_list, nullptr);
  return hipGetLastError();
}

}  // namespace som
