// Dense best-matching-unit search, fp32 pass (paper: BMU equation; "Parallelism": distances
// between every instance and every node through the linear-algebra form of the Euclidean
// distance).
//
// For instance x and node w the ranking score is s = |w'|^2 - 2 x'.w' with x' = x - mu and
// w' = w - mu (|x'|^2 is common to all nodes; mu is a centring vector that leaves distances
// unchanged and shrinks the rounding error, see norms.hip).  The x'.w' contraction runs on the
// fp32 matrix cores (v_mfma_f32_32x32x2_f32); the n x k score matrix is never stored.  The MFMA
// "M" side carries nodes and the "N" side instances, so each lane owns one instance column of a
// 32x32 block and 16 of its node rows: the running minimum over nodes needs no cross-lane
// traffic until the very end.
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
// time share a node group, so its weight vectors stay in every L2.  Tiles of
// both operands ([row][k], k contiguous, exactly the layout of X and W in memory) are staged
// through double-buffered LDS in chunks of kBK = 32 columns, prefetched through registers; the
// centring vector is subtracted on the way.
#include "som_internal.hpp"

#include <math.h>

namespace som {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTN = 128;          // nodes per tile
constexpr int kTI = 128;          // instances per tile
constexpr int kBK = 32;           // columns per LDS chunk
constexpr int kLS = kBK + 4;      // LDS row stride in floats: 16-byte aligned, conflict-free b128 reads
constexpr int kFlushChunks = kDenseAccumBlock / kBK;   // chunks between accumulator flushes
static_assert(kDenseAccumBlock % kBK == 0 && kFlushChunks >= 1, "flush interval must be whole chunks");

struct Top2 {
  float v0, v1, ov;   // two smallest scores seen by this lane, and the smallest score dropped
  int i0, i1;
};

__device__ __forceinline__ void top2_push(Top2 &L, float s, int node) {
  // Nodes reach a lane in ascending index order, so strict comparisons keep the lower index
  // ahead among equal scores.
  const bool c0 = s < L.v0;
  const bool c1 = s < L.v1;
  L.ov = c1 ? L.v1 : fminf(L.ov, s);
  L.i1 = c0 ? L.i0 : (c1 ? node : L.i1);
  L.v1 = c0 ? L.v0 : fminf(L.v1, s);
  L.i0 = c0 ? node : L.i0;
  L.v0 = fminf(L.v0, s);
}

__device__ __forceinline__ bool cand_less(float a, int ai, float b, int bi) {
  return a < b || (a == b && (unsigned)ai < (unsigned)bi);
}

// Four consecutive columns c..c+3 of one row, zero outside the matrix.
template <bool kVec4>
__device__ __forceinline__ f32x4 load_row4(const float *__restrict__ base, int64_t row, bool row_ok, int dim,
                                           int c) {
  f32x4 r = {0.f, 0.f, 0.f, 0.f};
  if (row_ok) {
    const float *p = base + row * dim + c;
    if (kVec4) {
      if (c < dim) r = *reinterpret_cast<const f32x4 *>(p);
    } else {
      if (c + 0 < dim) r[0] = p[0];
      if (c + 1 < dim) r[1] = p[1];
      if (c + 2 < dim) r[2] = p[2];
      if (c + 3 < dim) r[3] = p[3];
    }
  }
  return r;
}

// kCollect == false: instances are rows inst0 .. of X; output = candidate lists (CandView).
// kCollect == true : instances are X[rows[slot]] for slot < *n_slots; output = every node with
//                    score <= thr[slot], appended to list[slot][..kListCap) with count cnt[slot].
template <bool kVec4, bool kCollect>
__global__ __launch_bounds__(256, 2) void k_bmu_dense(const float *__restrict__ X, const float *__restrict__ W,
                                                      const float *__restrict__ mu,
                                                      const float *__restrict__ wn, int64_t n, int k, int dim,
                                                      CandView out, const int32_t *__restrict__ rows,
                                                      const int32_t *__restrict__ n_slots,
                                                      const float *__restrict__ thr, int32_t *__restrict__ cnt,
                                                      int32_t *__restrict__ list) {
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

  // fetch() only issues the global loads; the centring subtraction happens in stage(), after the
  // MFMA work of the current chunk, so that the load latency stays hidden behind that work.
  f32x4 rw[4], rx[4], rm;
  auto fetch = [&](int t) {
    const int nb = nb_first + t / nK, kc = t % nK;
    const int c = kc * kBK + ld_c4;
    rm = load_row4<kVec4>(mu, 0, true, dim, c);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int64_t node = (int64_t)nb * kTN + ld_row + 32 * p;
      rw[p] = load_row4<kVec4>(W, node, node < k, dim, c);
      rx[p] = load_row4<kVec4>(X, xrow[p], xok[p], dim, c);
    }
  };
  auto stage = [&](int t) {
    const int buf = t & 1;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      *reinterpret_cast<f32x4 *>(&sW[buf][(ld_row + 32 * p) * kLS + ld_c4]) = rw[p] - rm;
      *reinterpret_cast<f32x4 *>(&sX[buf][(ld_row + 32 * p) * kLS + ld_c4]) = rx[p] - rm;
    }
    const int nb = nb_first + t / nK;
    if (t % nK == 0 && tid < kTN) {
      const int node = nb * kTN + tid;
      sWn[nb & 1][tid] = node < k ? wn[node] : INFINITY;    // padded nodes can never win
    }
  };

  Top2 top[2];
  float lim[2];                       // collect mode: per-instance threshold
  int64_t slot_of[2];
#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    top[ni].v0 = top[ni].v1 = top[ni].ov = INFINITY;
    top[ni].i0 = top[ni].i1 = -1;
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

    if (last_k) {
      const float *swn = sWn[nb & 1];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int nl = wm * 64 + mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
          const float wnv = swn[nl];
          const int node = nb * kTN + nl;
#pragma unroll
          for (int ni = 0; ni < 2; ++ni) {
            const float s = fmaf(-2.f, tot[mi][ni][v], wnv);
            if (kCollect) {
              if (s <= lim[ni]) {
                const int pos = atomicAdd(&cnt[slot_of[ni]], 1);
                if (pos < kListCap) list[slot_of[ni] * kListCap + pos] = node;
              }
            } else {
              top2_push(top[ni], s, node);
            }
            tot[mi][ni][v] = 0.f;
          }
        }
    }

    if (t + 1 < total) stage(t + 1);
    __syncthreads();
  }
  if (kCollect) return;

  // Merge the four partial lists of every instance (two node halves x two lane halves).
  float *mval = &sW[0][0];                                  // [kTI][4][3]
  int *midx = reinterpret_cast<int *>(&sX[0][0]);           // [kTI][4][2]
#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    const int il = wi * 64 + ni * 32 + l32;
    const int contrib = wm * 2 + lhi;
    float *pv = mval + (il * 4 + contrib) * 3;
    int *pi = midx + (il * 4 + contrib) * 2;
    pv[0] = top[ni].v0; pv[1] = top[ni].v1; pv[2] = top[ni].ov;
    pi[0] = top[ni].i0; pi[1] = top[ni].i1;
  }
  __syncthreads();
  if (tid < kTI && inst0 + tid < n) {
    float v[kCand];
    int id[kCand];
    float ov = INFINITY;
#pragma unroll
    for (int t = 0; t < kCand; ++t) { v[t] = INFINITY; id[t] = -1; }
    for (int cidx = 0; cidx < 4; ++cidx) {
      const float *pv = mval + (tid * 4 + cidx) * 3;
      const int *pi = midx + (tid * 4 + cidx) * 2;
      ov = fminf(ov, pv[2]);
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const float x = pv[e];
        const int xi = pi[e];
        if (xi < 0) continue;
        if (!cand_less(x, xi, v[kCand - 1], id[kCand - 1])) { ov = fminf(ov, x); continue; }
        if (id[kCand - 1] >= 0) ov = fminf(ov, v[kCand - 1]);
        bool c[kCand];
#pragma unroll
        for (int t = 0; t < kCand; ++t) c[t] = cand_less(x, xi, v[t], id[t]);
#pragma unroll
        for (int t = kCand - 1; t >= 1; --t) {
          const float nv = c[t - 1] ? v[t - 1] : (c[t] ? x : v[t]);
          const int nid = c[t - 1] ? id[t - 1] : (c[t] ? xi : id[t]);
          v[t] = nv; id[t] = nid;
        }
        if (c[0]) { v[0] = x; id[0] = xi; }
      }
    }
    const int64_t j = (int64_t)blockIdx.y * n + inst0 + tid;      // lists are stored [node group][instance]
#pragma unroll
    for (int t = 0; t < kCand; ++t) {
      out.val[j * kCand + t] = v[t];
      out.idx[j * kCand + t] = id[t];
    }
    out.over[j] = ov;
  }
}

static bool use_vec4(const som_ctx *c, const float *X, const float *W) {
  return (c->dim % 4 == 0) && (((uintptr_t)X | (uintptr_t)W | (uintptr_t)c->mu) % 16 == 0);
}

// Number of node groups for n instances: enough workgroups for about eight rounds over the chip.
int bmu_dense_groups(const som_ctx *c, int64_t n) {
  const int64_t tiles = (n + kTI - 1) / kTI;
  const int nNB = (c->k + kTN - 1) / kTN;
  const int64_t slots = 2ll * c->n_cu;
  int64_t want = (8 * slots + tiles - 1) / tiles;
  if (want > nNB) want = nNB;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  const int nb_per = (int)((nNB + want - 1) / want);
  return (nNB + nb_per - 1) / nb_per;
}

hipError_t launch_bmu_dense(som_ctx *c, const float *X, int64_t n, const float *W) {
  CandView out{c->cand_val, c->cand_idx, c->cand_over};
  const unsigned blocks = (unsigned)((n + kTI - 1) / kTI);
  const unsigned groups = (unsigned)bmu_dense_groups(c, n);
  if (use_vec4(c, X, W))
    hipLaunchKernelGGL((k_bmu_dense<true, false>), dim3(blocks, groups), dim3(256), 0, c->stream, X, W, c->mu,
                       c->wn32, n, c->k, c->dim, out, nullptr, nullptr, nullptr, nullptr, nullptr);
  else
    hipLaunchKernelGGL((k_bmu_dense<false, false>), dim3(blocks, groups), dim3(256), 0, c->stream, X, W, c->mu,
                       c->wn32, n, c->k, c->dim, out, nullptr, nullptr, nullptr, nullptr, nullptr);
  return hipGetLastError();
}

// Repeats the sweep for the instances in c->collect_rows (their number is only known on the
// device: the grid covers the worst case and surplus workgroups leave at once).
hipError_t launch_bmu_dense_collect(som_ctx *c, const float *X, int64_t n, const float *W) {
  CandView out{nullptr, nullptr, nullptr};
  const unsigned blocks = (unsigned)((n + kTI - 1) / kTI);
  // usually only a few instance tiles are live: share the node blocks out over up to 16 workgroups each
  const int nNB = (c->k + kTN - 1) / kTN;
  const unsigned splits = (unsigned)(nNB < 16 ? nNB : 16);
  if (use_vec4(c, X, W))
    hipLaunchKernelGGL((k_bmu_dense<true, true>), dim3(blocks, splits), dim3(256), 0, c->stream, X, W, c->mu, c->wn32, n,
                       c->k, c->dim, out, c->collect_rows, c->list_counts + 1, c->collect_thr, c->collect_cnt,
                       c->collect_list);
  else
    hipLaunchKernelGGL((k_bmu_dense<false, true>), dim3(blocks, splits), dim3(256), 0, c->stream, X, W, c->mu, c->wn32, n,
                       c->k, c->dim, out, c->collect_rows, c->list_counts + 1, c->collect_thr, c->collect_cnt,
                       c->collect_list);
  return hipGetLastError();
}

}  // namespace som
