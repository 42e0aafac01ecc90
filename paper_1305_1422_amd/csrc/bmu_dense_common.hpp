// Pieces shared by the two variants of the dense fp32 BMU pass (bmu_dense.hip: operand tiles
// staged through registers, any shape; bmu_dense_dl.hip: operand tiles loaded straight into
// LDS, needs dim % 4 == 0 and 16-byte aligned pointers).
//
// Both compute, for instance x and node i, the score s = c_i - 2 x.w'_i with w'_i = fl(w_i - mu)
// and c_i = |w'_i|^2 + 2 mu.w'_i, which equals |x - mu - w'_i|^2 - |x - mu|^2 exactly: the same
// ranking as the squared Euclidean distance of the BMU equation, with a rounding error that
// scales with |w - mu| instead of |w|.
#pragma once

#include "som_internal.hpp"

#include <math.h>

namespace som {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kTN = 128;          // nodes per tile
constexpr int kTI = 128;          // instances per tile
constexpr int kBK = 32;           // feature columns per LDS chunk
constexpr int kFlushChunks = kDenseAccumBlock / kBK;   // chunks between accumulator flushes
static_assert(kDenseAccumBlock % kBK == 0 && kFlushChunks >= 1, "flush interval must be whole chunks");

struct Top2 {
  float v0, v1, ov;   // two smallest scores seen by this lane, and the smallest score dropped
  int i0, i1;
};

__device__ __forceinline__ void top2_init(Top2 &L) {
  L.v0 = L.v1 = L.ov = INFINITY;
  L.i0 = L.i1 = -1;
}

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

// MFMA 32x32 output element v of a lane: local node row within the 64-node half of a wavefront.
__device__ __forceinline__ int mfma_row(int mi, int v, int lhi) { return mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3); }

// Scores of one node block, s = c_i + factor * dot (factor = -2, times the operand scales where
// the operands were scaled): push into the running lists (filter mode) or append the nodes under
// the per-instance threshold to the collected lists (collect mode).  `tot` is cleared.  With `dump`
// (filter mode, test hook) the scores of the first n_dump instances are also written out.
template <bool kCollect>
__device__ __forceinline__ void consume_scores(f32x16 (&tot)[2][2], const float *__restrict__ swn, int node0, int k,
                                               int wm, int lhi, const float (&factor)[2], Top2 (&top)[2],
                                               const float (&lim)[2],
                                               const int64_t (&slot_of)[2], int32_t *__restrict__ cnt,
                                               int32_t *__restrict__ list, float *__restrict__ dump = nullptr,
                                               int64_t n_dump = 0) {
  if (!kCollect && dump) {
    // test hook: every score of the block goes to dump[instance][node] as well (tot is read, not cleared)
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int nl = wm * 64 + mfma_row(mi, v, lhi);
        const int node = node0 + nl;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          if (node < k && slot_of[ni] < n_dump) dump[slot_of[ni] * k + node] = fmaf(factor[ni], tot[mi][ni][v], swn[nl]);
      }
  }
  if (kCollect) {
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int nl = wm * 64 + mfma_row(mi, v, lhi);
        const float wnv = swn[nl];
        const int node = node0 + nl;
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          const float s = fmaf(factor[ni], tot[mi][ni][v], wnv);
          if (s <= lim[ni] && node < k) {
            const int pos = atomicAdd(&cnt[slot_of[ni]], 1);
            if (pos < kListCap) list[slot_of[ni] * kListCap + pos] = node;
          }
          tot[mi][ni][v] = 0.f;
        }
      }
    return;
  }
  // Filter mode.  After the first node blocks a score rarely beats the second-best of its lane, so
  // four scores (consecutive nodes) are tested together: if, for no lane of the wavefront, their
  // minimum is below the lane's second-best, all four only feed the smallest-dropped-score - one
  // minimum tree and one comparison instead of four list insertions.
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int v4 = 0; v4 < 16; v4 += 4) {
      float s[2][4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float wnv = swn[wm * 64 + mfma_row(mi, v4 + e, lhi)];
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          s[ni][e] = fmaf(factor[ni], tot[mi][ni][v4 + e], wnv);
          tot[mi][ni][v4 + e] = 0.f;
        }
      }
      const float m0 = fminf(fminf(s[0][0], s[0][1]), fminf(s[0][2], s[0][3]));
      const float m1 = fminf(fminf(s[1][0], s[1][1]), fminf(s[1][2], s[1][3]));
      if (__any(m0 < top[0].v1 || m1 < top[1].v1)) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int node = node0 + wm * 64 + mfma_row(mi, v4 + e, lhi);
          top2_push(top[0], s[0][e], node);
          top2_push(top[1], s[1][e], node);
        }
      } else {
        top[0].ov = fminf(top[0].ov, m0);
        top[1].ov = fminf(top[1].ov, m1);
      }
    }
}

// Merge the four partial lists of every instance of the tile (two node halves x two lane halves)
// into kCand candidates plus the smallest dropped score, and store them.  TI = instances per
// tile; mval/midx: LDS scratch of TI*4*3 floats and TI*4*2 ints that no wavefront reads any more.
// With `rows` the tile is positions inst0 .. of that index list and the lists are stored under the
// instances' own numbers.
template <int TI>
__device__ __forceinline__ void merge_and_store(const Top2 (&top)[2], float *mval, int *midx, int tid, int wm, int wi,
                                                int l32, int lhi, int64_t inst0, int64_t n, int64_t group,
                                                CandView out, const int32_t *__restrict__ rows = nullptr) {
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
  if (tid < TI && inst0 + tid < n) {
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
    const int64_t j = group * n + (rows ? (int64_t)rows[inst0 + tid] : inst0 + tid);      // lists are stored [node group][instance]
#pragma unroll
    for (int t = 0; t < kCand; ++t) {
      out.val[j * kCand + t] = v[t];
      out.idx[j * kCand + t] = id[t];
    }
    out.over[j] = ov;
  }
}

}  // namespace som
