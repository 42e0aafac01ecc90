// Dense best-matching-unit search, coarse pass of the two-level search (paper: BMU equation;
// "Parallelism": distances through linear algebra).  See bmu_two_level.hip for what the pass is for.
//
// Scores s = |w'_i|^2 - 2 x'.w'_i from ONE fp16 product per feature, on the hi halves of the split
// planes alone (split_f16.hip: rows of 64-feature chunks, 128 bytes each), accumulated in fp32 by
// v_mfma_f32_32x32x16_f16 without intermediate flushes; kept is only the smallest score per instance and
// block of 128 nodes.
//
// With one product per operand pair the pass is bound by LDS traffic, not by the matrix pipes: a
// wavefront tile of 64 x 64 outputs (the shape of the three-product pass, bmu_dense_h.hip) reads 1 KB of
// operands per MFMA.  So a wavefront owns 128 nodes x 64 instances here (4 x 2 MFMA blocks, 128
// accumulator registers, 0.75 KB per MFMA), a workgroup has 8 wavefronts on 256 nodes x 256 instances,
// two LDS stages of (256 + 256) rows x 128 bytes (128 KB), one workgroup per CU: measured 1.4 times the
// rate of the 64 x 64 shape at 1,000 features.  The 128 nodes of a wavefront are one block of the table,
// so the minima need no exchange between wavefronts.  Tile loads, swizzle and grid decoding are those of
// bmu_dense_h.hip.
#include "bmu_dense_common.hpp"

namespace som {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void *lptr_c_t;

constexpr int kCRow = 32;                  // floats per tile row (= 64 halves = one chunk of 64 features)
constexpr int kCTN = 256, kCTI = 256;      // nodes / instances per workgroup tile
constexpr int kCThreads = 512;

__device__ __forceinline__ unsigned lds_address_c(const float *p) { return (unsigned)(size_t)(lptr_c_t)p; }

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// Direct-to-LDS load of 16 bytes per lane, "wavefront-uniform base + 32-bit byte offset per lane" form
// (see bmu_dense_dl.hip for why this is inline assembly).
__device__ __forceinline__ void load16_to_lds_c(const void *base, unsigned lane_offset, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_offset), "s"(base), "s"(lds_base)
               : "memory", "m0");
}
// The same for 4 bytes per lane: lane l's word goes to LDS byte address lds_base + 4 l.
__device__ __forceinline__ void load4_to_lds_c(const void *base, unsigned lane_offset, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1"
               :
               : "v"(lane_offset), "s"(base), "s"(lds_base)
               : "memory", "m0");
}

#pragma clang diagnostic pop

__device__ __forceinline__ f16x8 as_halves_c(f32x4 v) { return __builtin_bit_cast(f16x8, v); }

// kDump = false: block_min[node block of 128][instance] = smallest score of the pair.
// kDump = true (test hook): every score to dump[instance * k + node].
// wc: node constants c_i, readable for i < k_const (a multiple of 128 >= k, +inf past k).
template <bool kDump>
__global__ __launch_bounds__(kCThreads, 1) void k_bmu_coarse(const float *__restrict__ Xh, const float *__restrict__ Wh,
                                                             const float *__restrict__ wc, int k_const,
                                                             const float *__restrict__ xscale,
                                                             const float *__restrict__ wscale, int64_t n, int k,
                                                             int nK, int groups, float *__restrict__ out) {
  __shared__ __attribute__((aligned(16))) float sW[2][kCTN * kCRow];
  __shared__ __attribute__((aligned(16))) float sX[2][kCTI * kCRow];
  __shared__ float sWn[2][kCTN];     // node constants of the node tiles in flight, by parity of the tile's ordinal

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2;          // which 128-node half of the tile
  const int wi = wave & 3;           // which 64-instance quarter of the tile
  const int l32 = lane & 31;
  const int lhi = lane >> 5;

  // workgroup -> (instance tile, node group): the groups of one instance tile are workgroups 8 apart
  const int64_t ntiles = (n + kCTI - 1) / kCTI;
  const int xcd = (int)(blockIdx.x & 7);
  const int64_t slot_id = blockIdx.x >> 3;
  const int group = (int)(slot_id % groups);
  const int64_t tile = (slot_id / groups) * 8 + xcd;
  if (tile >= ntiles) return;        // uniform over the workgroup
  const int64_t inst0 = tile * kCTI;
  const int nNB_all = (k + kCTN - 1) / kCTN;
  const int nb_per = (nNB_all + groups - 1) / groups;
  const int nb_first = group * nb_per;
  const int nNB = min(nb_per, nNB_all - nb_first);
  if (nNB <= 0) return;              // uniform over the workgroup
  const int total = nK * nNB;

  // ---- loader: one instruction fills 8 tile rows; wavefront w issues W slots 4 w .. 4 w + 3 and X slots
  // 4 w .. 4 w + 3.  Rows past the end of an operand are redirected to its last row (their outputs are
  // never used: such nodes get the constant +inf, such instances are not stored).
  const int ld_rloc = lane >> 3;
  const int ld_pos = lane & 7;
  const unsigned row_bytes = (unsigned)nK * (kCRow * 4);
  const char *xbase = reinterpret_cast<const char *>(Xh) + inst0 * (int64_t)row_bytes;
  const int64_t last_inst = n - 1 - inst0;       // >= 0
  unsigned xoff[4], woff[4], wq[4];
  int wrow[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = 8 * (4 * wave + i) + ld_rloc;
    const int q = ld_pos ^ ((row & 7) ^ ((row >> 3) & 1));
    const int rclamped = row < last_inst ? row : (int)last_inst;
    xoff[i] = (unsigned)rclamped * row_bytes + 16u * q;
    wrow[i] = row;
    wq[i] = 16u * q;
    woff[i] = 0;
  }
  const unsigned lds_w = lds_address_c(&sW[0][1024 * wave]);     // 4 slots of 256 floats
  const unsigned lds_x = lds_address_c(&sX[0][1024 * wave]);
  const unsigned lds_wn = lds_address_c(&sWn[0][0]);
  // Up to 128 features the whole instance tile fits the two X stages: it is loaded once, with the first node tile,
  // and only the node tiles stream (half the traffic from L2 into LDS, which is what bounds the pass at so few
  // features per tile).
  const bool x_stays = nK <= 2;
  int ld_nb = nb_first, ld_kc = 0;
  auto issue_loads = [&](int buf) {
    const char *wbase = reinterpret_cast<const char *>(Wh) + (int64_t)ld_nb * kCTN * row_bytes;
    if (ld_kc == 0) {                                             // entering a node tile
      const int last_node = k - 1 - ld_nb * kCTN;                 // >= 0
#pragma unroll
      for (int i = 0; i < 4; ++i) woff[i] = (unsigned)(wrow[i] < last_node ? wrow[i] : last_node) * row_bytes + wq[i];
      // node constants of the tile, as the oldest operation of the batch.  Past the padded constants the
      // last one is read again: either +inf, or a block of the table that is not written at all
      if (wave < 4) {
        const int node = min(ld_nb * kCTN + wave * 64 + lane, k_const - 1);
        load4_to_lds_c(wc, (unsigned)node * 4u, lds_wn + ((ld_nb - nb_first) & 1) * (kCTN * 4) + wave * 256);
      }
    }
    const unsigned off = (unsigned)ld_kc * (kCRow * 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) load16_to_lds_c(wbase + off, woff[i], lds_w + buf * (kCTN * kCRow * 4) + i * 1024);
    if (!x_stays) {
#pragma unroll
      for (int i = 0; i < 4; ++i) load16_to_lds_c(xbase + off, xoff[i], lds_x + buf * (kCTI * kCRow * 4) + i * 1024);
    } else if (ld_nb == nb_first) {                               // chunk kc of the instance tile lives in sX[kc]
#pragma unroll
      for (int i = 0; i < 4; ++i) load16_to_lds_c(xbase + off, xoff[i], lds_x + ld_kc * (kCTI * kCRow * 4) + i * 1024);
    }
    if (++ld_kc == nK) { ld_kc = 0; ++ld_nb; }
  };

  // ---- reader: 16-byte slot 2 t + (lane >> 5) of a row holds this lane's 8 features of k-step t
  const int rd_swz = (l32 & 7) ^ ((l32 >> 3) & 1);
  int rd_off[4];
#pragma unroll
  for (int g = 0; g < 4; ++g) rd_off[g] = 4 * ((2 * g + lhi) ^ rd_swz);
  const int a_base = (wm * 128 + l32) * kCRow;
  const int b_base = (wi * 64 + l32) * kCRow;

  const float sw = *wscale;
  float factor[2];
#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    const int64_t inst = inst0 + wi * 64 + ni * 32 + l32;
    factor[ni] = inst < n ? -2.f * xscale[inst] * sw : 0.f;
  }

  f32x16 acc[4][2];
  // Operands of two k-steps (ks and ks + 2 of the chunk's four): 12 LDS reads of 16 bytes for 16 MFMAs.
  struct Operands { f16x8 g1[4], g2[4], h1[2], h2[2]; };
  auto read_operands = [&](Operands &o, int st, int xst, int ks) {
    const float *pw = &sW[st][a_base];
    const float *px = &sX[xst][b_base];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      o.g1[b] = as_halves_c(*reinterpret_cast<const f32x4 *>(pw + b * 32 * kCRow + rd_off[ks]));
      o.g2[b] = as_halves_c(*reinterpret_cast<const f32x4 *>(pw + b * 32 * kCRow + rd_off[2 + ks]));
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      o.h1[b] = as_halves_c(*reinterpret_cast<const f32x4 *>(px + b * 32 * kCRow + rd_off[ks]));
      o.h2[b] = as_halves_c(*reinterpret_cast<const f32x4 *>(px + b * 32 * kCRow + rd_off[2 + ks]));
    }
  };
  // `fresh`: the accumulators start from C = 0 as an operand of the instruction itself.
  auto multiply = [&](const Operands &o, bool fresh) {
    __builtin_amdgcn_s_setprio(1);
    if (fresh) {
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(o.g2[mi], o.h2[ni], zero, 0, 0, 0);
    } else {
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(o.g2[mi], o.h2[ni], acc[mi][ni], 0, 0, 0);
    }
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(o.g1[mi], o.h1[ni], acc[mi][ni], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
  };

  // Two stages: chunk t + 1 is loaded during iteration t, every wavefront waits for its own loads before
  // the barrier that ends the iteration, and every operand is read after that barrier.
  issue_loads(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wavefront's direct-to-LDS loads have landed
  __syncthreads();

  bool fresh = true;
  Operands op0, op1;
  int stage = 0;
  for (int t = 0; t < total; ++t) {
    const int ord = t / nK, kc = t % nK;         // ordinal of the node tile in this workgroup's run
    if (t + 1 < total) issue_loads(stage ^ 1);   // that stage held chunk t - 1, which every wavefront has left
    const int xstage = x_stays ? kc : stage;
    read_operands(op0, stage, xstage, 0);
    read_operands(op1, stage, xstage, 1);
    multiply(op0, fresh);
    multiply(op1, false);
    fresh = (kc == nK - 1);
    if (fresh) {
      const int nb = nb_first + ord;
      const float *swn = &sWn[ord & 1][wm * 128];
      if (kDump) {
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int nl = mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
            const int node = nb * kCTN + wm * 128 + nl;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
              const int64_t inst = inst0 + wi * 64 + ni * 32 + l32;
              if (node < k && inst < n) out[inst * k + node] = fmaf(factor[ni], acc[mi][ni][v], swn[nl]);
            }
          }
      } else {
        // smallest score per instance over this wavefront's 128 nodes = one block of the table: over the
        // lane's 64 nodes (pairs: one three-way minimum per two scores), then the other lane half
        const int block = nb * 2 + wm;
        if (block * 128 < k) {                   // uniform over the wavefront
#pragma unroll
          for (int ni = 0; ni < 2; ++ni) {
            float m = INFINITY;
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
              for (int v = 0; v < 16; v += 2) {
                const int nl = mi * 32 + 8 * (v >> 2) + 4 * lhi + (v & 3);
                const float s0 = fmaf(factor[ni], acc[mi][ni][v], swn[nl]);
                const float s1 = fmaf(factor[ni], acc[mi][ni][v + 1], swn[nl + 1]);
                m = fminf(fminf(m, s0), s1);
              }
            m = fminf(m, __shfl_xor(m, 32, 64));
            const int64_t inst = inst0 + wi * 64 + ni * 32 + l32;
            if (lhi == 0 && inst < n) out[(int64_t)block * n + inst] = m;
          }
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
    __syncthreads();
    stage ^= 1;
  }
}

// Node groups per instance tile: enough workgroups for several rounds over the CUs (one workgroup each).
static int bmu_coarse_groups(const som_ctx *c, int64_t n) {
  const int64_t tiles = (n + kCTI - 1) / kCTI;
  const int nNB = (c->k + kCTN - 1) / kCTN;
  int64_t want = (8 * (int64_t)c->n_cu + tiles - 1) / tiles;
  if (want > nNB) want = nNB;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  const int nb_per = (int)((nNB + want - 1) / want);
  return (nNB + nb_per - 1) / nb_per;
}

// c->Xh1, c->Wh1 -> c->coarse_min [ceil(k/128)][n], or with `dump` every score [n][k] (test hook).
hipError_t launch_bmu_coarse(som_ctx *c, int64_t n, float *dump) {
  const int groups = bmu_coarse_groups(c, n);
  const int64_t tiles = (n + kCTI - 1) / kCTI;
  const int64_t blocks = (tiles + 7) / 8 * 8 * groups;
  const int nK = (c->dim + 63) / 64;
  const int k_const = (c->k + kTN - 1) / kTN * kTN;      // the node constants are padded to whole blocks of 128
  const float *Xh = reinterpret_cast<const float *>(c->Xh1);
  const float *Wh = reinterpret_cast<const float *>(c->Wh1);
  if (dump)
    hipLaunchKernelGGL((k_bmu_coarse<true>), dim3((unsigned)blocks), dim3(kCThreads), 0, c->stream, Xh, Wh, c->wn32,
                       k_const, c->xscale, c->wscale, n, c->k, nK, groups, dump);
  else
    hipLaunchKernelGGL((k_bmu_coarse<false>), dim3((unsigned)blocks), dim3(kCThreads), 0, c->stream, Xh, Wh, c->wn32,
                       k_const, c->xscale, c->wscale, n, c->k, nK, groups, c->coarse_min);
  return hipGetLastError();
}

}  // namespace som
