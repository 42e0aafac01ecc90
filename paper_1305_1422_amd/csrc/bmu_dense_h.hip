// Dense best-matching-unit search, filter pass on the fp16 matrix cores with split operands
// (paper: BMU equation; "Parallelism": distances through linear algebra).
//
// Same ranking as the fp32 pass (bmu_dense_dl.hip), from scores s = |w'_i|^2 - 2 x'.w'_i with w' = fl(w - mu)
// and x' = fl(x - mu) (the planes of the instances are the library's own, so they hold centred rows;
// the score differs from the fp32 pass's c_i - 2 x.w'_i by the rounding of x - mu only).  The
// dot product is evaluated as three fp16 MFMAs on the hi/lo planes written by split_f16.hip:
//     x.w' = sx sw (hi_x.hi_w + hi_x.lo_w + lo_x.hi_w) (1 + O(2^-22)),
// accumulated in fp32 by v_mfma_f32_32x32x16_f16.  On gfx950 that instruction issues in 8 passes
// for 16 k-values where the fp32 one needs 16 passes for 2: three of them per k-step are 5.3 times
// the fp32 rate.  The exact stage (bmu_exact.hip) decides as before; only its margin differs.
//
// Each wavefront owns 64 nodes x 64 instances (2 x 2 MFMA blocks) and sweeps the workgroup's group
// of node blocks of 128.  A workgroup has 4 wavefronts, 128 instances and two LDS stages of
// (128 + 128) rows x 128 bytes (64 KB), two workgroups per CU: at this MFMA rate a chunk is
// multiplied in about half a microsecond, so the gap every barrier leaves in the matrix pipe
// matters, and a second workgroup with barriers of its own fills it.  (A shape with 8 wavefronts,
// 256 instances and three stages, one workgroup per CU, moves a quarter less data through L2 but
// measured 3-12 % slower on the three dense configurations and is no longer compiled.)  The 128
// bytes of a tile row are one chunk of the split layout: 32 hi halves, 32 lo halves.  Tiles are
// loaded straight into LDS with the XOR swizzle of the fp32 pass (the two passes share the row
// geometry, so the same swizzle makes the ds_read_b128 operand reads conflict-free): 16-byte
// slot q of a row holds hi columns 8 q .. 8 q + 7 (q < 4) or lo columns 8 (q - 4) .. (q >= 4),
// and the MFMA k-step t takes slot 2 t + (lane >> 5) of either plane.
//
// The grid is one-dimensional and decoded so that the node groups of one instance tile are
// workgroups 8 apart: the dispatcher hands those to the same XCD one after the other, they
// stream the same instance tile at about the same time, and all but the first find it in that
// XCD's L2.
#include "bmu_dense_common.hpp"

namespace som {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void *lptr_h_t;

constexpr int kHRow = 32;                  // floats per tile row (= 64 halves = one chunk of 32 columns)
constexpr int kHWTile = kTN * kHRow;       // floats
constexpr int kHWI = 2;                    // 64-instance columns of wavefronts in a workgroup

__device__ __forceinline__ unsigned lds_address_h(const float *p) { return (unsigned)(size_t)(lptr_h_t)p; }

#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
// Direct-to-LDS load of 16 bytes per lane (see bmu_dense_dl.hip for why this is inline assembly),
// in the addressing form "wavefront-uniform 64-bit base in scalar registers + unsigned 32-bit byte
// offset per lane": the per-lane offsets are loop constants and the base advances with scalar
// arithmetic, so a load costs no vector ALU instruction.
__device__ __forceinline__ void load16_to_lds_h(const void *base, unsigned lane_offset, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_offset), "s"(base), "s"(lds_base)
               : "memory", "m0");
}
// The same for 4 bytes per lane: lane l's word goes to LDS byte address lds_base + 4 l.
__device__ __forceinline__ void load4_to_lds_h(const void *base, unsigned lane_offset, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1"
               :
               : "v"(lane_offset), "s"(base), "s"(lds_base)
               : "memory", "m0");
}
// 16 bytes per lane from a full 64-bit address per lane (rows gathered through an index list).
__device__ __forceinline__ void load16_to_lds_v(const void *lane_address, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(lane_address), "s"(lds_base) : "memory", "m0");
}
#pragma clang diagnostic pop

enum { kHFilter = 0, kHCollect = 1, kHDump = 2, kHPartial = 3, kHFine = 4 };

__device__ __forceinline__ f16x8 as_halves(f32x4 v) { return __builtin_bit_cast(f16x8, v); }

// kMode: kHFilter keeps candidates per instance; kHCollect runs over the instances listed in `rows`
// (their number is *n_slots) and appends every node whose score is at most thr[slot] to the
// instance's list; kHDump writes every score to dump[slot * k + node] (test hook); kHPartial is the
// hot-column block of the sparse search (csr_hot.hip): the plain dot products times the code book's
// scale go to dump[(node block * n + instance) * 128 + node within the block], four neighbouring nodes
// of one instance per 16-byte store.  No candidates, no constants.
// kHFine is the second pass of the two-level search (bmu_two_level.hip): the instance tiles are taken
// through the index list `rows` (all n instances, ordered so that neighbours in the list have nearly the
// same sets of candidate blocks), and the workgroups of tile t share out the tcnt[t] node blocks listed,
// ascending, in tlist[t * blocks of the map ..] instead of all of them; candidates are stored under the
// instances' own numbers.  Collect mode takes such lists too (for the tiles of ITS index list) when the
// search ran in two levels: a node outside the blocks listed for an instance cannot be its BMU.
// `unit` numbers the (instance tile, node group) pairs; see the decoding below.
template <int kMode>
__device__ __forceinline__ void bmu_dense_h_unit(const float *__restrict__ Xh, const float *__restrict__ Wh,
                                                 const float *__restrict__ wc, const float *__restrict__ xscale,
                                                 const float *__restrict__ wscale, int64_t n, int k, int nK,
                                                 int flush_chunks, int groups, CandView out, float *__restrict__ dump,
                                                 const int32_t *__restrict__ rows, const int32_t *__restrict__ n_slots,
                                                 const float *__restrict__ thr, int32_t *__restrict__ cnt,
                                                 int32_t *__restrict__ list, const int32_t *__restrict__ tcnt,
                                                 const int32_t *__restrict__ tlist, const int64_t unit) {
  constexpr bool kCollect = kMode == kHCollect;
  constexpr bool kDump = kMode == kHDump;
  constexpr bool kPartial = kMode == kHPartial;
  constexpr bool kFine = kMode == kHFine;
  constexpr bool kGather = kCollect || kFine;        // instance tiles through the index list `rows`
  constexpr int WI = kHWI;
  constexpr int kHTI = 64 * WI;              // instances per tile
  constexpr int kHXTile = kHTI * kHRow;      // floats
  constexpr int kHStages = 2;
  constexpr int kWSlots = 16 / (2 * WI);     // W-tile load instructions per wavefront and chunk
  __shared__ __attribute__((aligned(16))) float sW[kHStages][kHWTile];
  __shared__ __attribute__((aligned(16))) float sX[kHStages][kHXTile];
  __shared__ float sWn[4][kTN];      // node constants of the node blocks in flight

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WI;          // which 64-node half of the tile
  const int wi = wave % WI;          // which 64-instance column of the tile
  const int l32 = lane & 31;
  const int lhi = lane >> 5;

  // workgroup -> (instance tile, node group)
  const int64_t n_inst = kCollect ? (int64_t)*n_slots : n;      // slots this launch covers
  const int64_t ntiles = (n_inst + kHTI - 1) / kHTI;
  const int xcd = (int)(unit & 7);
  const int64_t slot_id = unit >> 3;
  const int group = (int)(slot_id % groups);
  const int64_t tile = (slot_id / groups) * 8 + xcd;
  if (tile >= ntiles) return;        // uniform over the workgroup
  const int64_t inst0 = tile * kHTI;

  // the node blocks of this workgroup: positions nb_first .. nb_first + nNB - 1 of the map's blocks, or
  // (fine mode) of the tile's own ascending list
  const int nNB_all = (k + kTN - 1) / kTN;
  const bool listed = kFine || (kCollect && tlist != nullptr);   // (collect mode: the lists are optional)
  const int32_t *blist = listed ? tlist + tile * (int64_t)nNB_all : nullptr;
  const int nNB_avail = listed ? min(tcnt[tile], nNB_all) : nNB_all;
  const int nb_per = (nNB_avail + groups - 1) / groups;
  const int nb_first = group * nb_per;
  const int nNB = min(nb_per, nNB_avail - nb_first);
  if (nNB <= 0) {                    // uniform over the workgroup
    if (kFine && tid < kHTI && inst0 + tid < n) {      // certify reads a list per (instance, group): an empty one
      const int64_t j = (int64_t)group * n + rows[inst0 + tid];
#pragma unroll
      for (int t = 0; t < kCand; ++t) { out.val[j * kCand + t] = INFINITY; out.idx[j * kCand + t] = -1; }
      out.over[j] = INFINITY;
    }
    return;
  }
  const int total = nK * nNB;

  // ---- loader: one instruction fills 8 tile rows (64 lanes x 16 bytes); wavefront w issues W slots
  // 2 w, 2 w + 1 and X slots 4 w .. 4 w + 3; lane l sits at row + (l >> 3), slot position l & 7.
  // Rows past the end of an operand are redirected to its last row: their products land in output
  // rows / columns that are never used (padded nodes carry c_i = +inf, padded instances are not stored).
  const int ld_rloc = lane >> 3;
  const int ld_pos = lane & 7;
  const unsigned row_bytes = (unsigned)nK * (kHRow * 4);
  const char *xbase = reinterpret_cast<const char *>(Xh) + inst0 * (int64_t)row_bytes;
  const int64_t last_inst = n_inst - 1 - inst0;  // >= 0
  unsigned xoff[4], woff[kWSlots], wq[kWSlots];
  const char *xptr[4];                           // collect mode: gathered rows, one address per lane
  int wrow[kWSlots];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = 8 * (4 * wave + i) + ld_rloc;
    const int q = ld_pos ^ ((row & 7) ^ ((row >> 3) & 1));
    const int rclamped = row < last_inst ? row : (int)last_inst;
    xoff[i] = (unsigned)rclamped * row_bytes + 16u * q;
    xptr[i] = kGather ? reinterpret_cast<const char *>(Xh) + (int64_t)rows[inst0 + rclamped] * row_bytes + 16 * q : nullptr;
  }
#pragma unroll
  for (int i = 0; i < kWSlots; ++i) {
    wrow[i] = 8 * (kWSlots * wave + i) + ld_rloc;
    wq[i] = 16u * (ld_pos ^ ((wrow[i] & 7) ^ ((wrow[i] >> 3) & 1)));
    woff[i] = 0;
  }
  const unsigned lds_w = lds_address_h(&sW[0][kWSlots * 256 * wave]);   // 256 floats per slot
  const unsigned lds_x = lds_address_h(&sX[0][1024 * wave]);    // 4 slots
  const unsigned lds_wn = lds_address_h(&sWn[0][0]);
  const unsigned wn_off = (unsigned)(wave * 64 + lane) * 4u;
  int ld_ord = 0, ld_kc = 0;        // ordinal of the node block being loaded within this workgroup's run
  int ld_nb = listed ? blist[nb_first] : nb_first;
  auto issue_loads = [&](int buf) {
    const char *wbase = reinterpret_cast<const char *>(Wh) + (int64_t)ld_nb * kTN * row_bytes;
    if (ld_kc == 0) {                                           // entering a node block
      const int last_node = k - 1 - ld_nb * kTN;                // >= 0
#pragma unroll
      for (int i = 0; i < kWSlots; ++i) woff[i] = (unsigned)(wrow[i] < last_node ? wrow[i] : last_node) * row_bytes + wq[i];
      // node constants of the block: wc is padded to whole blocks with +inf (such nodes can never
      // win), so the 128 values are loaded like the tiles, as the oldest operation of the batch
      if (!kPartial && wave < 2)
        load4_to_lds_h(wc + (int64_t)ld_nb * kTN, wn_off,
                       lds_wn + __builtin_amdgcn_readfirstlane(ld_ord & 3) * (kTN * 4) + wave * 256);
    }
    const unsigned off = (unsigned)ld_kc * (kHRow * 4);
#pragma unroll
    for (int i = 0; i < kWSlots; ++i) load16_to_lds_h(wbase + off, woff[i], lds_w + buf * (kHWTile * 4) + i * 1024);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (kGather) load16_to_lds_v(xptr[i] + off, lds_x + buf * (kHXTile * 4) + i * 1024);
      else load16_to_lds_h(xbase + off, xoff[i], lds_x + buf * (kHXTile * 4) + i * 1024);
    }
    if (++ld_kc == nK) {
      ld_kc = 0;
      ++ld_ord;
      ld_nb = listed ? (ld_ord < nNB ? blist[nb_first + ld_ord] : 0) : ld_nb + 1;
    }
  };

  // ---- reader
  const int rd_swz = (l32 & 7) ^ ((l32 >> 3) & 1);
  int rd_off[4];                     // [0], [1]: hi plane of k-steps 0, 1; [2], [3]: lo plane
#pragma unroll
  for (int g = 0; g < 4; ++g) rd_off[g] = 4 * ((2 * g + lhi) ^ rd_swz);
  const int a_base = (wm * 64 + l32) * kHRow;
  const int b_base = (wi * 64 + l32) * kHRow;

  Top2 top[2];
  float lim[2];
  int64_t slot_of[2];
  float factor[2];
  const float sw = *wscale;
#pragma unroll
  for (int ni = 0; ni < 2; ++ni) {
    top2_init(top[ni]);
    slot_of[ni] = inst0 + wi * 64 + ni * 32 + l32;
    const bool live = slot_of[ni] < n_inst;
    const int64_t inst = live ? (kGather ? (int64_t)rows[slot_of[ni]] : slot_of[ni]) : 0;
    factor[ni] = (live && !kPartial) ? -2.f * xscale[inst] * sw : 0.f;
    lim[ni] = (kCollect && live) ? thr[slot_of[ni]] : -INFINITY;
  }

  f32x16 acc[2][2], tot[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) tot[mi][ni][v] = 0.f;

  // Operands of one k-step (16 features): the hi and lo planes of this wavefront's two 32-node and
  // two 32-instance row blocks, eight 16-byte LDS reads per lane.
  struct Operands { f16x8 g1[2], g2[2], h1[2], h2[2]; };
  auto read_operands = [&](Operands &o, int st, int ks) {
    const float *pw = &sW[st][a_base];
    const float *px = &sX[st][b_base];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      o.g1[b] = as_halves(*reinterpret_cast<const f32x4 *>(pw + b * 32 * kHRow + rd_off[ks]));
      o.g2[b] = as_halves(*reinterpret_cast<const f32x4 *>(pw + b * 32 * kHRow + rd_off[2 + ks]));
      o.h1[b] = as_halves(*reinterpret_cast<const f32x4 *>(px + b * 32 * kHRow + rd_off[ks]));
      o.h2[b] = as_halves(*reinterpret_cast<const f32x4 *>(px + b * 32 * kHRow + rd_off[2 + ks]));
    }
  };
  // Twelve MFMAs of one k-step; the four output blocks take turns, so that an accumulator is reused
  // every fourth instruction only.  The small cross products go first.  `fresh`: the accumulators
  // start from C = 0 as an operand of the instruction itself, which spares clearing 64 registers.
  auto multiply = [&](const Operands &o, bool fresh) {
    __builtin_amdgcn_s_setprio(1);      // the wavefront that has operands ready goes first on the SIMD (-1.6 %)
    if (fresh) {
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(o.g2[mi], o.h1[ni], zero, 0, 0, 0);
    } else {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(o.g2[mi], o.h1[ni], acc[mi][ni], 0, 0, 0);
    }
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(o.g1[mi], o.h2[ni], acc[mi][ni], 0, 0, 0);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_f16(o.g1[mi], o.h1[ni], acc[mi][ni], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
  };

  // Two stages: chunk t + 1 is loaded during iteration t, every wavefront waits for its own loads
  // before the barrier that ends the iteration, and every operand is read after that barrier; the
  // second workgroup on the CU fills the gap.
  issue_loads(0);
  __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wavefront's direct-to-LDS loads have landed
  __syncthreads();

  // Wavefronts that share a SIMD flush their accumulators in alternate chunks, so that one's
  // additions overlap the other's MFMAs: the wavefronts of two workgroups that sit next to each
  // other in the launch order.  An interval is at most
  // flush_chunks chunks (2 or 4, see split_flush_chunks; the exact stage's margin prices it).
  const int flush_mask = flush_chunks - 1;
  const int flush_phase = (int)(slot_id & 1) * (flush_chunks >> 1);
  bool fresh = true;
  Operands op0, op1;
  int stage = 0;                                 // t % kHStages
  for (int t = 0; t < total; ++t) {
    const int ord = t / nK, kc = t % nK;           // ordinal of the node block in this workgroup's run
    const int next_stage = stage ^ 1;
    // the stage that is loaded now held chunk t - 1, which every wavefront has left
    if (t + 1 < total) issue_loads(next_stage);
    read_operands(op0, stage, 0);
    read_operands(op1, stage, 1);
    multiply(op0, fresh);
    multiply(op1, false);

    const bool last_k = (kc == nK - 1);
    fresh = last_k || ((kc + flush_phase) & flush_mask) == flush_mask;
    if (fresh) {
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
          for (int v = 0; v < 16; ++v) tot[mi][ni][v] += acc[mi][ni][v];
    }
    if (last_k) {
      const int nb = listed ? blist[nb_first + ord] : nb_first + ord;
      if (kPartial) {
        // lane = instance wi 64 + ni 32 + l32 of the tile; registers 4 g .. 4 g + 3 of an output block are
        // nodes wm 64 + mi 32 + 8 g + 4 lhi .. + 3 of the node block, which lie side by side in the table
        // [node block][instance][128 nodes]: one 16-byte store each, and the 128 x 128 results of a
        // workgroup and node block fill one contiguous 64 KB run
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
          const int64_t inst = inst0 + wi * 64 + ni * 32 + l32;
          float *prow = dump + ((int64_t)nb * n + inst) * kTN + wm * 64 + 4 * lhi;
#pragma unroll
          for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const f32x4 val = {sw * tot[mi][ni][4 * g], sw * tot[mi][ni][4 * g + 1], sw * tot[mi][ni][4 * g + 2],
                                 sw * tot[mi][ni][4 * g + 3]};
              if (inst < n) *reinterpret_cast<f32x4 *>(prow + mi * 32 + 8 * g) = val;
#pragma unroll
              for (int e = 0; e < 4; ++e) tot[mi][ni][4 * g + e] = 0.f;
            }
        }
      } else if (kDump) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int nl = wm * 64 + mfma_row(mi, v, lhi);
            const int node = nb * kTN + nl;
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
              if (node < k && slot_of[ni] < n) dump[slot_of[ni] * k + node] = fmaf(factor[ni], tot[mi][ni][v], sWn[ord & 3][nl]);
              tot[mi][ni][v] = 0.f;
            }
          }
      } else {
        consume_scores<kCollect>(tot, sWn[ord & 3], nb * kTN, k, wm, lhi, factor, top, lim, slot_of, cnt, list);
      }
    }

    __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
    __syncthreads();
    stage = next_stage;
  }
  if (kDump || kCollect || kPartial) return;
  merge_and_store<kHTI>(top, &sW[0][0], reinterpret_cast<int *>(&sX[0][0]), tid, wm, wi, l32, lhi, inst0, n, group,
                        out, kFine ? rows : nullptr);
}

// Filter, dump, partial and fine modes: one unit per workgroup.  Collect mode: the number
// of live instance tiles is only known on the device, so a fixed grid walks the units; its size is a
// multiple of 8, which keeps unit mod 8 = workgroup mod 8 = the XCD the decoding assumes.
template <int kMode>
__global__ __launch_bounds__(128 * kHWI, 2) void k_bmu_dense_h(const float *__restrict__ Xh, const float *__restrict__ Wh,
                                                        const float *__restrict__ wc,
                                                        const float *__restrict__ xscale,
                                                        const float *__restrict__ wscale,
                                                        int64_t n, int k, int nK, int flush_chunks,
                                                        int groups, CandView out, float *__restrict__ dump,
                                                        const int32_t *__restrict__ rows,
                                                        const int32_t *__restrict__ n_slots,
                                                        const float *__restrict__ thr, int32_t *__restrict__ cnt,
                                                        int32_t *__restrict__ list, const int32_t *__restrict__ tcnt,
                                                        const int32_t *__restrict__ tlist) {
  if (kMode == kHCollect) {
    const int64_t ntiles = ((int64_t)*n_slots + 64 * kHWI - 1) / (64 * kHWI);
    const int64_t units = (ntiles + 7) / 8 * 8 * groups;
    for (int64_t unit = blockIdx.x; unit < units; unit += gridDim.x) {
      bmu_dense_h_unit<kMode>(Xh, Wh, wc, xscale, wscale, n, k, nK, flush_chunks, groups, out, dump, rows,
                              n_slots, thr, cnt, list, tcnt, tlist, unit);
      __syncthreads();               // the next unit reuses the LDS stages
    }
  } else {
    bmu_dense_h_unit<kMode>(Xh, Wh, wc, xscale, wscale, n, k, nK, flush_chunks, groups, out, dump, rows,
                            n_slots, thr, cnt, list, tcnt, tlist, (int64_t)blockIdx.x);
  }
}

// Node groups per instance tile: enough workgroups for about ten rounds over the resident slots, at
// least two when there are many node blocks (shorter workgroups even out the last round: -3 % on
// configuration 5), and a block count per group that leaves the last group as full as the others
// (20 node blocks in groups of 3 leave one group of 2 and measured 3 % slower than groups of 2 or 4).
int bmu_dense_h_groups(const som_ctx *c, int64_t n) {
  const int64_t tiles = (n + 64 * kHWI - 1) / (64 * kHWI);
  const int nNB = (c->k + kTN - 1) / kTN;
  const int64_t slots = (int64_t)c->n_cu * 2;      // two workgroups per CU
  int64_t want = (10 * slots + tiles - 1) / tiles;
  if (want < 2 && nNB >= 16) want = 2;
  if (want > nNB) want = nNB;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  int nb_per = (int)((nNB + want - 1) / want);
  // among nb_per - 1, nb_per, nb_per + 1 take the one that wastes the fewest block slots
  int best = nb_per;
  int64_t best_waste = (int64_t)((nNB + nb_per - 1) / nb_per) * nb_per - nNB;
  for (int cand = nb_per - 1; cand <= nb_per + 1; cand += 2) {
    if (cand < 1 || (nNB + cand - 1) / cand > 64) continue;
    const int64_t waste = (int64_t)((nNB + cand - 1) / cand) * cand - nNB;
    if (waste < best_waste) { best_waste = waste; best = cand; }
  }
  return (nNB + best - 1) / best;
}

// Workgroups per instance tile in the second pass of the two-level search: a tile usually lists a few
// node blocks only, so the tiles themselves fill the chip unless there are few of them.
int bmu_dense_h_fine_groups(const som_ctx *c, int64_t n) {
  const int64_t tiles = (n + 64 * kHWI - 1) / (64 * kHWI);
  const int nNB = (c->k + kTN - 1) / kTN;
  const int64_t slots = (int64_t)c->n_cu * 2;
  int64_t want = (4 * slots + tiles - 1) / tiles;
  if (want > 8) want = 8;
  if (want > nNB) want = nNB;
  if (want < 1) want = 1;
  return (int)want;
}

hipError_t launch_bmu_dense_h(som_ctx *c, int64_t n, float *dump) {
  const int groups = bmu_dense_h_groups(c, n);
  const int64_t tiles = (n + 64 * kHWI - 1) / (64 * kHWI);
  const int64_t blocks = (tiles + 7) / 8 * 8 * groups;
  const int nK = (c->dim + 31) / 32;
  CandView out{c->cand_val, c->cand_idx, c->cand_over};
  const float *Xh = reinterpret_cast<const float *>(c->Xh);
  const float *Wh = reinterpret_cast<const float *>(c->Wh);
  if (dump)
    hipLaunchKernelGGL((k_bmu_dense_h<kHDump>), dim3((unsigned)blocks), dim3(128 * kHWI), 0, c->stream, Xh, Wh,
                       c->wn32, c->xscale, c->wscale, n, c->k, nK, split_flush_chunks(c->dim), groups, out, dump, nullptr, nullptr, nullptr,
                       nullptr, nullptr, nullptr, nullptr);
  else
    hipLaunchKernelGGL((k_bmu_dense_h<kHFilter>), dim3((unsigned)blocks), dim3(128 * kHWI), 0, c->stream, Xh, Wh,
                       c->wn32, c->xscale, c->wscale, n, c->k, nK, split_flush_chunks(c->dim), groups, out, dump, nullptr, nullptr, nullptr,
                       nullptr, nullptr, nullptr, nullptr);
  return hipGetLastError();
}

// Second pass of the two-level search: the split-fp16 filter over the instance tiles of the order
// c->sort_val[0] and the node blocks c->tile_list lists for each (c->tile_cnt of them).
hipError_t launch_bmu_dense_h_fine(som_ctx *c, int64_t n) {
  const int groups = bmu_dense_h_fine_groups(c, n);
  const int64_t tiles = (n + 64 * kHWI - 1) / (64 * kHWI);
  const int64_t blocks = (tiles + 7) / 8 * 8 * groups;
  const int nK = (c->dim + 31) / 32;
  CandView out{c->cand_val, c->cand_idx, c->cand_over};
  hipLaunchKernelGGL((k_bmu_dense_h<kHFine>), dim3((unsigned)blocks), dim3(128 * kHWI), 0, c->stream,
                     reinterpret_cast<const float *>(c->Xh), reinterpret_cast<const float *>(c->Wh), c->wn32,
                     c->xscale, c->wscale, n, c->k, nK, split_flush_chunks(c->dim), groups, out, nullptr, c->sort_val[0],
                     nullptr, nullptr, nullptr, nullptr, c->tile_cnt, c->tile_list);
  return hipGetLastError();
}

// Hot-column block of the sparse search: P[node block][n][128] = (x_hot . w'_hot) / (scale of the instance), from the
// planes c->hot_Xh [n][kHot] and c->hot_Wh [k][kHot]; the same tiling and launch shape as the filter.
hipError_t launch_hot_partial(som_ctx *c, int64_t n) {
  const int groups = bmu_dense_h_groups(c, n);
  const int64_t tiles = (n + 64 * kHWI - 1) / (64 * kHWI);
  const int64_t blocks = (tiles + 7) / 8 * 8 * groups;
  CandView out{nullptr, nullptr, nullptr};
  hipLaunchKernelGGL((k_bmu_dense_h<kHPartial>), dim3((unsigned)blocks), dim3(128 * kHWI), 0, c->stream,
                     reinterpret_cast<const float *>(c->hot_Xh), reinterpret_cast<const float *>(c->hot_Wh), nullptr,
                     nullptr, c->hot_wscale, n, c->k, kHot / 32, split_flush_chunks(kHot), groups, out, c->hot_P,
                     nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  return hipGetLastError();
}

// Repeats the sweep for the instances in c->collect_rows.  Their number is only known on the
// device: the grid is the worst case capped at eight workgroups per CU, and the workgroups walk
// the live units.  Usually only a few instance tiles are live, so the node blocks are shared out
// over up to 16 workgroups.
// lists: the node blocks of every tile of 128 collect slots are given in c->ctile_cnt / c->ctile_list.
hipError_t launch_bmu_dense_h_collect(som_ctx *c, int64_t n, bool lists) {
  const int nNB = (c->k + kTN - 1) / kTN;
  const int groups = nNB < 16 ? nNB : 16;
  const int64_t tiles = (n + 64 * kHWI - 1) / (64 * kHWI);
  int64_t blocks = (tiles + 7) / 8 * 8 * groups;
  if (blocks > (int64_t)c->n_cu * 8) blocks = (int64_t)c->n_cu * 8;
  blocks = (blocks + 7) / 8 * 8;
  const int nK = (c->dim + 31) / 32;
  CandView out{nullptr, nullptr, nullptr};
  hipLaunchKernelGGL((k_bmu_dense_h<kHCollect>), dim3((unsigned)blocks), dim3(128 * kHWI), 0, c->stream,
                     reinterpret_cast<const float *>(c->Xh), reinterpret_cast<const float *>(c->Wh), c->wn32,
                     c->xscale, c->wscale, n, c->k, nK, split_flush_chunks(c->dim), groups, out, nullptr, c->collect_rows, c->list_counts + 1,
                     c->collect_thr, c->collect_cnt, c->collect_list, lists ? c->ctile_cnt : nullptr,
                     lists ? c->ctile_list : nullptr);
  return hipGetLastError();
}

}  // namespace som
