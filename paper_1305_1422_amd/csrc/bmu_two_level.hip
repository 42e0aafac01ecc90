// Dense best-matching-unit search in two levels (paper: BMU equation; "Parallelism": distances
// through linear algebra).
//
// The split-fp16 filter (bmu_dense_h.hip) spends three matrix products per feature on EVERY
// (instance, node) pair to get fp32-grade scores, although all it needs of most pairs is the
// knowledge that the node is not the best one.  One product on the hi halves alone gives scores with
// 11-bit operands at a third of the work, and a proven bound e_j on their error (margin.hpp).  So:
//   1. coarse pass (k_bmu_dense_h, block-minimum mode): m[b][j] = the smallest coarse score of instance
//      j among the 128 nodes of block b;
//   2. k_select_blocks: with m_j = min_b m[b][j], the BMU of j lies in a block with
//      m[b][j] <= m_j + 2 e_j - a node of any other block has an exact score above that of the node
//      that gave m_j, strictly, so it is not the BMU and does not tie with it.  The kernel writes that
//      block set as a bit mask, and a sort key made of the size class of the set (1, 2, 3-4, 5-8, ...
//      blocks; the widest class first) and its lowest block;
//   3. the instances are put in the order of their keys (segsum.hip's radix sort).  A fine-pass tile
//      works on the union of its 128 instances' sets, so one instance with a wide set (one that lies
//      between clusters, say) makes its whole tile expensive: the size class keeps such instances among
//      themselves, and within a class the lowest block puts instances with nearly the same sets side
//      by side (on a map that has begun to order itself the sets are runs of neighbouring blocks);
//   4. k_tile_lists: the union of the masks over every 128 consecutive instances of that order, as an
//      ascending list of blocks;
//   5. fine pass (k_bmu_dense_h, fine mode): the split-fp16 filter over those (tile, block) pairs only.
// Its candidates go through the exact stage like those of the one-level filter: the nodes it never saw
// are out by the argument of step 2, whatever the exact stage decides about the others.
// The price is steps 2-4 and the table m (4 bytes per instance and node block, written once and read
// twice); when every block of every tile is listed (a code book of equal rows) the fine pass is the
// whole one-level filter and the coarse pass is lost: a third more work in that worst case.
#include "margin.hpp"

namespace som {

// kParts threads per instance (one per wavefront of the workgroup, so that a wavefront reads 64 consecutive
// instances of a table row); thread p of an instance takes the blocks p, p + kParts, ... and keeps the first
// 32 of them in registers, so that the table is read once for maps of up to 32 kParts blocks (beyond that the
// rest is read again for the comparison); minima, mask words and the key are combined through LDS.
template <int kParts>
__global__ __launch_bounds__(64 * kParts) void k_select_blocks(const float *__restrict__ m, int64_t n, int blocks,
                                                              const float *__restrict__ xn32,
                                                              const unsigned *__restrict__ wmax_bits,
                                                              const float *__restrict__ mu_norm2, MarginModel mm,
                                                              int classes, int32_t *__restrict__ key,
                                                              uint32_t *__restrict__ mask) {
  constexpr int kHold = 32;
  constexpr int kWordsAtOnce = 8;               // mask words combined per round: 256 blocks
  __shared__ float s_best[kParts][64];
  __shared__ uint32_t s_bits[kParts][kWordsAtOnce][64];
  const int lane = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int64_t j = (int64_t)blockIdx.x * 64 + lane;
  const bool live = j < n;
  float held[kHold];
  float best = INFINITY;
#pragma unroll
  for (int i = 0; i < kHold; ++i) {
    const int b = part + i * kParts;
    held[i] = (live && b < blocks) ? m[(int64_t)b * n + j] : INFINITY;
    best = fminf(best, held[i]);
  }
  if (live)
    for (int b = part + kHold * kParts; b < blocks; b += kParts) best = fminf(best, m[(int64_t)b * n + j]);
  s_best[part][lane] = best;
  __syncthreads();
  best = s_best[0][lane];
#pragma unroll
  for (int p = 1; p < kParts; ++p) best = fminf(best, s_best[p][lane]);
  float t32 = INFINITY;                         // no finite score at all: every block stays in
  if (live && best < INFINITY) {
    // score_margin is the bound for a PAIR of scores (2 e_j and slack): exactly the window of step 2
    const double thr = (double)best + score_margin(mm, j, (double)xn32[j], (double)__uint_as_float(*wmax_bits), (double)*mu_norm2);
    t32 = (float)thr;                           // rounded up: no block inside the window is lost
    if ((double)t32 < thr) t32 = nextafterf(t32, INFINITY);
  }
  int listed = 0, lowest = 0x7fffffff;          // kept by part 0
  for (int w0 = 0; w0 < blocks; w0 += 32 * kWordsAtOnce) {
    uint32_t bits[kWordsAtOnce];
#pragma unroll
    for (int w = 0; w < kWordsAtOnce; ++w) bits[w] = 0;
    if (w0 == 0) {                              // the blocks held in registers: 32 kParts <= 256 of them
#pragma unroll
      for (int i = 0; i < kHold; ++i) {
        const int b = part + i * kParts;        // compile-time word and bit position up to `part`
        if (b < blocks && !(held[i] > t32)) bits[(i * kParts) >> 5] |= 1u << ((part + i * kParts) & 31);   // a NaN keeps its block in
      }
    }
    if (w0 > 0 && live) {                       // (the launcher picks kParts so that the first round is all held)
#pragma unroll
      for (int w = 0; w < kWordsAtOnce; ++w)
#pragma unroll
        for (int t = 0; t < 32 / kParts; ++t) {
          const int b = w0 + 32 * w + part + kParts * t;
          if (b < blocks && !(m[(int64_t)b * n + j] > t32)) bits[w] |= 1u << (part + kParts * t);
        }
    }
#pragma unroll
    for (int w = 0; w < kWordsAtOnce; ++w) s_bits[part][w][lane] = bits[w];
    __syncthreads();
    if (part == 0 && live) {
#pragma unroll
      for (int w = 0; w < kWordsAtOnce; ++w) {
        if (w0 + 32 * w >= blocks) break;
        uint32_t all = 0;
#pragma unroll
        for (int p = 0; p < kParts; ++p) all |= s_bits[p][w][lane];
        mask[(int64_t)((w0 >> 5) + w) * n + j] = all;
        if (all && lowest == 0x7fffffff) lowest = w0 + 32 * w + __ffs((int)all) - 1;
        listed += __popc(all);
      }
    }
    __syncthreads();
  }
  if (part == 0 && live) {
    const int size_class = listed <= 1 ? 0 : 32 - __clz(listed - 1);      // ceil(log2(listed))
    // widest sets first: their tiles are the longest workgroups of the fine pass and should not start last
    key[j] = (classes - 1 - size_class) * blocks + (lowest == 0x7fffffff ? 0 : lowest);
  }
}

// Size classes 0 .. ceil(log2(blocks)) of a block set.
static int size_classes(int blocks) {
  int classes = 1;
  while ((1 << (classes - 1)) < blocks) ++classes;
  return classes;
}

// Keys of k_select_blocks are below this.
int two_level_key_range(int blocks) { return size_classes(blocks) * blocks; }

// One wavefront per tile of 128 consecutive entries of `rows`: OR of their masks, expanded to a list.
// The masks are stored with stride n; `rows` has n entries, or *n_rows of them if n_rows is given.
__global__ __launch_bounds__(256) void k_tile_lists(const uint32_t *__restrict__ mask, const int32_t *__restrict__ rows,
                                                    int64_t n, const int32_t *__restrict__ n_rows, int blocks,
                                                    int32_t *__restrict__ tile_cnt, int32_t *__restrict__ tile_list) {
  const int lane = threadIdx.x & 63;
  const int64_t tile = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t entries = n_rows ? (int64_t)*n_rows : n;
  if (tile * 128 >= entries) return;            // uniform over the wavefront
  const int64_t p0 = tile * 128 + lane, p1 = p0 + 64;
  const int64_t r0 = p0 < entries ? rows[p0] : -1, r1 = p1 < entries ? rows[p1] : -1;
  int32_t *out = tile_list + tile * blocks;
  int count = 0;
  for (int w0 = 0; w0 < blocks; w0 += 32) {
    uint32_t bits = 0;
    if (r0 >= 0) bits |= mask[(int64_t)(w0 >> 5) * n + r0];
    if (r1 >= 0) bits |= mask[(int64_t)(w0 >> 5) * n + r1];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) bits |= __shfl_xor(bits, o, 64);
    const bool set = lane < 32 && w0 + lane < blocks && ((bits >> lane) & 1u);
    const unsigned long long bal = __ballot(set);
    if (set) out[count + __popcll(bal & ((1ull << lane) - 1ull))] = w0 + lane;
    count += __popcll(bal);
  }
  if (lane == 0) tile_cnt[tile] = count;
}

hipError_t launch_select_blocks(som_ctx *c, int64_t n) {
  const int blocks = (c->k + 127) / 128;
  if (blocks <= 128)      // 32 blocks held per thread: all of them
    hipLaunchKernelGGL(k_select_blocks<4>, dim3((unsigned)((n + 63) / 64)), dim3(256), 0, c->stream, c->coarse_min, n,
                       blocks, c->xn32, c->wmax_bits, c->mu_norm2, margin_model(c, kCertifyCoarse, nullptr),
                       size_classes(blocks), c->coarse_key, c->coarse_mask);
  else
    hipLaunchKernelGGL(k_select_blocks<8>, dim3((unsigned)((n + 63) / 64)), dim3(512), 0, c->stream, c->coarse_min, n,
                       blocks, c->xn32, c->wmax_bits, c->mu_norm2, margin_model(c, kCertifyCoarse, nullptr),
                       size_classes(blocks), c->coarse_key, c->coarse_mask);
  return hipGetLastError();
}

hipError_t launch_tile_lists(som_ctx *c, int64_t n) {
  const int blocks = (c->k + 127) / 128;
  const int64_t tiles = (n + 127) / 128;
  hipLaunchKernelGGL(k_tile_lists, dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0, c->stream, c->coarse_mask,
                     c->sort_val[0], n, nullptr, blocks, c->tile_cnt, c->tile_list);
  return hipGetLastError();
}

// The same for the instances the exact stage sweeps again (c->collect_rows, their number on the device).
hipError_t launch_collect_tile_lists(som_ctx *c, int64_t n) {
  const int blocks = (c->k + 127) / 128;
  const int64_t tiles = (n + 127) / 128;
  hipLaunchKernelGGL(k_tile_lists, dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0, c->stream, c->coarse_mask,
                     c->collect_rows, n, c->list_counts + 1, blocks, c->ctile_cnt, c->ctile_list);
  return hipGetLastError();
}

}  // namespace som
