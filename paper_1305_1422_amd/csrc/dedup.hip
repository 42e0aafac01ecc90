// Bit-identical code-book rows (paper: BMU equation with ties to the lowest node index; option -n).
//
// A bubble neighbourhood gives every node whose radius covers the same set of chosen nodes the same
// weight vector, bit for bit (the smoothing adds the same sources in the same order).  Such a node
// can never be a BMU unless it has the lowest index of its class, but to the filter pass the whole
// class is one big tie that no rounding bound can break: the candidate lists overflow and the
// instance falls through to the exact rescan of all nodes.  So before a search on such a map the
// duplicates are found and taken out of the filter pass by setting their node constant c_i to
// +inf; the exact stage needs no change (a duplicate ties with its representative there and loses
// on the index).
//
//   k_row_hash      64-bit hash of the raw bits of every row (a commutative sum over the columns, so
//                   the order in which lanes add is irrelevant)
//   k_dedup_insert  open-addressing table keyed by the hash, each slot keeps the lowest node index
//   k_dedup_mark    a node whose slot names a lower index compares its row with that node's, bit by
//                   bit, and masks itself if they are equal.  Unequal rows with equal hashes are
//                   left alone: a missed duplicate costs time, never correctness.
#include "som_internal.hpp"

#include <math.h>

namespace som {

__device__ __forceinline__ uint64_t mix64(uint64_t z) {      // the finaliser of the splitmix64 generator
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void k_row_hash(const float *__restrict__ W, int k, int dim,
                                                  uint64_t *__restrict__ hash) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int nwaves = gridDim.x * (blockDim.x / kWave);
  for (int i = wave; i < k; i += nwaves) {
    const float *w = W + (int64_t)i * dim;
    uint64_t h = 0;
    for (int c = lane; c < dim; c += kWave)
      h += mix64(((uint64_t)(unsigned)c << 32) | (uint64_t)__float_as_uint(w[c]));
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) h += (uint64_t)__shfl_xor((long long)h, o, kWave);
    if (lane == 0) hash[i] = h ? h : 1;                      // 0 marks an empty slot
  }
}

__global__ __launch_bounds__(256) void k_dedup_clear(unsigned long long *__restrict__ keys,
                                                     int32_t *__restrict__ lowest, int slots) {
  for (int s = blockIdx.x * blockDim.x + threadIdx.x; s < slots; s += gridDim.x * blockDim.x) {
    keys[s] = 0ull;
    lowest[s] = 0x7fffffff;
  }
}

// slots is a power of two >= 2 k, so the table is at most half full and every probe sequence ends.
__global__ __launch_bounds__(256) void k_dedup_insert(const uint64_t *__restrict__ hash, int k,
                                                      unsigned long long *__restrict__ keys,
                                                      int32_t *__restrict__ lowest, int slots) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= k) return;
  const unsigned long long h = hash[i];
  int s = (int)(h & (unsigned long long)(slots - 1));
  for (int probe = 0; probe < slots; ++probe) {
    const unsigned long long prev = atomicCAS(&keys[s], 0ull, h);
    if (prev == 0ull || prev == h) {
      atomicMin(&lowest[s], i);
      return;
    }
    s = (s + 1) & (slots - 1);
  }
}

__global__ __launch_bounds__(256) void k_dedup_mark(const float *__restrict__ W, int k, int dim,
                                                    const uint64_t *__restrict__ hash,
                                                    const unsigned long long *__restrict__ keys,
                                                    const int32_t *__restrict__ lowest, int slots,
                                                    float *__restrict__ node_const) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  const int nwaves = gridDim.x * (blockDim.x / kWave);
  for (int i = wave; i < k; i += nwaves) {
    const unsigned long long h = hash[i];
    int s = (int)(h & (unsigned long long)(slots - 1));
    int rep = i;
    for (int probe = 0; probe < slots; ++probe) {
      const unsigned long long key = keys[s];
      if (key == h) { rep = lowest[s]; break; }
      if (key == 0ull) break;                                // not reached: every hash was inserted
      s = (s + 1) & (slots - 1);
    }
    if (rep >= i) continue;                                  // the lowest index of its class stays
    const float *a = W + (int64_t)i * dim;
    const float *b = W + (int64_t)rep * dim;
    int differ = 0;
    for (int c = lane; c < dim; c += kWave) differ |= (__float_as_uint(a[c]) != __float_as_uint(b[c]));
    if (!__any(differ) && lane == 0) node_const[i] = INFINITY;
  }
}

hipError_t launch_mask_duplicate_rows(som_ctx *c, const float *W) {
  const int waves_grid = (c->k + 3) / 4 < c->n_cu * 8 ? (c->k + 3) / 4 : c->n_cu * 8;
  const int slots = c->dedup_slots;
  unsigned long long *keys = reinterpret_cast<unsigned long long *>(c->dedup_keys);
  hipLaunchKernelGGL(k_dedup_clear, dim3((slots + 255) / 256), dim3(256), 0, c->stream, keys, c->dedup_lowest, slots);
  hipLaunchKernelGGL(k_row_hash, dim3(waves_grid), dim3(256), 0, c->stream, W, c->k, c->dim, c->row_hash);
  hipLaunchKernelGGL(k_dedup_insert, dim3((c->k + 255) / 256), dim3(256), 0, c->stream, c->row_hash, c->k, keys,
                     c->dedup_lowest, slots);
  hipLaunchKernelGGL(k_dedup_mark, dim3(waves_grid), dim3(256), 0, c->stream, W, c->k, c->dim, c->row_hash, keys,
                     c->dedup_lowest, slots, c->wn32);
  return hipGetLastError();
}

}  // namespace som
