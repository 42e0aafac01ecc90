// Per-node sums of the batch update (paper: batch equation; "Parallelism": the accumulation of
// local weights used to be the bottleneck when done by one process).
//
// The neighbourhood weight of an instance depends on it only through its BMU, so the update
// needs S_b = sum of the instances whose BMU is b and C_b = their number.  Dense data:
//   1. stable LSD radix sort of the instance ids by BMU (8-bit digits, ballot-based ranking),
//      so every segment lists its instances in ascending order;
//   2. segment offsets by binary search in the sorted keys, C_b = their differences;
//   3. every segment is cut into chunks of kChunkRows instances; one workgroup sums one chunk
//      (fp64 registers, instances read as whole rows through the permutation);
//   4. chunks of a node are added in order.
// No floating-point atomics: the result is bit-reproducible.  Sparse data uses the same sort and
// chunking, with a column tile in LDS per chunk and atomic adds (k_accumulate_csr below): the order of
// the additions is not fixed there, so two sparse runs agree to rounding only.
#include "som_internal.hpp"

namespace som {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int clamp_node(int b, int k) { return b < 0 ? 0 : (b >= k ? k - 1 : b); }

// Segment offsets of the sorted keys: seg_off[b] = first position whose key is >= b.
__global__ __launch_bounds__(256) void k_segment_bounds(const int32_t *__restrict__ sorted_keys, int64_t n, int k,
                                                        int32_t *__restrict__ seg_off,
                                                        int32_t *__restrict__ counts) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= k) return;
  int bound[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if (sorted_keys[mid] < b + e) lo = mid + 1; else hi = mid;
    }
    bound[e] = (int)lo;
  }
  seg_off[b] = bound[0];
  counts[b] = bound[1] - bound[0];
  if (b == k - 1) seg_off[k] = (int32_t)n;
}

// Exclusive scan of in[0..len) into out[0..len], out[len] = total.  One workgroup of 1024 walks the
// array in steps of 4096: a thread takes four consecutive elements (one 16-byte access when the
// arrays allow it), the wavefronts scan the thread sums with shuffles and the sixteen wavefront
// totals are combined through LDS.
// `transform` > 0: scan ceil(in / transform) instead of in (chunks per node).
// in and out may be the same array (a thread reads its elements before it writes them).
__global__ __launch_bounds__(1024) void k_scan_exclusive(const int32_t *in, int32_t *out, int len, int transform) {
  __shared__ int s_wave[2][16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool vec = (len & 3) == 0 && (((uintptr_t)in | (uintptr_t)out) & 15) == 0;
  int carry = 0;
  int phase = 0;
  for (int base = 0; base < len; base += 4096, phase ^= 1) {
    const int i = base + 4 * tid;
    int v[4] = {0, 0, 0, 0};
    if (vec) {
      if (i < len) {
        const int4 q = *reinterpret_cast<const int4 *>(in + i);
        v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (i + e < len) v[e] = in[i + e];
    }
    if (transform > 0) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (v[e] + transform - 1) / transform;
    }
    const int sum = (v[0] + v[1]) + (v[2] + v[3]);
    int inc = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    if (lane == 63) s_wave[phase][wave] = inc;
    __syncthreads();                       // one barrier per step: the totals alternate between two rows
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      const int t = s_wave[phase][w];
      before += w < wave ? t : 0;
      all += t;
    }
    int run = carry + before + inc - sum;
    if (vec) {
      if (i < len) {
        int4 q;
        q.x = run; q.y = run + v[0]; q.z = q.y + v[1]; q.w = q.z + v[2];
        *reinterpret_cast<int4 *>(out + i) = q;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (i + e < len) out[i + e] = run;
        run += v[e];
      }
    }
    carry += all;
  }
  if (tid == 0) out[len] = carry;
}

// ---------------------------------------------------------------- stable radix sort
// Digits of `bits` bits (at most 8) at `shift`; hist[digit][tile].
__global__ __launch_bounds__(256) void k_radix_hist(const int32_t *__restrict__ keys, int64_t n, int shift, int bits,
                                                    int nblk, int tile, int k, int32_t *__restrict__ hist) {
  __shared__ int s_hist[256];
  const int mask = (1 << bits) - 1;
  s_hist[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * tile;
  for (int e = threadIdx.x; e < tile; e += 256) {
    const int64_t j = base + e;
    if (j < n) atomicAdd(&s_hist[(clamp_node(keys[j], k) >> shift) & mask], 1);
  }
  __syncthreads();
  if ((int)threadIdx.x <= mask) hist[(int64_t)threadIdx.x * nblk + blockIdx.x] = s_hist[threadIdx.x];
}

// One wavefront ranks its tile 64 keys at a time, in order: a key's position is the running
// count of its digit plus the number of lower lanes holding the same digit (a ballot per digit bit).
__global__ __launch_bounds__(64) void k_radix_scatter(const int32_t *__restrict__ keys_in,
                                                      const int32_t *__restrict__ vals_in,
                                                      int32_t *__restrict__ keys_out,
                                                      int32_t *__restrict__ vals_out, int64_t n, int shift, int bits,
                                                      int nblk, int tile, int k,
                                                      const int32_t *__restrict__ hist_scanned) {
  __shared__ int s_cnt[256];
  const int lane = threadIdx.x;
  const int mask = (1 << bits) - 1;
  for (int d = lane; d <= mask; d += 64) s_cnt[d] = hist_scanned[(int64_t)d * nblk + blockIdx.x];
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * tile;
  for (int step = 0; step < tile / 64; ++step) {
    const int64_t j = base + step * 64 + lane;
    const bool valid = j < n;
    const int key = valid ? clamp_node(keys_in[j], k) : 0;
    const int val = valid ? (vals_in ? vals_in[j] : (int32_t)j) : 0;
    const int d = (key >> shift) & mask;
    unsigned long long same = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      if (b < bits) {                              // uniform
        const bool bit = (d >> b) & 1;
        const unsigned long long bal = __ballot(bit);
        same &= bit ? bal : ~bal;
      }
    }
    const int rank = __popcll(same & ((1ull << lane) - 1ull));
    const int before = valid ? s_cnt[d] : 0;
    __syncthreads();
    if (valid && rank == 0) s_cnt[d] = before + __popcll(same);
    __syncthreads();
    if (valid) {
      keys_out[before + rank] = key;
      vals_out[before + rank] = val;
    }
  }
}

// ---------------------------------------------------------------- chunks
__global__ __launch_bounds__(256) void k_fill_chunk_nodes(const int32_t *__restrict__ chunk_off, int k,
                                                          int32_t *__restrict__ chunk_node) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * 4;
  for (int b = wave; b < k; b += nwaves)
    for (int t = chunk_off[b] + lane; t < chunk_off[b + 1]; t += 64) chunk_node[t] = b;
}

template <bool kVec4>
__global__ __launch_bounds__(256) void k_accumulate_dense(const float *__restrict__ X, int dim,
                                                          const int32_t *__restrict__ perm,
                                                          const int32_t *__restrict__ seg_off,
                                                          const int32_t *__restrict__ chunk_off,
                                                          const int32_t *__restrict__ chunk_node, int k,
                                                          float *__restrict__ S, float *__restrict__ partial) {
  __shared__ int s_rows[kChunkRows];
  const int chunk = blockIdx.x;
  if (chunk >= chunk_off[k]) return;
  const int b = chunk_node[chunk];
  const int first_chunk = chunk_off[b];
  const int lo = seg_off[b] + (chunk - first_chunk) * kChunkRows;
  const int hi = min(lo + kChunkRows, seg_off[b + 1]);
  const int nrows = hi - lo;
  if (threadIdx.x < nrows) s_rows[threadIdx.x] = perm[lo + threadIdx.x];
  __syncthreads();
  const bool single = (chunk_off[b + 1] - first_chunk) == 1;
  float *dst = single ? S + (int64_t)b * dim : partial + (int64_t)chunk * dim;
  if (kVec4) {
    for (int q = threadIdx.x; q < dim / 4; q += blockDim.x) {
      double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
      for (int r = 0; r < nrows; ++r) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(X + (int64_t)s_rows[r] * dim + 4 * q);
        a0 += (double)v[0]; a1 += (double)v[1]; a2 += (double)v[2]; a3 += (double)v[3];
      }
      f32x4 o = {(float)a0, (float)a1, (float)a2, (float)a3};
      *reinterpret_cast<f32x4 *>(dst + 4 * q) = o;
    }
  } else {
    for (int c = threadIdx.x; c < dim; c += blockDim.x) {
      double a = 0;
      for (int r = 0; r < nrows; ++r) a += (double)X[(int64_t)s_rows[r] * dim + c];
      dst[c] = (float)a;
    }
  }
}

// Nodes with many chunks (early in training a few nodes hold most of the instances, thousands of chunks
// each; one workgroup adding them one after the other took three times as long as computing them): every
// group of kCombineGroup consecutive chunks of such a node is first added up, in place, into the group's
// first chunk.  One workgroup per chunk slot; only the group leaders of large nodes do anything.
constexpr int kCombineGroup = 32;

__global__ __launch_bounds__(256) void k_combine_groups(const int32_t *__restrict__ chunk_off,
                                                        const int32_t *__restrict__ chunk_node, int k, int dim,
                                                        float *__restrict__ partial) {
  const int chunk = blockIdx.x;
  if (chunk >= chunk_off[k]) return;
  const int b = chunk_node[chunk];
  const int c0 = chunk_off[b], nc = chunk_off[b + 1] - c0;
  const int at = chunk - c0;
  if (nc <= kCombineGroup || at % kCombineGroup != 0) return;
  const int len = min(kCombineGroup, nc - at);
  float *dst = partial + (int64_t)chunk * dim;
  for (int c = blockIdx.y * blockDim.x + threadIdx.x; c < dim; c += gridDim.y * blockDim.x) {
    double a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int t = 0;
    for (; t + 8 <= len; t += 8)
#pragma unroll
      for (int u = 0; u < 8; ++u) a[u] += (double)dst[(int64_t)(t + u) * dim + c];
    for (int u = 0; t < len; ++t, ++u) a[u] += (double)dst[(int64_t)t * dim + c];
    dst[c] = (float)(((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7])));
  }
}

// Empty node: zero row.  One chunk: already written.  Several: add the partial rows (of a node with more
// than kCombineGroup chunks: the group sums k_combine_groups left in every kCombineGroup-th row), eight
// interleaved running sums (term t goes to sum t mod 8) combined pairwise at the end: a fixed order, with
// eight loads in flight instead of one.
__global__ __launch_bounds__(256) void k_combine_chunks(const int32_t *__restrict__ chunk_off, int dim,
                                                        const float *__restrict__ partial, float *__restrict__ S) {
  const int b = blockIdx.x;
  const int c0 = chunk_off[b], nc = chunk_off[b + 1] - c0;
  if (nc == 1) return;
  float *dst = S + (int64_t)b * dim;
  const bool grouped = nc > kCombineGroup;
  const int terms = grouped ? (nc + kCombineGroup - 1) / kCombineGroup : nc;
  const int64_t step = (int64_t)(grouped ? kCombineGroup : 1) * dim;
  const float *src = partial + (int64_t)c0 * dim;
  // grid.y splits the columns: late in training a few dozen nodes hold all the chunks
  for (int c = blockIdx.y * blockDim.x + threadIdx.x; c < dim; c += gridDim.y * blockDim.x) {
    double a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    int t = 0;
    for (; t + 8 <= terms; t += 8)
#pragma unroll
      for (int u = 0; u < 8; ++u) a[u] += (double)src[(t + u) * step + c];
    for (int u = 0; t < terms; ++t, ++u) a[u] += (double)src[t * step + c];
    dst[c] = (float)(((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7])));
  }
}

// ---------------------------------------------------------------- sparse rows
// S_b for CSR data.
//
// Rows of up to kCsrTile columns: the instances are sorted by BMU as in the dense path and cut into
// chunks of kCsrChunkRows; a workgroup adds the nonzeros of its chunk into a copy of the node's row
// in LDS (LDS atomics: the rows of a node share their frequent columns).  A node with a single chunk
// is then written with plain stores, zeros included, so its row needs no clearing beforehand; the
// chunks of a larger node add their nonzero entries to a row cleared by k_zero_rows_if.
//
// Longer rows: every chosen row is cleared and every nonzero goes straight into S with a global
// atomic, in instance order.  Measured alternatives on configuration 4 (rows of 50,000 columns, 1e7
// nonzeros, 0.64 ms + 0.1 ms of clearing this way): the sorted chunks with one LDS tile of columns
// after the other 0.71 ms (walking a chunk is a chain of dependent loads - permutation, row pointer,
// entries - and is repeated per tile); the sorted chunks with global atomics 0.79 ms (the sort costs
// what the locality gains).  On configuration 6 (rows of 1,000 columns, 5e6 nonzeros colliding on
// 10 MB) the LDS copy took the stage from 0.51 to 0.14 ms.
constexpr int kCsrChunkRows = 256;
constexpr int kCsrTile = 16384;           // columns of a row copy in LDS (64 KB: two workgroups per CU)
static_assert(kCsrChunkRows % kChunkRows == 0, "the chunk tables are sized for kChunkRows");

// Clears the rows of S whose node has more than `lo` instances.
__global__ __launch_bounds__(256) void k_zero_rows_if(const int32_t *__restrict__ counts, int lo, int dim,
                                                      float *__restrict__ S) {
  const int b = blockIdx.x;
  if (counts[b] <= lo) return;
  float *dst = S + (int64_t)b * dim;
  for (int c = blockIdx.y * 256 + threadIdx.x; c < dim; c += gridDim.y * 256) dst[c] = 0.f;
}

__global__ __launch_bounds__(256) void k_accumulate_csr(const int64_t *__restrict__ indptr,
                                                        const int32_t *__restrict__ indices,
                                                        const float *__restrict__ values, int dim,
                                                        const int32_t *__restrict__ perm,
                                                        const int32_t *__restrict__ seg_off,
                                                        const int32_t *__restrict__ chunk_off,
                                                        const int32_t *__restrict__ chunk_node, int k,
                                                        float *__restrict__ S) {
  extern __shared__ float s_row[];           // dim floats
  const int chunk = blockIdx.x;
  if (chunk >= chunk_off[k]) return;          // uniform over the workgroup
  const int b = chunk_node[chunk];
  const int first_chunk = chunk_off[b];
  const int lo = seg_off[b] + (chunk - first_chunk) * kCsrChunkRows;
  const int hi = min(lo + kCsrChunkRows, seg_off[b + 1]);
  const bool single = (chunk_off[b + 1] - first_chunk) == 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *dst = S + (int64_t)b * dim;
  for (int c = threadIdx.x; c < dim; c += 256) s_row[c] = 0.f;
  __syncthreads();
  for (int r = lo + wave; r < hi; r += 4) {
    const int64_t j = perm[r];
    for (int64_t p = indptr[j] + lane; p < indptr[j + 1]; p += 64) {
      int c = indices[p];
      c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
      atomicAdd(&s_row[c], values[p]);
    }
  }
  __syncthreads();
  if (single) {
    for (int c = threadIdx.x; c < dim; c += 256) dst[c] = s_row[c];
  } else {
    for (int c = threadIdx.x; c < dim; c += 256) {
      const float v = s_row[c];
      if (v != 0.f) unsafeAtomicAdd(dst + c, v);
    }
  }
}

// Long rows of a context that holds a split into frequent columns and the rest (csr_hot.hip; the tables
// describe the registered set, but any table gives correct sums): the instances are sorted by BMU and cut
// into chunks as above, the nonzeros of the kHot frequent columns - about half of all, and the ones whose
// atomics collide - are added up in LDS per chunk and leave as at most kHot atomics, the others go straight
// into S.  The rows of the chosen nodes are cleared beforehand.
__global__ __launch_bounds__(256) void k_accumulate_csr_hot(const int64_t *__restrict__ indptr,
                                                            const int32_t *__restrict__ indices,
                                                            const float *__restrict__ values, int dim,
                                                            const int32_t *__restrict__ perm,
                                                            const int32_t *__restrict__ seg_off,
                                                            const int32_t *__restrict__ chunk_off,
                                                            const int32_t *__restrict__ chunk_node, int k,
                                                            const int32_t *__restrict__ rank,
                                                            const int32_t *__restrict__ hot_cols,
                                                            float *__restrict__ S) {
  __shared__ float s_hot[kHot];
  const int chunk = blockIdx.x;
  if (chunk >= chunk_off[k]) return;          // uniform over the workgroup
  const int b = chunk_node[chunk];
  const int first_chunk = chunk_off[b];
  const int lo = seg_off[b] + (chunk - first_chunk) * kCsrChunkRows;
  const int hi = min(lo + kCsrChunkRows, seg_off[b + 1]);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float *dst = S + (int64_t)b * dim;
  for (int h = threadIdx.x; h < kHot; h += 256) s_hot[h] = 0.f;
  __syncthreads();
  for (int r = lo + wave; r < hi; r += 4) {
    const int64_t j = perm[r];
    for (int64_t p = indptr[j] + lane; p < indptr[j + 1]; p += 64) {
      int c = indices[p];
      c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
      const int h = rank[c];
      if (h >= 0) atomicAdd(&s_hot[h], values[p]);
      else unsafeAtomicAdd(dst + c, values[p]);
    }
  }
  __syncthreads();
  for (int h = threadIdx.x; h < kHot; h += 256) {
    const float v = s_hot[h];
    if (v != 0.f) unsafeAtomicAdd(dst + hot_cols[h], v);
  }
}

// C_b for the sparse path.  Trained maps send most instances to few nodes, so the lanes of a
// wavefront that hold the same node are merged into one atomic add.
__global__ __launch_bounds__(256) void k_count_bmus(const int32_t *__restrict__ bmus, int64_t n, int k,
                                                    int32_t *__restrict__ counts) {
  const int lane = threadIdx.x & 63;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const int64_t rounds = (n + stride - 1) / stride;
  for (int64_t r = 0; r < rounds; ++r) {
    const int64_t j = r * stride + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool pending = j < n;
    const int b = pending ? clamp_node(bmus[j], k) : 0;
    unsigned long long todo = __ballot(pending);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int lb = __shfl(b, leader, 64);
      const unsigned long long same = __ballot(pending && b == lb);
      if (lane == leader) atomicAdd(&counts[lb], __popcll(same));
      if (pending && b == lb) pending = false;
      todo &= ~same;
    }
  }
}

__global__ __launch_bounds__(256) void k_scatter_csr(const int64_t *__restrict__ indptr,
                                                     const int32_t *__restrict__ indices,
                                                     const float *__restrict__ values, int64_t n, int dim, int k,
                                                     const int32_t *__restrict__ bmus, float *__restrict__ S) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * 4;
  for (int64_t j = wave; j < n; j += nwaves) {
    float *dst = S + (int64_t)clamp_node(bmus[j], k) * dim;
    for (int64_t p = indptr[j] + lane; p < indptr[j + 1]; p += 64) {
      int c = indices[p];
      c = c < 0 ? 0 : (c >= dim ? dim - 1 : c);
      unsafeAtomicAdd(dst + c, values[p]);
    }
  }
}

// Stable permutation of the ids 0 .. n - 1 by integer keys in [0, key_range) (larger keys are clamped).
// On return c->sort_val[0] holds the permutation, c->sort_key[0] the sorted keys.
hipError_t launch_sort_keys(som_ctx *c, const int32_t *bmus, int64_t n, int key_range) {
  const RadixPlan plan = radix_plan(n, key_range);
  const int bins = 1 << plan.digit_bits;
  const int32_t *kin = bmus;
  const int32_t *vin = nullptr;
  // an even number of hops ends in buffer 0: start in buffer 1 when the pass count is even
  int dst = (plan.passes % 2 == 0) ? 1 : 0;
  for (int p = 0; p < plan.passes; ++p) {
    hipLaunchKernelGGL(k_radix_hist, dim3(plan.nblk), dim3(256), 0, c->stream, kin, n, plan.digit_bits * p,
                       plan.digit_bits, plan.nblk, plan.tile, key_range, c->radix_hist);
    hipLaunchKernelGGL(k_scan_exclusive, dim3(1), dim3(1024), 0, c->stream, c->radix_hist, c->radix_hist,
                       bins * plan.nblk, 0);
    hipLaunchKernelGGL(k_radix_scatter, dim3(plan.nblk), dim3(64), 0, c->stream, kin, vin, c->sort_key[dst],
                       c->sort_val[dst], n, plan.digit_bits * p, plan.digit_bits, plan.nblk, plan.tile, key_range,
                       c->radix_hist);
    kin = c->sort_key[dst];
    vin = c->sort_val[dst];
    dst ^= 1;
  }
  return hipGetLastError();
}

// Stable permutation of instance ids by BMU, segment offsets and counts.
// On return c->sort_val[0] holds the permutation (c->sort_key[0] the sorted BMUs).
hipError_t launch_sort_by_bmu(som_ctx *c, const int32_t *bmus, int64_t n) {
  hipError_t e = launch_sort_keys(c, bmus, n, c->k);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_segment_bounds, dim3((c->k + 255) / 256), dim3(256), 0, c->stream, c->sort_key[0], n, c->k,
                     c->seg_off, c->counts);
  return hipGetLastError();
}

hipError_t launch_scan_exclusive_i32(som_ctx *c, const int32_t *in, int32_t *out, int len) {
  hipLaunchKernelGGL(k_scan_exclusive, dim3(1), dim3(1024), 0, c->stream, in, out, len, 0);
  return hipGetLastError();
}

hipError_t launch_accumulate_dense(som_ctx *c, const float *X, int64_t n) {
  hipLaunchKernelGGL(k_scan_exclusive, dim3(1), dim3(1024), 0, c->stream, c->counts, c->chunk_off, c->k,
                     kChunkRows);
  hipLaunchKernelGGL(k_fill_chunk_nodes, dim3(c->n_cu * 2), dim3(256), 0, c->stream, c->chunk_off, c->k,
                     c->chunk_node);
  int64_t max_chunks = n / kChunkRows + (n < c->k ? n : c->k);
  if (max_chunks < 1) max_chunks = 1;
  const bool vec4 = (c->dim % 4 == 0) && ((uintptr_t)X % 16 == 0);
  int threads = vec4 ? c->dim / 4 : c->dim;
  threads = ((threads + 63) / 64) * 64;
  if (threads > 256) threads = 256;
  if (threads < 64) threads = 64;
  if (vec4)
    hipLaunchKernelGGL(k_accumulate_dense<true>, dim3((unsigned)max_chunks), dim3(threads), 0, c->stream, X,
                       c->dim, c->sort_val[0], c->seg_off, c->chunk_off, c->chunk_node, c->k, c->S, c->partial);
  else
    hipLaunchKernelGGL(k_accumulate_dense<false>, dim3((unsigned)max_chunks), dim3(threads), 0, c->stream, X,
                       c->dim, c->sort_val[0], c->seg_off, c->chunk_off, c->chunk_node, c->k, c->S, c->partial);
  int ysplit = (c->dim + 255) / 256;
  if (ysplit > 16) ysplit = 16;
  const int cthreads = c->dim >= 256 ? 256 : (c->dim + 63) / 64 * 64;
  if (max_chunks > kCombineGroup)
    hipLaunchKernelGGL(k_combine_groups, dim3((unsigned)max_chunks, ysplit), dim3(cthreads), 0, c->stream, c->chunk_off,
                       c->chunk_node, c->k, c->dim, c->partial);
  hipLaunchKernelGGL(k_combine_chunks, dim3(c->k, ysplit), dim3(256), 0, c->stream, c->chunk_off, c->dim, c->partial,
                     c->S);
  return hipGetLastError();
}

hipError_t launch_accumulate_csr(som_ctx *c, const int64_t *indptr, const int32_t *indices,
                                 const float *values, int64_t n, const int32_t *bmus) {
  int ysplit = (c->dim + 4095) / 4096;
  if (ysplit > 64) ysplit = 64;
  if (c->dim <= kCsrTile) {
    hipError_t e = launch_sort_by_bmu(c, bmus, n);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_scan_exclusive, dim3(1), dim3(1024), 0, c->stream, c->counts, c->chunk_off, c->k,
                       kCsrChunkRows);
    hipLaunchKernelGGL(k_fill_chunk_nodes, dim3(c->n_cu * 2), dim3(256), 0, c->stream, c->chunk_off, c->k,
                       c->chunk_node);
    if (c->GxT) {          // matrix smoothing only reads the rows of chosen nodes
      hipLaunchKernelGGL(k_zero_rows_if, dim3(c->k, ysplit), dim3(256), 0, c->stream, c->counts, kCsrChunkRows, c->dim,
                         c->S);
    } else {               // the stencil smoothing reads every row: those of nodes nobody chose must be zero
      e = launch_fill_zero_u32(c->stream, c->S, (int64_t)c->k * c->dim);
      if (e != hipSuccess) return e;
    }
    int64_t max_chunks = n / kCsrChunkRows + (n < c->k ? n : c->k);
    if (max_chunks < 1) max_chunks = 1;
    hipLaunchKernelGGL(k_accumulate_csr, dim3((unsigned)max_chunks), dim3(256), (size_t)c->dim * sizeof(float),
                       c->stream, indptr, indices, values, c->dim, c->sort_val[0], c->seg_off, c->chunk_off,
                       c->chunk_node, c->k, c->S);
    return hipGetLastError();
  }
  // (worth the sort only with several instances per node: with 12,347 instances on 68,880 nodes it cost 0.09 ms
  // more than the plain scatter, with 100,000 on 2,500 it saves 0.14)
  if (c->hot_valid && c->hot_on && n >= 8 * (int64_t)c->k) {
    hipError_t e = launch_sort_by_bmu(c, bmus, n);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_scan_exclusive, dim3(1), dim3(1024), 0, c->stream, c->counts, c->chunk_off, c->k,
                       kCsrChunkRows);
    hipLaunchKernelGGL(k_fill_chunk_nodes, dim3(c->n_cu * 2), dim3(256), 0, c->stream, c->chunk_off, c->k,
                       c->chunk_node);
    if (c->GxT) {
      hipLaunchKernelGGL(k_zero_rows_if, dim3(c->k, ysplit), dim3(256), 0, c->stream, c->counts, 0, c->dim, c->S);
    } else {
      e = launch_fill_zero_u32(c->stream, c->S, (int64_t)c->k * c->dim);
      if (e != hipSuccess) return e;
    }
    int64_t max_chunks = n / kCsrChunkRows + (n < c->k ? n : c->k);
    if (max_chunks < 1) max_chunks = 1;
    hipLaunchKernelGGL(k_accumulate_csr_hot, dim3((unsigned)max_chunks), dim3(256), 0, c->stream, indptr, indices,
                       values, c->dim, c->sort_val[0], c->seg_off, c->chunk_off, c->chunk_node, c->k, c->hot_rank,
                       c->hot_cols, c->S);
    return hipGetLastError();
  }
  hipError_t e = launch_fill_zero_u32(c->stream, c->counts, c->k);
  if (e != hipSuccess) return e;
  int64_t cb = (n + 255) / 256;
  if (cb > (int64_t)c->n_cu * 16) cb = (int64_t)c->n_cu * 16;
  hipLaunchKernelGGL(k_count_bmus, dim3((unsigned)cb), dim3(256), 0, c->stream, bmus, n, c->k, c->counts);
  if (c->GxT) {
    hipLaunchKernelGGL(k_zero_rows_if, dim3(c->k, ysplit), dim3(256), 0, c->stream, c->counts, 0, c->dim, c->S);
  } else {
    e = launch_fill_zero_u32(c->stream, c->S, (int64_t)c->k * c->dim);
    if (e != hipSuccess) return e;
  }
  int64_t sb = (n + 3) / 4;
  if (sb > (int64_t)c->n_cu * 32) sb = (int64_t)c->n_cu * 32;
  hipLaunchKernelGGL(k_scatter_csr, dim3((unsigned)sb), dim3(256), 0, c->stream, indptr, indices, values, n,
                     c->dim, c->k, bmus, c->S);
  return hipGetLastError();
}

}  // namespace som
