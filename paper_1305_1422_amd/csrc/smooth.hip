// Cooling schedules and the neighbourhood part of the batch update (paper: neighbourhood
// equation, batch equation, options -t/-T, -r/-R, -l/-L, -g, -m; "Parallelism": the influence
// radius of a best matching node is thresholded).
//
// New weights: w_i = N_i / D_i with N_i = sum_b h(b,i) S_b and D_i = sum_b h(b,i) C_b, where
// h(b,i) = exp(-d^2(b,i) / (2 r^2)) and S_b, C_b are the per-node sums and counts.
//
// With q = 4 d^2 = m^2 + 4 a^2 (square) or m^2 + 3 a^2 (hexagonal), a = row distance and
// m = twice the embedded column distance, the Gaussian factors: h = gx[m] * gy[a].  For a
// hexagonal grid m depends on the column offset and on the row parities of both nodes only.
// The sum over the k source nodes is therefore two one-dimensional passes over the map
// (a (dim+1)-channel image of S and C):
//   pass x: T_p[yb][xi] = sum_xb gx[m(xi, xb, p, parity(yb))] S[yb][xb]     (p = parity of the
//           destination row; one image for square grids, two for hexagonal ones)
//   pass y: N[yi][xi]   = sum_yb gy[a(yi, yb)] T_parity(yi)[yb][xi],  then w = N / D or keep.
// Cost 2 k (rows + cols) dim instead of 2 k^2 dim flops.  The count channel is done the same
// way in fp64 by two small kernels.  A node with D < SOM_EPS_MASS keeps its weights.
//
// Cooling and the two factor tables are evaluated by a one-workgroup kernel, so a whole
// training schedule can be enqueued without the host computing anything per epoch.
#include "som_internal.hpp"

#include <math.h>

namespace som {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ double cooled(double v0, double vN, int n_epochs, int epoch, int kind) {
  if (n_epochs <= 1) return v0;
  const double t = (double)epoch / (double)(n_epochs - 1);
  return kind == SOM_COOL_EXPONENTIAL ? v0 * pow(vN / v0, t) : v0 + (vN - v0) * t;
}

__global__ __launch_bounds__(256) void k_epoch_params(EpochParams *__restrict__ params, float *__restrict__ gx,
                                                      float *__restrict__ gy, int rows, int cols, int hex,
                                                      int epoch, int n_epochs, double r0, double rN, double s0,
                                                      double sN, int cooling, int scale_cooling) {
  const double radius = cooled(r0, rN, n_epochs, epoch, cooling);
  const double inv = 1.0 / (8.0 * radius * radius);
  if (threadIdx.x == 0) {
    params->radius = radius;
    params->scale = cooled(s0, sN, n_epochs, epoch, scale_cooling);
    params->inv8r2 = inv;
  }
  for (int m = threadIdx.x; m <= 2 * cols; m += blockDim.x) gx[m] = (float)exp(-(double)m * (double)m * inv);
  const double ya = hex ? 3.0 : 4.0;
  for (int a = threadIdx.x; a < rows; a += blockDim.x) gy[a] = (float)exp(-ya * (double)a * (double)a * inv);
}

__global__ __launch_bounds__(256) void k_cool_schedule(int n_epochs, double r0, double rN, double s0, double sN,
                                                       int cooling, int scale_cooling,
                                                       double *__restrict__ radius_out,
                                                       double *__restrict__ scale_out) {
  for (int e = blockIdx.x * blockDim.x + threadIdx.x; e < n_epochs; e += gridDim.x * blockDim.x) {
    if (radius_out) radius_out[e] = cooled(r0, rN, n_epochs, e, cooling);
    if (scale_out) scale_out[e] = cooled(s0, sN, n_epochs, e, scale_cooling);
  }
}

// twice the embedded column distance between destination column xi (row parity pi) and source
// column xb (row parity pb)
__device__ __forceinline__ int col_offset2(int xi, int xb, int pi, int pb, int hex, int toroid, int cols) {
  int m = 2 * (xi - xb) + (hex ? pi - pb : 0);
  m = m < 0 ? -m : m;
  if (toroid && 2 * cols - m < m) m = 2 * cols - m;
  return m;
}

__device__ __forceinline__ int row_offset(int yi, int yb, int toroid, int rows) {
  int a = yi > yb ? yi - yb : yb - yi;
  if (toroid && rows - a < a) a = rows - a;
  return a;
}

// ---------------------------------------------------------------- count channel (fp64)
__global__ __launch_bounds__(256) void k_count_pass_x(const int32_t *__restrict__ counts,
                                                      const float *__restrict__ gx, int rows, int cols, int hex,
                                                      int toroid, double *__restrict__ cntT) {
  const int k = rows * cols;
  const int images = hex ? 2 : 1;
  for (int o = blockIdx.x * blockDim.x + threadIdx.x; o < images * k; o += gridDim.x * blockDim.x) {
    const int p = o / k, i = o - p * k;
    const int y = i / cols, xi = i - y * cols;
    double s = 0.0;
    for (int xb = 0; xb < cols; ++xb) {
      const int cb = counts[y * cols + xb];
      if (cb) s += (double)gx[col_offset2(xi, xb, p, y & 1, hex, toroid, cols)] * (double)cb;
    }
    cntT[o] = s;
  }
}

__global__ __launch_bounds__(256) void k_count_pass_y(const double *__restrict__ cntT,
                                                      const float *__restrict__ gy, int rows, int cols, int hex,
                                                      int toroid, double *__restrict__ massD) {
  const int k = rows * cols;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < k; i += gridDim.x * blockDim.x) {
    const int yi = i / cols, x = i - yi * cols;
    const double *img = cntT + (hex ? (int64_t)(yi & 1) * k : 0);
    // four running sums: the loads of four source rows are in flight together (a single chain of
    // dependent fp64 additions made this small kernel latency-bound)
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int yb = 0;
    for (; yb + 4 <= rows; yb += 4) {
      s0 += (double)gy[row_offset(yi, yb, toroid, rows)] * img[yb * cols + x];
      s1 += (double)gy[row_offset(yi, yb + 1, toroid, rows)] * img[(yb + 1) * cols + x];
      s2 += (double)gy[row_offset(yi, yb + 2, toroid, rows)] * img[(yb + 2) * cols + x];
      s3 += (double)gy[row_offset(yi, yb + 3, toroid, rows)] * img[(yb + 3) * cols + x];
    }
    for (; yb < rows; ++yb) s0 += (double)gy[row_offset(yi, yb, toroid, rows)] * img[yb * cols + x];
    massD[i] = (s0 + s1) + (s2 + s3);
  }
}

// ---------------------------------------------------------------- feature channels (fp32)
constexpr int kSmoothCols = 64;    // feature columns per workgroup (one per lane)
constexpr int kSmoothOut = 4;      // outputs per thread along the smoothed direction

// pass x.  grid = (ceil(dim/64), rows, images); wavefront w of the workgroup produces the
// destination columns xi = 4 (w + 4 t) .. + 3.
template <bool kHex>
__global__ __launch_bounds__(256) void k_smooth_x(const float *__restrict__ S, float *__restrict__ T,
                                                  const float *__restrict__ gx, int rows, int cols, int dim,
                                                  int toroid) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.x * kSmoothCols + lane;
  const int y = blockIdx.y;
  const int p = blockIdx.z;                    // parity of the destination rows this image serves
  const bool live = c < dim;
  const float *src = S + (int64_t)y * cols * dim + (live ? c : 0);
  float *dst = T + ((int64_t)p * rows + y) * (int64_t)cols * dim + c;
  for (int x0 = wave * kSmoothOut; x0 < cols; x0 += 4 * kSmoothOut) {
    float acc[kSmoothOut] = {0.f, 0.f, 0.f, 0.f};
    for (int xb = 0; xb < cols; ++xb) {
      const float s = live ? src[(int64_t)xb * dim] : 0.f;
#pragma unroll
      for (int e = 0; e < kSmoothOut; ++e)
        acc[e] = fmaf(gx[col_offset2(x0 + e < cols ? x0 + e : cols - 1, xb, p, y & 1, kHex, toroid, cols)], s,
                      acc[e]);
    }
    if (live)
#pragma unroll
      for (int e = 0; e < kSmoothOut; ++e)
        if (x0 + e < cols) dst[(int64_t)(x0 + e) * dim] = acc[e];
  }
}

// pass y with the division.  grid = (ceil(dim/64), cols).
template <bool kHex>
__global__ __launch_bounds__(256) void k_smooth_y_divide(const float *__restrict__ T, float *__restrict__ W,
                                                         const float *__restrict__ gy,
                                                         const double *__restrict__ massD, int rows, int cols,
                                                         int dim, int toroid) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.x * kSmoothCols + lane;
  const int x = blockIdx.y;
  const bool live = c < dim;
  const int64_t img = (int64_t)rows * cols * dim;
  const float *src = T + (int64_t)x * dim + (live ? c : 0);
  for (int y0 = wave * kSmoothOut; y0 < rows; y0 += 4 * kSmoothOut) {
    float acc[kSmoothOut] = {0.f, 0.f, 0.f, 0.f};
    for (int yb = 0; yb < rows; ++yb) {
      const int64_t off = (int64_t)yb * cols * dim;
      const float t0 = live ? src[off] : 0.f;                                 // image for even rows
      const float t1 = kHex ? (live ? src[img + off] : 0.f) : t0;             // image for odd rows
#pragma unroll
      for (int e = 0; e < kSmoothOut; ++e) {
        const int yi = y0 + e;
        acc[e] = fmaf(gy[row_offset(yi < rows ? yi : rows - 1, yb, toroid, rows)], (kHex && (yi & 1)) ? t1 : t0,
                      acc[e]);
      }
    }
    if (live)
#pragma unroll
      for (int e = 0; e < kSmoothOut; ++e) {
        const int yi = y0 + e;
        if (yi < rows) {
          const int64_t i = (int64_t)yi * cols + x;
          const double D = massD[i];
          if (D >= SOM_EPS_MASS) W[i * dim + c] = acc[e] / (float)D;
        }
      }
  }
}

// The learning rate follows its own cooling kind if one was set (som_set_scale_cooling), else the radius' kind.
static int scale_cooling_of(const som_ctx *c, int cooling) { return c->scale_cooling >= 0 ? c->scale_cooling : cooling; }

hipError_t launch_epoch_params(som_ctx *c, int epoch, int n_epochs, double r0, double rN, double s0, double sN,
                               int cooling) {
  hipLaunchKernelGGL(k_epoch_params, dim3(1), dim3(256), 0, c->stream, c->params, c->gx, c->gy, c->rows, c->cols,
                     c->grid_type == SOM_GRID_HEXAGONAL, epoch, n_epochs, r0, rN, s0, sN, cooling,
                     scale_cooling_of(c, cooling));
  return hipGetLastError();
}

hipError_t launch_cool_schedule(som_ctx *c, int n_epochs, double r0, double rN, double s0, double sN,
                                int cooling, double *radius_out, double *scale_out) {
  hipLaunchKernelGGL(k_cool_schedule, dim3((n_epochs + 255) / 256), dim3(256), 0, c->stream, n_epochs, r0, rN, s0,
                     sN, cooling, scale_cooling_of(c, cooling), radius_out, scale_out);
  return hipGetLastError();
}

// ---------------------------------------------------------------- feature channels, coefficient matrices
// Faster variant for maps whose sides are at most kSmoothMatMax: the one-dimensional filters
// are first written out as dense coefficient matrices, transposed so that the 16 coefficients
// a wavefront needs for 16 neighbouring outputs and one source are contiguous (one scalar
// load).  A lane owns one feature column, keeps 16 outputs in registers and streams over the
// sources: 16 multiply-adds per loaded value, all operands but that value in scalar registers.
//   GxT[image][source parity][xb][xi]  (xi padded to a multiple of 16 with zeros)
//   GyT[class][yb][e], destination row yi = classes * e + class  (hex: classes = parities)
constexpr int kSmoothTile = 16;
constexpr int kSmoothUnroll = 8;    // source nodes whose loads are in flight together

__global__ __launch_bounds__(256) void k_smooth_tables(const float *__restrict__ gx, const float *__restrict__ gy,
                                                       int rows, int cols, int hex, int toroid, int xi_pad,
                                                       int e_pad, float *__restrict__ GxT, float *__restrict__ GyT) {
  const int par = hex ? 2 : 1;
  const int64_t nx = (int64_t)par * par * cols * xi_pad;
  const int64_t ny = (int64_t)par * rows * e_pad;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < nx + ny; o += stride) {
    if (o < nx) {
      const int xi = (int)(o % xi_pad);
      const int xb = (int)((o / xi_pad) % cols);
      const int ps = (int)((o / ((int64_t)xi_pad * cols)) % par);
      const int img = (int)(o / ((int64_t)xi_pad * cols * par));
      GxT[o] = xi < cols ? gx[col_offset2(xi, xb, img, ps, hex, toroid, cols)] : 0.f;
    } else {
      const int64_t q = o - nx;
      const int e = (int)(q % e_pad);
      const int yb = (int)((q / e_pad) % rows);
      const int cls = (int)(q / ((int64_t)e_pad * rows));
      const int yi = par * e + cls;
      GyT[q] = yi < rows ? gy[row_offset(yi, yb, toroid, rows)] : 0.f;
    }
  }
}

// Nodes that no instance chose contribute nothing to the sums.  Per map row the columns of the
// nodes with C > 0 are listed in ascending order (hit_x, hit_n), and the map rows that have any
// (hit_rows, hit_rows[rows] = their number), so that both passes only touch what counts and the
// rows of S that belong to empty nodes are never read.  One wavefront per map row.
__global__ __launch_bounds__(64) void k_hit_lists(const int32_t *__restrict__ counts, int rows, int cols,
                                                  int32_t *__restrict__ hit_x, int32_t *__restrict__ hit_n) {
  const int lane = threadIdx.x;
  for (int y = blockIdx.x; y < rows; y += gridDim.x) {
    int n = 0;
    for (int x0 = 0; x0 < cols; x0 += 64) {
      const int x = x0 + lane;
      const bool hit = x < cols && counts[y * cols + x] > 0;
      const unsigned long long m = __ballot(hit);
      if (hit) hit_x[y * cols + n + __popcll(m & ((1ull << lane) - 1ull))] = x;
      n += __popcll(m);
    }
    if (lane == 0) hit_n[y] = n;
  }
}

__global__ __launch_bounds__(64) void k_hit_rows(const int32_t *__restrict__ hit_n, int rows,
                                                 int32_t *__restrict__ hit_rows) {
  const int lane = threadIdx.x;
  int n = 0;
  for (int y0 = 0; y0 < rows; y0 += 64) {
    const int y = y0 + lane;
    const bool hit = y < rows && hit_n[y] > 0;
    const unsigned long long m = __ballot(hit);
    if (hit) hit_rows[n + __popcll(m & ((1ull << lane) - 1ull))] = y;
    n += __popcll(m);
  }
  if (lane == 0) hit_rows[rows] = n;
}

// Channel block and output tile of a workgroup.  Plain launch: channel block on grid.x, tile on
// grid.z.  Folded launch (grid.z == 1, used when there are at least 8 channel blocks): the tiles
// that read the same sources sit on workgroups 8 apart on grid.x, which the dispatcher hands to the
// same XCD one after the other, so that all but the first of their reads hit that XCD's L2.
__device__ __forceinline__ bool smooth_tile_of_block(int ntiles, int cblocks, int &cblk, int &tile) {
  if (gridDim.z > 1 || ntiles == 1) {
    cblk = blockIdx.x;
    tile = blockIdx.z;
    return true;
  }
  const int p = blockIdx.x & 7, r = blockIdx.x >> 3;
  tile = r % ntiles;
  cblk = (r / ntiles) * 8 + p;
  return cblk < cblocks;
}

// pass x.  grid = (ceil(dim/256), rows, images * ceil(cols/16)), or folded (see above).
template <bool kHex>
__global__ __launch_bounds__(256) void k_smooth_x_mat(const float *__restrict__ S, float *__restrict__ T,
                                                      const float *__restrict__ GxT,
                                                      const int32_t *__restrict__ hit_x,
                                                      const int32_t *__restrict__ hit_n, int rows, int cols, int dim,
                                                      int xi_pad) {
  const int y = blockIdx.y;
  const int nh = hit_n[y];
  if (nh == 0) return;               // pass y skips this map row
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ntile = (cols + kSmoothTile - 1) / kSmoothTile;
  int cblk, zt;
  if (!smooth_tile_of_block((kHex ? 2 : 1) * ntile, (dim + 255) / 256, cblk, zt)) return;
  const int c = cblk * 256 + wave * 64 + lane;
  const bool live = c < dim;
  const int img = zt / ntile;
  const int xi0 = (zt - img * ntile) * kSmoothTile;
  const int ps = kHex ? (y & 1) : 0;
  const float *G = GxT + ((int64_t)(img * (kHex ? 2 : 1) + ps) * cols) * xi_pad + xi0;
  const float *src = S + (int64_t)y * cols * dim + (live ? c : 0);
  const int32_t *hx = hit_x + (int64_t)y * cols;
  float acc[kSmoothTile];
#pragma unroll
  for (int e = 0; e < kSmoothTile; ++e) acc[e] = 0.f;
  for (int t = 0; t < nh; t += kSmoothUnroll) {
    int xb[kSmoothUnroll];
    float s[kSmoothUnroll];
#pragma unroll
    for (int u = 0; u < kSmoothUnroll; ++u) {
      xb[u] = hx[min(t + u, nh - 1)];
      s[u] = (live && t + u < nh) ? src[(int64_t)xb[u] * dim] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kSmoothUnroll; ++u) {
      const float *g = G + (int64_t)xb[u] * xi_pad;
#pragma unroll
      for (int e = 0; e < kSmoothTile; ++e) acc[e] = fmaf(g[e], s[u], acc[e]);
    }
  }
  if (live) {
    float *dst = T + ((int64_t)img * rows + y) * (int64_t)cols * dim + c;
#pragma unroll
    for (int e = 0; e < kSmoothTile; ++e)
      if (xi0 + e < cols) dst[(int64_t)(xi0 + e) * dim] = acc[e];
  }
}

// pass y with the division.  grid = (ceil(dim/256), cols, classes * ceil(E/16)), E = rows per class.
template <bool kHex>
__global__ __launch_bounds__(256) void k_smooth_y_mat(const float *__restrict__ T, float *__restrict__ W,
                                                      const float *__restrict__ GyT,
                                                      const int32_t *__restrict__ hit_rows,
                                                      const double *__restrict__ massD, int rows, int cols, int dim,
                                                      int e_pad) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int classes = kHex ? 2 : 1;
  const int ntile = e_pad / kSmoothTile;
  int cblk, zt;
  if (!smooth_tile_of_block(classes * ntile, (dim + 255) / 256, cblk, zt)) return;
  const int c = cblk * 256 + wave * 64 + lane;
  const bool live = c < dim;
  const int x = blockIdx.y;
  const int cls = zt / ntile;
  const int e0 = (zt - cls * ntile) * kSmoothTile;
  const float *G = GyT + ((int64_t)cls * rows) * e_pad + e0;
  const float *src = T + (kHex ? (int64_t)cls * rows * cols * dim : 0) + (int64_t)x * dim + (live ? c : 0);
  const int64_t ystride = (int64_t)cols * dim;
  float acc[kSmoothTile];
#pragma unroll
  for (int e = 0; e < kSmoothTile; ++e) acc[e] = 0.f;
  const int nr = hit_rows[rows];       // map rows that hold at least one chosen node
  for (int r = 0; r < nr; r += kSmoothUnroll) {
    int yb[kSmoothUnroll];
    float t[kSmoothUnroll];
#pragma unroll
    for (int u = 0; u < kSmoothUnroll; ++u) {
      yb[u] = hit_rows[min(r + u, nr - 1)];
      t[u] = (live && r + u < nr) ? src[(int64_t)yb[u] * ystride] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < kSmoothUnroll; ++u) {
      const float *g = G + (int64_t)yb[u] * e_pad;
#pragma unroll
      for (int e = 0; e < kSmoothTile; ++e) acc[e] = fmaf(g[e], t[u], acc[e]);
    }
  }
  if (live) {
#pragma unroll
    for (int e = 0; e < kSmoothTile; ++e) {
      const int yi = classes * (e0 + e) + cls;
      if (yi < rows) {
        const int64_t i = (int64_t)yi * cols + x;
        const double D = massD[i];
        if (D >= SOM_EPS_MASS) W[i * dim + c] = acc[e] / (float)D;
      }
    }
  }
}

// ---------------------------------------------------------------- feature channels, matrix cores
// On a map with a side of a hundred nodes or more, a pass of the separable filter is a real matrix
// product: out[m][c] = sum_t G[m][src_t] In[src_t][c] over the sources of one map line (pass x: the
// chosen nodes of a map row; pass y: the map rows that hold chosen nodes), m = the outputs along the
// line, c = the feature channels.  k_smooth_mfma runs it on v_mfma_f32_32x32x2_f32 - fp32 operands as
// they are, fp32 accumulation, the same arithmetic class as the vector kernels above.  MFMA rows =
// outputs m (A operand = coefficients from the transposed coefficient matrices), MFMA columns = 32
// consecutive channels (B operand = the source rows as they lie in memory), so a lane ends up with one
// channel and 16 outputs per block and every store instruction writes whole 128-byte runs.  A
// wavefront owns 32 channels and MB blocks of 32 outputs (all outputs of the line when they fit into
// seven blocks: the sources are then read exactly once), a workgroup 256 channels.  Both operands go
// through LDS in chunks of 16 sources, double-buffered: the coefficients because all wavefronts of
// the workgroup multiply with the same ones, the source rows because the workgroup can then fetch each
// of them as one contiguous kilobyte (one wavefront instruction) instead of eight separate 128-byte
// pieces at different times - the rows of one line are megabytes apart, and what the memory system
// sees of this kernel is a stream of such row visits.
constexpr int kMfmaChunk = 16;      // sources per LDS stage (8 MFMA k-steps of 2)
constexpr int kMfmaMaxBlocks = 7;   // 32-output blocks per wavefront: 7 x 16 accumulator registers
constexpr int kMfmaWaves = 8;       // wavefronts (32-channel slices) per workgroup

template <int MB, bool kPassY, bool kHex, bool kVec4>
__global__ __launch_bounds__(64 * kMfmaWaves) void k_smooth_mfma(const float *__restrict__ In, float *__restrict__ Out,
                                                     const float *__restrict__ Gt,
                                                     const int32_t *__restrict__ hit_x,
                                                     const int32_t *__restrict__ hit_n,
                                                     const int32_t *__restrict__ hit_rows,
                                                     const double *__restrict__ massD, int rows, int cols, int dim,
                                                     int g_pad, int groups) {
  constexpr int kM = 32 * MB;                        // outputs per workgroup
  constexpr int kCh = 32 * kMfmaWaves;               // channels per workgroup
  constexpr int kThreads = 64 * kMfmaWaves;
  constexpr int kVecs = kMfmaChunk * (kM / 4);       // 16-byte pieces of one coefficient chunk
  constexpr int kPer = (kVecs + kThreads - 1) / kThreads;
  constexpr int kBPer = kMfmaChunk * (kCh / 4) / kThreads;      // 16-byte pieces of a source chunk per thread
  static_assert(kMfmaChunk * (kCh / 4) % kThreads == 0, "source chunk must divide evenly among the threads");
  __shared__ __attribute__((aligned(16))) float sG[2][kMfmaChunk][kM];
  __shared__ __attribute__((aligned(16))) float sB[2][kMfmaChunk][kCh];
  __shared__ int sSrc[kSmoothMatMax + kMfmaChunk];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lhi = lane >> 5;
  const int cb0 = blockIdx.x * kCh;                  // first channel of the workgroup
  const int c = cb0 + wave * 32 + l32;
  const bool live = c < dim;
  const int line = blockIdx.y;                       // pass x: map row y; pass y: map column x
  const int part = blockIdx.z / groups;              // pass x: image (parity of the destination rows); pass y: class
  const int m0 = (blockIdx.z - part * groups) * kM;
  const int classes = kHex ? 2 : 1;

  int ns;                                            // sources of this line
  const int32_t *src;
  const float *G;                                    // coefficient rows: G[source * g_pad + m]
  const float *in;                                   // In[source * in_stride + channel]
  int64_t in_stride;
  if (kPassY) {
    ns = hit_rows[rows];
    if (ns <= 0) return;                             // nothing was chosen: every node keeps its weights
    src = hit_rows;
    G = Gt + (int64_t)part * rows * g_pad;
    in = In + (kHex ? (int64_t)part * rows * cols * dim : 0) + (int64_t)line * dim;
    in_stride = (int64_t)cols * dim;
  } else {
    ns = hit_n[line];
    if (ns == 0) return;                             // pass y skips this map row
    src = hit_x + (int64_t)line * cols;
    G = Gt + ((int64_t)(part * classes + (kHex ? (line & 1) : 0)) * cols) * g_pad;
    in = In + (int64_t)line * cols * dim;
    in_stride = dim;
  }

  // The source list of the line goes into LDS once, padded with its last entry to a whole chunk, so
  // that the loads below need neither an index fetch from memory nor a bounds branch: a source past
  // the end repeats the last one, and its values are replaced by zeros before they are multiplied.
  for (int i = tid; i < ns + kMfmaChunk; i += kThreads) sSrc[i] = src[i < ns ? i : ns - 1];
  __syncthreads();

  // Coefficients of a chunk, [source][output]: thread t fetches the 16-byte pieces t, t + kThreads, ...
  // Outputs past the padded row are read from its last piece; they are never stored.
  f32x4 greg[kPer];
  auto fetch_coefficients = [&](int t0) {
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = min(tid + i * kThreads, kVecs - 1);
      const int r = e / (kM / 4), q = e - r * (kM / 4);
      greg[i] = *reinterpret_cast<const f32x4 *>(G + (int64_t)sSrc[t0 + r] * g_pad + min(m0 + 4 * q, g_pad - 4));
    }
  };
  // Source rows of a chunk, [source][channel]: a wavefront fetches one row of kCh channels per
  // instruction.  Channels past dim repeat the last ones (their outputs are not stored).
  f32x4 breg[kBPer];
  auto fetch_sources = [&](int t0) {
#pragma unroll
    for (int i = 0; i < kBPer; ++i) {
      const int e = tid + i * kThreads;
      const int r = e / (kCh / 4), q = e - r * (kCh / 4);
      const float *row = in + (int64_t)sSrc[t0 + r] * in_stride;
      const int ch = cb0 + 4 * q;
      if (kVec4) {
        breg[i] = *reinterpret_cast<const f32x4 *>(row + min(ch, dim - 4));
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) breg[i][j] = row[min(ch + j, dim - 1)];
      }
    }
  };
  auto stash = [&](int stage, int t0) {
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = tid + i * kThreads;
      if (e < kVecs) *reinterpret_cast<f32x4 *>(&sG[stage][0][0] + 4 * e) = greg[i];
    }
#pragma unroll
    for (int i = 0; i < kBPer; ++i) {
      const int e = tid + i * kThreads;
      const bool on = t0 + e / (kCh / 4) < ns;
      *reinterpret_cast<f32x4 *>(&sB[stage][0][0] + 4 * e) = on ? breg[i] : f32x4{0.f, 0.f, 0.f, 0.f};
    }
  };

  f32x16 acc[MB];
#pragma unroll
  for (int b = 0; b < MB; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

  fetch_coefficients(0);
  fetch_sources(0);
  stash(0, 0);
  __syncthreads();
  int stage = 0;
  for (int t0 = 0; t0 < ns; t0 += kMfmaChunk) {
    const bool more = t0 + kMfmaChunk < ns;
    if (more) {
      fetch_coefficients(t0 + kMfmaChunk);
      fetch_sources(t0 + kMfmaChunk);
    }
    // operands of pair u + 1 are read from LDS while the matrix instructions of pair u run
    float a[2][MB], bv[2];
#pragma unroll
    for (int b = 0; b < MB; ++b) a[0][b] = sG[stage][lhi][32 * b + l32];
    bv[0] = sB[stage][lhi][wave * 32 + l32];
#pragma unroll
    for (int u = 0; u < kMfmaChunk / 2; ++u) {
      if (u + 1 < kMfmaChunk / 2) {
#pragma unroll
        for (int b = 0; b < MB; ++b) a[(u + 1) & 1][b] = sG[stage][2 * (u + 1) + lhi][32 * b + l32];
        bv[(u + 1) & 1] = sB[stage][2 * (u + 1) + lhi][wave * 32 + l32];
      }
      __builtin_amdgcn_sched_barrier(0);             // keep those reads ahead of the multiplications they overlap with
#pragma unroll
      for (int b = 0; b < MB; ++b) acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u & 1][b], bv[u & 1], acc[b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (more) stash(stage ^ 1, t0 + kMfmaChunk);     // that stage was last read before the previous barrier
    __syncthreads();
    stage ^= 1;
  }

  const int mtot = kPassY ? (rows - part + classes - 1) / classes : cols;     // outputs of this line (and class)
  // pass y divides by the neighbourhood mass: the masses of the line's outputs are fetched by the
  // workgroup once (0 stands for "below the floor: keep the weights"), so that the stores below are
  // not interleaved with dependent loads
  float *sD = &sG[0][0][0];                          // every wavefront has left the loop: the stages are free
  if (kPassY) {
    for (int ml = tid; ml < kM; ml += kThreads) {
      const int m = m0 + ml;
      double D = 0.0;
      if (m < mtot) D = massD[(int64_t)(classes * m + part) * cols + line];
      sD[ml] = D >= SOM_EPS_MASS ? (float)D : 0.f;
    }
    __syncthreads();
  }
  if (!live) return;
#pragma unroll
  for (int b = 0; b < MB; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int ml = 32 * b + 8 * (v >> 2) + 4 * lhi + (v & 3);
      const int m = m0 + ml;
      if (m >= mtot) continue;
      if (kPassY) {
        const float D = sD[ml];
        if (D > 0.f) Out[((int64_t)(classes * m + part) * cols + line) * dim + c] = acc[b][v] / D;
      } else {
        Out[(((int64_t)part * rows + line) * cols + m) * (int64_t)dim + c] = acc[b][v];
      }
    }
}

// The same product on the bf16 matrix cores, which run sixteen times the fp32 ones' rate: every fp32
// operand is carried as three bf16 parts, x = hi + mid + lo exactly up to 2^-25 |x| (each part is the
// rounding of what the parts before it leave), and a product a b as the six part products of order down
// to 2^-16: hi hi, hi mid, mid hi, mid mid, hi lo, lo hi.  What is dropped is below 2^-23 |a b|, the
// accumulation is fp32 as before: the same arithmetic class as the fp32 instruction, at three eighths of
// its matrix-pipe time (6 x 8 passes against 8 x 16 per 16 sources).  bf16 has the exponent range of
// fp32, so no operand needs a scale (fp16 parts would: coefficients of far nodes reach 1e-20).
// The parts are made once per workgroup and chunk, when the chunk goes into LDS: a thread fetches the
// values of eight consecutive sources for one output (coefficients) or one channel (source rows) -
// neighbouring lanes read neighbouring addresses - and writes their three times eight parts as three
// 16-byte pieces, which is exactly what a lane of v_mfma_f32_32x32x16_bf16 takes as its A or B operand.
// LDS rows of 32 bytes (16 sources); the two halves of a row swap places in every second group of
// eight rows, which spreads the 16-byte reads of 16 lanes over all banks.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Two values at a time: one packed conversion gives both bf16 parts, and their fp32 values are the two
// halves of that word shifted into place.
__device__ __forceinline__ uint32_t bf16_pair(float a, float b, float &a_back, float &b_back) {
  const bf16x2 h = __builtin_convertvector(f32x2{a, b}, bf16x2);
  const uint32_t u = __builtin_bit_cast(uint32_t, h);
  a_back = __uint_as_float(u << 16);
  b_back = __uint_as_float(u & 0xffff0000u);
  return u;
}

__device__ __forceinline__ void split_bf16x3(const float (&v)[8], bf16x8 &hi, bf16x8 &mid, bf16x8 &lo) {
  uint32_t h[4], m[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float a, b, c, d;
    h[i] = bf16_pair(v[2 * i], v[2 * i + 1], a, b);
    const float ra = v[2 * i] - a, rb = v[2 * i + 1] - b;       // exact
    m[i] = bf16_pair(ra, rb, c, d);
    float e, f;
    l[i] = bf16_pair(ra - c, rb - d, e, f);
  }
  hi = __builtin_bit_cast(bf16x8, uint4{h[0], h[1], h[2], h[3]});
  mid = __builtin_bit_cast(bf16x8, uint4{m[0], m[1], m[2], m[3]});
  lo = __builtin_bit_cast(bf16x8, uint4{l[0], l[1], l[2], l[3]});
}

template <int MB, bool kPassY, bool kHex, int kWaves>
__global__ __launch_bounds__(64 * kWaves) void k_smooth_mfma_split(const float *__restrict__ In, float *__restrict__ Out,
                                                       const float *__restrict__ Gt,
                                                       const int32_t *__restrict__ hit_x,
                                                       const int32_t *__restrict__ hit_n,
                                                       const int32_t *__restrict__ hit_rows,
                                                       const double *__restrict__ massD, int rows, int cols,
                                                       int dim, int g_pad, int groups) {
  constexpr int kM = 32 * MB;                        // outputs per workgroup
  constexpr int kMp = (kM + 63) / 64 * 64;           // ... rounded up to whole wavefronts of staging tasks
  constexpr int kCh = 32 * kWaves;                   // channels per workgroup
  constexpr int kThreads = 64 * kWaves;
  constexpr int kGPer = (2 * kMp + kThreads - 1) / kThreads;      // coefficient staging tasks per thread
  static_assert(kMfmaChunk == 16, "one matrix instruction takes 16 sources");
  static_assert(kWaves >= 2 && 2 * kCh == kThreads, "one source staging task per thread, its half the same for a wavefront");
  __shared__ __attribute__((aligned(16))) bf16x8 sG[2][3][kM][2];      // [stage][part][output][half of the 16 sources]
  __shared__ __attribute__((aligned(16))) bf16x8 sB[2][3][kCh][2];     // [stage][part][channel][half]
  __shared__ __attribute__((aligned(16))) int sSrc[kSmoothMatMax + kMfmaChunk];
  __shared__ float sD[kM];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lhi = lane >> 5;
  const int cb0 = blockIdx.x * kCh;
  const int c = cb0 + wave * 32 + l32;
  const bool live = c < dim;
  const int line = blockIdx.y;
  const int part = blockIdx.z / groups;
  const int m0 = (blockIdx.z - part * groups) * kM;
  const int classes = kHex ? 2 : 1;

  int ns;
  const int32_t *src;
  const float *G;
  const float *in;
  int64_t in_stride;
  if (kPassY) {
    ns = hit_rows[rows];
    if (ns <= 0) return;
    src = hit_rows;
    G = Gt + (int64_t)part * rows * g_pad;
    in = In + (kHex ? (int64_t)part * rows * cols * dim : 0) + (int64_t)line * dim;
    in_stride = (int64_t)cols * dim;
  } else {
    ns = hit_n[line];
    if (ns == 0) return;
    src = hit_x + (int64_t)line * cols;
    G = Gt + ((int64_t)(part * classes + (kHex ? (line & 1) : 0)) * cols) * g_pad;
    in = In + (int64_t)line * cols * dim;
    in_stride = dim;
  }
  for (int i = tid; i < ns + kMfmaChunk; i += kThreads) sSrc[i] = src[i < ns ? i : ns - 1];
  __syncthreads();

  // Staging tasks.  Source values: channel b_chl, the sources 8 b_half .. + 7 of the chunk (one task per thread).
  // Coefficients: task g = tid + i kThreads is output g % kMp, sources 8 (g / kMp) .. + 7.  Either half is the same
  // for a whole wavefront, so a source's row offset is a scalar and the loads need no per-lane address arithmetic.
  const int b_half = __builtin_amdgcn_readfirstlane(tid / kCh);
  const int b_chl = tid % kCh;
  const float *b_lane = in + min(cb0 + b_chl, dim - 1);     // channels past dim repeat the last one; never stored
  int g_half[kGPer], g_m[kGPer];
  bool g_task[kGPer];
  const float *g_lane[kGPer];
#pragma unroll
  for (int i = 0; i < kGPer; ++i) {
    const int g = tid + i * kThreads;
    g_half[i] = __builtin_amdgcn_readfirstlane(g / kMp);
    g_m[i] = g % kMp;
    g_task[i] = g_half[i] < 2 && g_m[i] < kM;
    g_lane[i] = G + min(m0 + g_m[i], g_pad - 1);            // outputs past the padded row repeat its last one; never stored
  }
  float gval[kGPer][8], bval[8];
  // the eight source indices of a task come out of LDS in two 16-byte reads (every lane the same address)
  auto source_rows = [&](int first, int64_t (&row)[8]) {
    const int4 lo4 = *reinterpret_cast<const int4 *>(&sSrc[first]), hi4 = *reinterpret_cast<const int4 *>(&sSrc[first + 4]);
    row[0] = __builtin_amdgcn_readfirstlane(lo4.x); row[1] = __builtin_amdgcn_readfirstlane(lo4.y);
    row[2] = __builtin_amdgcn_readfirstlane(lo4.z); row[3] = __builtin_amdgcn_readfirstlane(lo4.w);
    row[4] = __builtin_amdgcn_readfirstlane(hi4.x); row[5] = __builtin_amdgcn_readfirstlane(hi4.y);
    row[6] = __builtin_amdgcn_readfirstlane(hi4.z); row[7] = __builtin_amdgcn_readfirstlane(hi4.w);
  };
  auto fetch = [&](int t0) {
    int64_t row[8];
    source_rows(t0 + 8 * b_half, row);
#pragma unroll
    for (int u = 0; u < 8; ++u) bval[u] = b_lane[row[u] * in_stride];
#pragma unroll
    for (int i = 0; i < kGPer; ++i)
      if (g_task[i]) {
        source_rows(t0 + 8 * (g_half[i] & 1), row);
#pragma unroll
        for (int u = 0; u < 8; ++u) gval[i][u] = g_lane[i][row[u] * g_pad];
      }
  };
  auto stash = [&](int stage, int t0) {
    bf16x8 hi, mid, lo;
#pragma unroll
    for (int i = 0; i < kGPer; ++i)
      if (g_task[i]) {
        split_bf16x3(gval[i], hi, mid, lo);
        const int h = g_half[i] ^ ((g_m[i] >> 3) & 1);
        sG[stage][0][g_m[i]][h] = hi;
        sG[stage][1][g_m[i]][h] = mid;
        sG[stage][2][g_m[i]][h] = lo;
      }
    float bz[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) bz[u] = t0 + 8 * b_half + u < ns ? bval[u] : 0.f;     // sources past the end count as zero
    split_bf16x3(bz, hi, mid, lo);
    const int h = b_half ^ ((b_chl >> 3) & 1);
    sB[stage][0][b_chl][h] = hi;
    sB[stage][1][b_chl][h] = mid;
    sB[stage][2][b_chl][h] = lo;
  };

  f32x16 acc[MB];
#pragma unroll
  for (int b = 0; b < MB; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[b][v] = 0.f;

  // The loads of the next chunk are issued before this chunk's matrix instructions and used after them.  (Loads
  // of two or three chunks ahead, in more register buffers, measured slower: 6.2 and 6.7 against 6.1 ms for both passes on
  // a 336 x 205 map of 20,000 features - the passes are bound by how the memory system takes these visits of
  // rows a map line apart, and more of them in flight at once only scatter them further.)
  fetch(0);
  stash(0, 0);
  __syncthreads();
  int stage = 0;
  const int b_row = wave * 32 + l32;
  const int b_sel = lhi ^ ((b_row >> 3) & 1);
  for (int t0 = 0; t0 < ns; t0 += kMfmaChunk) {
    const bool more = t0 + kMfmaChunk < ns;
    if (more) fetch(t0 + kMfmaChunk);
    const bf16x8 bh = sB[stage][0][b_row][b_sel], bm = sB[stage][1][b_row][b_sel], bl = sB[stage][2][b_row][b_sel];
#pragma unroll
    for (int b = 0; b < MB; ++b) {
      const int a_row = 32 * b + l32;
      const int a_sel = lhi ^ ((a_row >> 3) & 1);
      const bf16x8 ah = sG[stage][0][a_row][a_sel], am = sG[stage][1][a_row][a_sel], al = sG[stage][2][a_row][a_sel];
      // the small products first
      acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, bh, acc[b], 0, 0, 0);
      acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bl, acc[b], 0, 0, 0);
      acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bm, acc[b], 0, 0, 0);
      acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(am, bh, acc[b], 0, 0, 0);
      acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bm, acc[b], 0, 0, 0);
      acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, bh, acc[b], 0, 0, 0);
    }
    if (more) stash(stage ^ 1, t0 + kMfmaChunk);     // that stage was last read before the previous barrier
    __syncthreads();
    stage ^= 1;
  }

  const int mtot = kPassY ? (rows - part + classes - 1) / classes : cols;
  if (kPassY) {
    for (int ml = tid; ml < kM; ml += kThreads) {
      const int m = m0 + ml;
      double D = 0.0;
      if (m < mtot) D = massD[(int64_t)(classes * m + part) * cols + line];
      sD[ml] = D >= SOM_EPS_MASS ? (float)D : 0.f;
    }
    __syncthreads();
  }
  if (!live) return;
#pragma unroll
  for (int b = 0; b < MB; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int ml = 32 * b + 8 * (v >> 2) + 4 * lhi + (v & 3);
      const int m = m0 + ml;
      if (m >= mtot) continue;
      if (kPassY) {
        const float D = sD[ml];
        if (D > 0.f) Out[((int64_t)(classes * m + part) * cols + line) * dim + c] = acc[b][v] / D;
      } else {
        Out[(((int64_t)part * rows + line) * cols + m) * (int64_t)dim + c] = acc[b][v];
      }
    }
}

// Blocks of 32 outputs per wavefront and groups of such wavefront tiles for a line of `outputs` outputs.
static void mfma_tiling(int outputs, int *mb, int *groups) {
  const int nb = (outputs + 31) / 32;
  *groups = (nb + kMfmaMaxBlocks - 1) / kMfmaMaxBlocks;
  *mb = (nb + *groups - 1) / *groups;
}

constexpr int kSplitWaves = 8;      // wavefronts of a k_smooth_mfma_split workgroup


template <bool kPassY, bool kHex>
static void launch_smooth_mfma(som_ctx *c, const float *In, float *Out, const float *Gt, int g_pad, int outputs,
                               int lines, int parts, bool split) {
  int mb, groups;
  mfma_tiling(outputs, &mb, &groups);
  const dim3 grid((unsigned)((c->dim + 32 * kMfmaWaves - 1) / (32 * kMfmaWaves)), (unsigned)lines, (unsigned)(parts * groups));
  const dim3 split_grid((unsigned)((c->dim + 32 * kSplitWaves - 1) / (32 * kSplitWaves)), (unsigned)lines, (unsigned)(parts * groups));
  // 16-byte loads of the source rows need rows that start and stay on 16-byte boundaries
  const bool vec4 = c->dim % 4 == 0 && c->dim >= 4 && (reinterpret_cast<uintptr_t>(In) & 15) == 0;
#define SOM_SMOOTH_MFMA(B)                                                                                          \
  do {                                                                                                              \
    if (split)                                                                                                      \
      hipLaunchKernelGGL((k_smooth_mfma_split<B, kPassY, kHex, kSplitWaves>), split_grid, dim3(64 * kSplitWaves), 0, \
                         c->stream, In, Out, Gt, c->hit_x, c->hit_n, c->hit_rows, c->massD, c->rows, c->cols, c->dim, \
                         g_pad, groups);                                                                            \
    else if (vec4)                                                                                                  \
      hipLaunchKernelGGL((k_smooth_mfma<B, kPassY, kHex, true>), grid, dim3(64 * kMfmaWaves), 0, c->stream, In, Out, \
                         Gt, c->hit_x, c->hit_n, c->hit_rows, c->massD, c->rows, c->cols, c->dim, g_pad, groups);    \
    else                                                                                                            \
      hipLaunchKernelGGL((k_smooth_mfma<B, kPassY, kHex, false>), grid, dim3(64 * kMfmaWaves), 0, c->stream, In,     \
                         Out, Gt, c->hit_x, c->hit_n, c->hit_rows, c->massD, c->rows, c->cols, c->dim, g_pad, groups); \
  } while (0)
  switch (mb) {
    case 1: SOM_SMOOTH_MFMA(1); break;
    case 2: SOM_SMOOTH_MFMA(2); break;
    case 3: SOM_SMOOTH_MFMA(3); break;
    case 4: SOM_SMOOTH_MFMA(4); break;
    case 5: SOM_SMOOTH_MFMA(5); break;
    case 6: SOM_SMOOTH_MFMA(6); break;
    default: SOM_SMOOTH_MFMA(7); break;
  }
#undef SOM_SMOOTH_MFMA
}

// ---------------------------------------------------------------- neighbourhoods with compact support
// The bubble function and the Gaussian cut off at the current radius (options -n and -p of the
// paper's command line) are not products of a factor in x and a factor in y, so the two-pass
// scheme above does not apply.  Their weights still depend only on the row distance a, the
// column offset and (hexagonal grids) the parities of the two rows, so they are tabulated once
// per epoch,
//   H2[class][a][t],  class = parity(yi) - parity(yb) + 1 (square grids: 0),
//   t = xi - xb + cols - 1 (planar)  or  (xi - xb) mod cols, continued cyclically past cols (toroid),
// so that the 16 weights of 16 neighbouring destination columns and one source node are
// contiguous: the same "lane owns a feature column, 16 outputs in registers, coefficients through
// scalar loads" kernel as k_smooth_x_mat, now in one pass over all chosen source nodes whose row is
// within reach, with the division at the end.  The count channel is summed in fp64 from the same table.
__device__ __forceinline__ int direct_table_width(int cols, int toroid) {
  return (toroid ? cols : 2 * cols - 1) + kSmoothTile;
}

__global__ __launch_bounds__(256) void k_direct_table(const EpochParams *__restrict__ params, int rows, int cols,
                                                      int hex, int toroid, int function, int compact,
                                                      float *__restrict__ H2) {
  const int width = direct_table_width(cols, toroid);
  const int classes = hex ? 3 : 1;
  const double r = params->radius;
  const double reach = 4.0 * r * r;               // q = 4 d^2 <= 4 r^2: inside the radius
  const double inv = params->inv8r2;
  const int64_t total = (int64_t)classes * rows * width;
  for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total; o += (int64_t)gridDim.x * blockDim.x) {
    const int t = (int)(o % width);
    const int a_raw = (int)((o / width) % rows);
    const int cls = (int)(o / ((int64_t)width * rows));
    const int dpar = hex ? cls - 1 : 0;
    const int dx = toroid ? t % cols : t - (cols - 1);
    long long m = 2ll * dx + dpar;
    m = m < 0 ? -m : m;
    long long a = a_raw;
    if (toroid) {
      if (2ll * cols - m < m) m = 2ll * cols - m;
      if (rows - a < a) a = rows - a;
    }
    const double q = (double)(m * m + (hex ? 3 : 4) * a * a);
    const bool inside = q <= reach;
    float h;
    if (function == SOM_NEIGHBORHOOD_BUBBLE) h = inside ? 1.f : 0.f;
    else h = (compact && !inside) ? 0.f : (float)exp(-q * inv);
    H2[o] = h;
  }
}

__device__ __forceinline__ int direct_table_index(int xi, int xb, int cols, int toroid) {
  if (!toroid) return xi - xb + cols - 1;
  int d = xi - xb;
  return d < 0 ? d + cols : d;
}

__global__ __launch_bounds__(256) void k_count_direct(const int32_t *__restrict__ counts,
                                                      const int32_t *__restrict__ hit_x,
                                                      const int32_t *__restrict__ hit_n,
                                                      const int32_t *__restrict__ hit_rows,
                                                      const float *__restrict__ H2, int rows, int cols, int hex,
                                                      int toroid, double *__restrict__ massD) {
  const int k = rows * cols;
  const int width = direct_table_width(cols, toroid);
  const int nr = hit_rows[rows];
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < k; i += gridDim.x * blockDim.x) {
    const int yi = i / cols, xi = i - yi * cols;
    double s = 0.0;
    for (int r = 0; r < nr; ++r) {
      const int yb = hit_rows[r];
      const int a = yi > yb ? yi - yb : yb - yi;
      const int cls = hex ? (yi & 1) - (yb & 1) + 1 : 0;
      const float *row = H2 + ((int64_t)cls * rows + a) * width;
      const int32_t *hx = hit_x + (int64_t)yb * cols;
      const int nh = hit_n[yb];
      for (int t = 0; t < nh; ++t) {
        const int xb = hx[t];
        s += (double)row[direct_table_index(xi, xb, cols, toroid)] * (double)counts[yb * cols + xb];
      }
    }
    massD[i] = s;
  }
}

// Positions in the ascending list a[0..n) of the first entries that are >= v0, >= v1 and >= v2: every
// wavefront counts the smaller entries 64 at a time (one load per 64 entries, all in flight together;
// a bisection would be a chain of dependent loads per row).
__device__ __forceinline__ void first_not_below3(const int32_t *__restrict__ a, int n, int lane, int v0, int v1, int v2,
                                                 int &p0, int &p1, int &p2) {
  p0 = p1 = p2 = 0;
  for (int t0 = 0; t0 < n; t0 += 64) {
    const int t = t0 + lane;
    const int x = t < n ? a[t] : 0x7fffffff;
    p0 += __popcll(__ballot(x < v0));
    p1 += __popcll(__ballot(x < v1));
    p2 += __popcll(__ballot(x < v2));
  }
  p0 = __builtin_amdgcn_readfirstlane(p0);      // the same in every lane: keep the loops over them scalar
  p1 = __builtin_amdgcn_readfirstlane(p1);
  p2 = __builtin_amdgcn_readfirstlane(p2);
}

// grid = (ceil(dim/256), rows, ceil(cols/16)).  Source rows whose distance alone puts them out of
// reach are skipped whole, and of the others only the source nodes whose column can be within reach of
// one of the tile's 16 destination columns are visited: at row distance a that is |dx| <=
// (sqrt(4 r^2 - (4 or 3) a^2) + 1) / 2, a stretch of the row's ascending hit list (two stretches
// where it wraps round a toroid map).  The table holds zeros for everything
// skipped, so the sums are the same; on a 336-column map at r = 30 the stretch is a seventh of the row.
template <bool kHex>
__global__ __launch_bounds__(256) void k_smooth_direct(const float *__restrict__ S, float *__restrict__ W,
                                                       const float *__restrict__ H2,
                                                       const int32_t *__restrict__ hit_x,
                                                       const int32_t *__restrict__ hit_n,
                                                       const int32_t *__restrict__ hit_rows,
                                                       const double *__restrict__ massD,
                                                       const EpochParams *__restrict__ params, int rows, int cols,
                                                       int dim, int toroid, int bounded) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.x * 256 + wave * 64 + lane;
  const bool live = c < dim;
  const int yi = blockIdx.y;
  const int xi0 = blockIdx.z * kSmoothTile;
  const int width = direct_table_width(cols, toroid);
  const double reach = 4.0 * params->radius * params->radius;
  float acc[kSmoothTile];
#pragma unroll
  for (int e = 0; e < kSmoothTile; ++e) acc[e] = 0.f;
  const int nr = hit_rows[rows];
  for (int r = 0; r < nr; ++r) {
    const int yb = hit_rows[r];
    int a = yi > yb ? yi - yb : yb - yi;
    const int a_wrapped = (toroid && rows - a < a) ? rows - a : a;
    const double left = reach - (double)((kHex ? 3ll : 4ll) * a_wrapped * a_wrapped);
    if (bounded && left < 0.0) continue;
    const int cls = kHex ? (yi & 1) - (yb & 1) + 1 : 0;
    const float *trow = H2 + ((int64_t)cls * rows + a) * width;
    const float *src = S + (int64_t)yb * cols * dim + (live ? c : 0);
    const int32_t *hx = hit_x + (int64_t)yb * cols;
    const int nh = hit_n[yb];
    // stretches [seg_lo[s], seg_hi[s]) of the hit list
    int seg_lo[2] = {0, 0}, seg_hi[2] = {nh, 0};
    if (bounded && nh >= 8) {
      const int half = (int)(0.5 * sqrt(left)) + 2;        // |dx| of a node within reach is below this
      if (2 * half + kSmoothTile < cols) {
        int lo = xi0 - half, hi = xi0 + kSmoothTile - 1 + half;
        if (toroid) {
          const int span = hi - lo;                         // < cols - 1
          lo %= cols;
          if (lo < 0) lo += cols;
          hi = lo + span;
        }
        int p_lo, p_hi, p_wrap;                             // hi >= cols (toroid only): lo .. cols - 1, then 0 .. hi - cols
        first_not_below3(hx, nh, lane, lo, hi + 1, hi - cols + 1, p_lo, p_hi, p_wrap);
        seg_lo[0] = p_lo;
        seg_hi[0] = p_hi;
        if (toroid && hi >= cols) seg_hi[1] = p_wrap;
      }
    }
#pragma unroll
    for (int sgm = 0; sgm < 2; ++sgm) {
      const int t_end = seg_hi[sgm];
      for (int t = seg_lo[sgm]; t < t_end; t += kSmoothUnroll) {
        int xb[kSmoothUnroll];
        float s[kSmoothUnroll];
#pragma unroll
        for (int u = 0; u < kSmoothUnroll; ++u) {
          xb[u] = hx[min(t + u, t_end - 1)];
          s[u] = (live && t + u < t_end) ? src[(int64_t)xb[u] * dim] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kSmoothUnroll; ++u) {
          const float *g = trow + direct_table_index(xi0, xb[u], cols, toroid);
#pragma unroll
          for (int e = 0; e < kSmoothTile; ++e) acc[e] = fmaf(g[e], s[u], acc[e]);
        }
      }
    }
  }
  if (live) {
#pragma unroll
    for (int e = 0; e < kSmoothTile; ++e) {
      const int xi = xi0 + e;
      if (xi < cols) {
        const int64_t i = (int64_t)yi * cols + xi;
        const double D = massD[i];
        if (D >= SOM_EPS_MASS) W[i * dim + c] = acc[e] / (float)D;
      }
    }
  }
}

static hipError_t launch_smooth_direct(som_ctx *c, float *W) {
  const int hex = c->grid_type == SOM_GRID_HEXAGONAL;
  const int toroid = c->map_type == SOM_MAP_TOROID;
  const int width = (toroid ? c->cols : 2 * c->cols - 1) + kSmoothTile;
  const int64_t entries = (int64_t)(hex ? 3 : 1) * c->rows * width;
  int tb = (int)((entries + 255) / 256);
  if (tb > c->n_cu * 8) tb = c->n_cu * 8;
  hipLaunchKernelGGL(k_direct_table, dim3(tb), dim3(256), 0, c->stream, c->params, c->rows, c->cols, hex, toroid,
                     c->nb_function, c->nb_compact, c->H2);
  hipLaunchKernelGGL(k_hit_lists, dim3(c->rows < 1024 ? c->rows : 1024), dim3(64), 0, c->stream, c->counts, c->rows,
                     c->cols, c->hit_x, c->hit_n);
  hipLaunchKernelGGL(k_hit_rows, dim3(1), dim3(64), 0, c->stream, c->hit_n, c->rows, c->hit_rows);
  int cb = (c->k + 255) / 256;
  hipLaunchKernelGGL(k_count_direct, dim3(cb), dim3(256), 0, c->stream, c->counts, c->hit_x, c->hit_n, c->hit_rows,
                     c->H2, c->rows, c->cols, hex, toroid, c->massD);
  const dim3 grid((unsigned)((c->dim + 255) / 256), (unsigned)c->rows,
                  (unsigned)((c->cols + kSmoothTile - 1) / kSmoothTile));
  const int bounded = c->nb_function == SOM_NEIGHBORHOOD_BUBBLE || c->nb_compact;
  if (hex)
    hipLaunchKernelGGL(k_smooth_direct<true>, grid, dim3(256), 0, c->stream, c->S, W, c->H2, c->hit_x, c->hit_n,
                       c->hit_rows, c->massD, c->params, c->rows, c->cols, c->dim, toroid, bounded);
  else
    hipLaunchKernelGGL(k_smooth_direct<false>, grid, dim3(256), 0, c->stream, c->S, W, c->H2, c->hit_x, c->hit_n,
                       c->hit_rows, c->massD, c->params, c->rows, c->cols, c->dim, toroid, bounded);
  return hipGetLastError();
}

hipError_t launch_smooth_and_divide(som_ctx *c, float *W) {
  if (c->nb_function != SOM_NEIGHBORHOOD_GAUSSIAN || c->nb_compact) return launch_smooth_direct(c, W);
  const int hex = c->grid_type == SOM_GRID_HEXAGONAL;
  const int toroid = c->map_type == SOM_MAP_TOROID;
  const int images = hex ? 2 : 1;
  int cb = (images * c->k + 255) / 256;
  hipLaunchKernelGGL(k_count_pass_x, dim3(cb), dim3(256), 0, c->stream, c->counts, c->gx, c->rows, c->cols, hex,
                     toroid, c->cntT);
  hipLaunchKernelGGL(k_count_pass_y, dim3((c->k + 255) / 256), dim3(256), 0, c->stream, c->cntT, c->gy, c->rows,
                     c->cols, hex, toroid, c->massD);
  if (c->GxT) {           // sides small enough for coefficient matrices
    const int par = hex ? 2 : 1;
    const int64_t entries = (int64_t)par * par * c->cols * c->xi_pad + (int64_t)par * c->rows * c->e_pad;
    int tb = (int)((entries + 255) / 256);
    if (tb > c->n_cu * 8) tb = c->n_cu * 8;
    hipLaunchKernelGGL(k_smooth_tables, dim3(tb), dim3(256), 0, c->stream, c->gx, c->gy, c->rows, c->cols, hex, toroid,
                       c->xi_pad, c->e_pad, c->GxT, c->GyT);
    hipLaunchKernelGGL(k_hit_lists, dim3(c->rows < 1024 ? c->rows : 1024), dim3(64), 0, c->stream, c->counts, c->rows,
                       c->cols, c->hit_x, c->hit_n);
    hipLaunchKernelGGL(k_hit_rows, dim3(1), dim3(64), 0, c->stream, c->hit_n, c->rows, c->hit_rows);
    const unsigned cb256 = (unsigned)((c->dim + 255) / 256);
    const unsigned xt = (unsigned)(images * ((c->cols + kSmoothTile - 1) / kSmoothTile));
    const unsigned yt = (unsigned)(par * (c->e_pad / kSmoothTile));
    const bool fold = cb256 >= 8;       // enough channel blocks to keep every XCD busy
    const unsigned cb8 = (cb256 + 7) / 8 * 8;
    const dim3 gx = fold ? dim3(cb8 * xt, c->rows, 1) : dim3(cb256, c->rows, xt);
    const dim3 gy = fold ? dim3(cb8 * yt, c->cols, 1) : dim3(cb256, c->cols, yt);
    // a pass runs on the matrix cores when its line is long enough to fill their 32-output blocks
    const bool mfma_x = c->smooth_mfma_min > 0 && c->cols >= c->smooth_mfma_min;
    const bool mfma_y = c->smooth_mfma_min > 0 && c->rows >= c->smooth_mfma_min;
    // ... and on the bf16 ones, operands in three parts, when the line is long enough for the matrix pipe to be the limit
    const bool split_x = mfma_x && c->smooth_split_min > 0 && c->cols >= c->smooth_split_min;
    const bool split_y = mfma_y && c->smooth_split_min > 0 && c->rows >= c->smooth_split_min;
    if (hex) {
      if (mfma_x) launch_smooth_mfma<false, true>(c, c->S, c->T, c->GxT, c->xi_pad, c->cols, c->rows, 2, split_x);
      else hipLaunchKernelGGL(k_smooth_x_mat<true>, gx, dim3(256), 0, c->stream, c->S, c->T, c->GxT,
                              c->hit_x, c->hit_n, c->rows, c->cols, c->dim, c->xi_pad);
      if (mfma_y) launch_smooth_mfma<true, true>(c, c->T, W, c->GyT, c->e_pad, (c->rows + 1) / 2, c->cols, 2, split_y);
      else hipLaunchKernelGGL(k_smooth_y_mat<true>, gy, dim3(256), 0, c->stream, c->T, W, c->GyT,
                              c->hit_rows, c->massD, c->rows, c->cols, c->dim, c->e_pad);
    } else {
      if (mfma_x) launch_smooth_mfma<false, false>(c, c->S, c->T, c->GxT, c->xi_pad, c->cols, c->rows, 1, split_x);
      else hipLaunchKernelGGL(k_smooth_x_mat<false>, gx, dim3(256), 0, c->stream, c->S, c->T, c->GxT,
                              c->hit_x, c->hit_n, c->rows, c->cols, c->dim, c->xi_pad);
      if (mfma_y) launch_smooth_mfma<true, false>(c, c->T, W, c->GyT, c->e_pad, c->rows, c->cols, 1, split_y);
      else hipLaunchKernelGGL(k_smooth_y_mat<false>, gy, dim3(256), 0, c->stream, c->T, W, c->GyT,
                              c->hit_rows, c->massD, c->rows, c->cols, c->dim, c->e_pad);
    }
    return hipGetLastError();
  }
  const unsigned cblk = (unsigned)((c->dim + kSmoothCols - 1) / kSmoothCols);
  if (hex) {
    hipLaunchKernelGGL(k_smooth_x<true>, dim3(cblk, c->rows, 2), dim3(256), 0, c->stream, c->S, c->T, c->gx,
                       c->rows, c->cols, c->dim, toroid);
    hipLaunchKernelGGL(k_smooth_y_divide<true>, dim3(cblk, c->cols), dim3(256), 0, c->stream, c->T, W, c->gy,
                       c->massD, c->rows, c->cols, c->dim, toroid);
  } else {
    hipLaunchKernelGGL(k_smooth_x<false>, dim3(cblk, c->rows, 1), dim3(256), 0, c->stream, c->S, c->T, c->gx,
                       c->rows, c->cols, c->dim, toroid);
    hipLaunchKernelGGL(k_smooth_y_divide<false>, dim3(cblk, c->cols), dim3(256), 0, c->stream, c->T, W, c->gy,
                       c->massD, c->rows, c->cols, c->dim, toroid);
  }
  return hipGetLastError();
}

}  // namespace som
