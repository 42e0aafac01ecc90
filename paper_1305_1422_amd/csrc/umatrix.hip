// U-matrix (paper: U-matrix equation): U(j) = mean over the immediate neighbours i of node j of
// the Euclidean distance |w_i - w_j|.  Immediate neighbours are the other nodes at grid distance
// <= 1: up to four on a square grid, up to six on a hexagonal one, fewer on the border of a
// planar map; on a toroid the map wraps.  One wavefront per node; distances summed in fp64.
#include "som_internal.hpp"

#include <math.h>

namespace som {

__global__ __launch_bounds__(256) void k_umatrix(const float *__restrict__ W, int rows, int cols, int dim,
                                                 int toroid, int hex, float *__restrict__ U) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int nwaves = gridDim.x * 4;
  const int k = rows * cols;
  for (int j = wave; j < k; j += nwaves) {
    const int yj = j / cols, xj = j - yj * cols;
    int nb[8];
    int cnt = 0;
    for (int dy = -1; dy <= 1; ++dy)
      for (int dx = -1; dx <= 1; ++dx) {
        if (dx == 0 && dy == 0) continue;
        int x = xj + dx, y = yj + dy;
        if (toroid) {
          x = (x + cols) % cols;
          y = (y + rows) % rows;
        } else if (x < 0 || x >= cols || y < 0 || y >= rows) {
          continue;
        }
        const int i = y * cols + x;
        if (i == j || grid_q(rows, cols, toroid, hex, x, y, xj, yj) > 4) continue;
        bool seen = false;
        for (int t = 0; t < cnt; ++t) seen |= (nb[t] == i);      // tiny toroids alias offsets
        if (!seen) nb[cnt++] = i;
      }
    double sum = 0.0;
    const float *wj = W + (int64_t)j * dim;
    for (int t = 0; t < cnt; ++t) {
      const float *wi = W + (int64_t)nb[t] * dim;
      double s = 0.0;
      for (int c = lane; c < dim; c += kWave) {
        const double d = (double)wi[c] - (double)wj[c];
        s += d * d;
      }
      sum += sqrt(wave_sum(s));
    }
    if (lane == 0) U[j] = cnt ? (float)(sum / cnt) : 0.f;
  }
}

hipError_t launch_umatrix(som_ctx *c, const float *W, float *U) {
  int blocks = (c->k + 3) / 4;
  if (blocks > c->n_cu * 16) blocks = c->n_cu * 16;
  hipLaunchKernelGGL(k_umatrix, dim3(blocks), dim3(256), 0, c->stream, W, c->rows, c->cols, c->dim,
                     c->map_type == SOM_MAP_TOROID, c->grid_type == SOM_GRID_HEXAGONAL, U);
  return hipGetLastError();
}

}  // namespace som
