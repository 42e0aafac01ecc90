// Rounding-error bound of the filter scores of the best-matching-unit search (paper: BMU equation):
// the model of one filter variant and the margin it gives an instance.  Used by the exact stage
// (bmu_exact.hip) and by the block selection of the two-level dense search (bmu_two_level.hip).
#pragma once

#include "som_internal.hpp"

#include <math.h>

namespace som {

// Coefficients of the bound for one filter variant: |s_filter - s_exact| <=
//   u [ coef_xw X Wm + coef_floor (xscale_j Wm + wscale X) + 4 Wm^2 + 6 M Wm ].
struct MarginModel {
  double coef_xw;
  double coef_floor;         // 0 for the fp32 pass
  const float *xscale;       // [n] power-of-two scale of every instance (split-fp16 pass), else null
  const float *wscale;       // [1] power-of-two scale of the centred code book, else null
  int x_centered;            // the instances were centred too (split-fp16 pass): X = |x - mu|, no term in M
  const int64_t *indptr;     // sparse rows: coef_xw = 2 max(row length, 1) + 6 (one FMA chain over the row)
  const float *row_q;        // [n] sparse rows scored against the 16-bit code book: sum_nz |v_c| step_c
  // sparse rows whose frequent columns went through the matrix cores (csr_hot.hip): the split-fp16 bound
  // of that block, coef_hot |x_hot| Wm + sqrt(kHot) (hot_xscale_j Wm + hot_wscale |x_hot|), in units of u
  double coef_hot;           // 0: no hot block
  const float *hot_xn;       // [n] |x_hot|^2
  const float *hot_xscale;   // [n]
  const float *hot_wscale;   // [1]
};

__device__ __forceinline__ double score_margin(const MarginModel &mm, int64_t j, double xnorm2, double wmax2,
                                               double munorm2) {
  const double u = 5.9604644775390625e-08;   // 2^-24
  const double xn = sqrt(xnorm2 * (1.0 + 1.2e-7));
  const double wm = sqrt(wmax2 * (1.0 + 1.2e-7));
  const double mn = mm.x_centered ? 0.0 : sqrt(munorm2 * (1.0 + 1.2e-7));
  double coef = mm.coef_xw;
  double absolute = 0.0;
  if (mm.indptr) {
    const double len = (double)(mm.indptr[j + 1] - mm.indptr[j]);
    coef = 2.0 * (len < 1.0 ? 1.0 : len) + 6.0;     // + 2: the product of value and column step is rounded
    // a quantised entry is within 0.51 steps of w' (0.5 from rounding, the rest from the fp32
    // division), so the dot product moves by at most 0.51 sum |v_c| step_c (the sum itself carries
    // fp32 rounding: 1e-5 relative is ample), the score by twice that
    if (mm.row_q) absolute = 2.0 * 0.51 * (1.0 + 1e-5) * (double)mm.row_q[j];
  }
  double bound = coef * xn * wm + 4.0 * wm * wm + 6.0 * mn * wm;
  if (mm.coef_hot > 0.0) {
    const double xh = sqrt((double)mm.hot_xn[j] * (1.0 + 1.2e-7));
    bound += mm.coef_hot * xh * wm + sqrt((double)kHot) * ((double)mm.hot_xscale[j] * wm + (double)*mm.hot_wscale * xh);
  }
  if (mm.xscale) bound += mm.coef_floor * ((double)mm.xscale[j] * wm + (double)*mm.wscale * xn);
  return 2.125 * (u * bound + absolute);          // both scores of a pair may err, plus slack for higher-order terms
}

// The rounding model of the filter that produced the scores (mode = kCertify*); host code, bmu_exact.hip.
MarginModel margin_model(const som_ctx *c, int mode, const int64_t *indptr, bool hot = false);

}  // namespace som
