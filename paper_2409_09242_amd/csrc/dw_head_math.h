// Softmax cross-entropy of one sample and its derivative along Rs (Section II eq.(2) with the softmax loss; the
// R-derivative is the one of Section IV-B's Hessian-vector product), shared by the head kernel and by the fp32
// output-layer kernel that computes the logits itself.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>

#include "dw.h"

namespace dw {

// s[c], rs[c]: logits and their directional derivative for c < C (entries beyond C are ignored), y: the label.
// d[c] = (p_c - [c == y]) * invB, rd[c] = p_c (Rs_c - <p, Rs>) * invB for c < C, zero beyond.  Returns -log p_y.
__device__ __forceinline__ float head_row(const float (&s_in)[DW_MAX_CLASSES], const float (&rs_in)[DW_MAX_CLASSES],
                                          int y, int C, float invB, float (&d)[DW_MAX_CLASSES],
                                          float (&rd)[DW_MAX_CLASSES]) {
  float s[DW_MAX_CLASSES], rs[DW_MAX_CLASSES];
  float mx = -INFINITY;
  int amax = 0;
#pragma unroll
  for (int c = 0; c < DW_MAX_CLASSES; ++c) {
    s[c] = c < C ? s_in[c] : -INFINITY;
    rs[c] = c < C ? rs_in[c] : 0.f;
    if (s[c] > mx) { mx = s[c]; amax = c; }
  }
  // e_c = exp(s_c - max); the largest term is exactly 1, so sums that leave it (or the label's term)
  // out keep full relative precision when the prediction is confident
  float rest_max = 0.f, rest_y = 0.f, sy = 0.f;
#pragma unroll
  for (int c = 0; c < DW_MAX_CLASSES; ++c) {
    const float e = c < C ? expf(s[c] - mx) : 0.f;
    if (c == y) sy = s[c] - mx;
    if (c != amax) rest_max += e;
    if (c != y) rest_y += e;
    s[c] = e;
  }
  const float sum = 1.0f + rest_max;
  const float inv = 1.0f / sum;
#pragma unroll
  for (int c = 0; c < DW_MAX_CLASSES; ++c) s[c] *= inv;   // p_c
  const float one_minus_py = rest_y * inv;         // 1 - p_y without cancellation
#pragma unroll
  for (int c = 0; c < DW_MAX_CLASSES; ++c) {
    d[c] = 0.f; rd[c] = 0.f;
    if (c < C) {
      d[c] = (c == y ? -one_minus_py : s[c]) * invB;  // d(mean loss)/d s_L = (p - onehot)/B
      // its derivative along Rs_L: p_c (Rs_c - <p, Rs>) / B, with Rs_c - <p, Rs> written as
      // sum_c' p_c' (Rs_c - Rs_c') so that a confident prediction does not cancel
      float ctr = 0.f;
#pragma unroll
      for (int c2 = 0; c2 < DW_MAX_CLASSES; ++c2) ctr += s[c2] * (rs[c] - rs[c2]);
      rd[c] = s[c] * ctr * invB;
    }
  }
  return log1pf(rest_max) - sy;                    // -log p_y = log(sum_c e_c) - (s_y - max)
}

}  // namespace dw
