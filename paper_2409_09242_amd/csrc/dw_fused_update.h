// The AdaHessian update of Section IV-B applied to one wave's tile of a weight-gradient product while g and Hz are
// still in registers (same arithmetic as update_kernel, Hessian power 1); shared by the bf16 and the fp32 dual GEMM.
//
// The tile is TM x 2 MFMA tiles of 32 x 32 (TM*32 rows x 64 columns of W_l); element (m, n) is parameter m*ldc + n of
// the layer's W block.  The epilogue is bound by HBM, and HBM streams a quarter faster when a wave instruction
// touches 256 contiguous bytes per row instead of 128 (measured).  The MFMA layout gives a lane one column, i.e.
// 128-byte row pieces per half-wave, so g and Hz go through a private LDS region of the wave: the accumulators of one
// row of MFMA tiles (32 rows x 64 columns) are scattered into [row][72 floats] arrays and read back as one float4 per
// lane, 16 lanes per row.  A batch is then 4 rows x 256 bytes per access, all state is moved as float4 (bf16 copy:
// 8 bytes) with non-temporal accesses (it streams through once), the sign bits of a lane's four parameters come
// from one word, and the block mean of D = z*Hz along fan-in is the update kernel's: four values in the lane, then
// a butterfly over avg_block / 4 lanes.  The loads of two later batches are in flight while a batch is computed;
// scheduling fences keep the compiler from hoisting more.  Whole tiles only (no element out of range), offsets
// inside the W block fit 32 bits, the block's first parameter is a multiple of 32.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dw_internal.h"
#include "dw_device_util.h"

namespace dw {

typedef float fu_floatx16 __attribute__((ext_vector_type(16)));

// floats of LDS one wave needs: g and Hz of one row of MFMA tiles, [32][72] each
__host__ __device__ constexpr int fused_update_lds_floats() { return 2 * 32 * 72; }

// acc, racc: the wave's accumulators (plain product = g, R-companion = Hz), MFMA 32x32 layout: lane holds column
// lane%32 of each tile, rows (r/4)*8 + (lane/32)*4 + r%4.  gl: the wave's LDS region.  wbase: the worker's offset
// in theta, m, v (and the bf16 copy).  row_base, col_base: first row and column of the wave's tile in W_l.
// zrow: sign bits of z from the first parameter of the W block on.  ib1, ib2: the worker's 1/(1 - beta^t).
// Returns this lane's share of the squared distance of the new parameters to the centre (0 unless f.dist).
// B16: also store the bf16 copy of the new parameters.  PROBES: the diagonal estimate is the mean over several
// Hutchinson probes, D = (f.dacc + z*Hz) * f.d_scale, f.dacc holding the sum over the earlier probes.
template <int TM, bool B16, bool PROBES = false>
__device__ __forceinline__ float fused_update_wave_tile(const fu_floatx16 (&acc)[TM][2], const fu_floatx16 (&racc)[TM][2],
                                                        float* gl, const FuseArgs& f, int64_t wbase, int ldc,
                                                        int row_base, int col_base, const uint32_t* zrow, float ib1,
                                                        float ib2, int lane) {
  const int l32 = lane & 31, lhalf = lane >> 5;
  float* th_w = f.theta + wbase; float* m_w = f.m + wbase; float* v_w = f.v + wbase;
  uint16_t* b16_w = B16 ? f.wb16 + wbase : nullptr;
  const float inv_b = 1.0f / (float)f.avg_block;
  constexpr int PR = 72;                                    // floats per LDS row: both half-waves hit distinct banks
  float* hl = gl + 32 * PR;
  constexpr int NB = TM * 8, DEPTH = 3;
  struct Batch { uint32_t e, zw; float4 th, mm, vv, cc, dd; };
  const float* dacc_w = PROBES ? f.dacc + wbase : nullptr;
  const int brow = lane >> 4, bcol = (lane & 15) * 4;
  auto load_batch = [&](Batch& bt, int bb) {
    const int i = bb / 8, b = bb % 8;
    const uint32_t m = (uint32_t)(row_base + i * 32 + b * 4 + brow), n = (uint32_t)(col_base + bcol);
    bt.e = m * (uint32_t)ldc + n;                         // offset inside the W block, a multiple of 4
    bt.th = nt_load4(th_w + bt.e); bt.mm = nt_load4(m_w + bt.e);   // the state streams through once: no reuse in L2
    bt.vv = nt_load4(v_w + bt.e);
    bt.cc = f.dist ? *reinterpret_cast<const float4*>(f.centre + bt.e) : make_float4(0.f, 0.f, 0.f, 0.f);
    bt.zw = zrow[bt.e >> 5];
    if constexpr (PROBES) bt.dd = nt_load4(dacc_w + bt.e);
  };
  float nsum = 0.f;
  const int group_lanes = f.avg_block >> 2;                 // lanes that share one averaging block (when b > 4)
  auto finish_batch = [&](const Batch& bt, int b) {
    const float4 g4 = *reinterpret_cast<const float4*>(gl + (b * 4 + brow) * PR + bcol);
    const float4 h4 = *reinterpret_cast<const float4*>(hl + (b * 4 + brow) * PR + bcol);
    const float g[4] = {g4.x, g4.y, g4.z, g4.w}, hz[4] = {h4.x, h4.y, h4.z, h4.w};
    const float th[4] = {bt.th.x, bt.th.y, bt.th.z, bt.th.w}, mm[4] = {bt.mm.x, bt.mm.y, bt.mm.z, bt.mm.w};
    const float vv[4] = {bt.vv.x, bt.vv.y, bt.vv.z, bt.vv.w}, cc[4] = {bt.cc.x, bt.cc.y, bt.cc.z, bt.cc.w};
    const uint32_t zb4 = bt.zw >> (bt.e & 31u);
    float D[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) D[q] = ((zb4 >> q) & 1u) ? hz[q] : -hz[q];      // Hutchinson: z * Hz
    if constexpr (PROBES) {
      const float dd[4] = {bt.dd.x, bt.dd.y, bt.dd.z, bt.dd.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) D[q] = (dd[q] + D[q]) * f.d_scale;
    }
    if (f.avg_block == 2) {
      const float p0 = 0.5f * (D[0] + D[1]), p1 = 0.5f * (D[2] + D[3]);
      D[0] = D[1] = p0; D[2] = D[3] = p1;
    } else if (f.avg_block >= 4) {
      float sD = (D[0] + D[1]) + (D[2] + D[3]);
#pragma unroll
      for (int off = 1; off < 8; off <<= 1) {
        const float t = __shfl_xor(sD, off);
        sD += off < group_lanes ? t : 0.f;
      }
      sD *= inv_b;
      D[0] = D[1] = D[2] = D[3] = sD;
    }
    float t1[4], m1[4], v1[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      m1[q] = f.beta1 * mm[q] + (1.0f - f.beta1) * g[q];
      v1[q] = f.beta2 * vv[q] + (1.0f - f.beta2) * (D[q] * D[q]);
      const float mhat = m1[q] * ib1, vhat = v1[q] * ib2;
      t1[q] = th[q] - f.lr * (mhat / (sqrtf(vhat) + f.eps));
      const float d = t1[q] - cc[q];
      nsum += d * d;
    }
    nt_store4(th_w + bt.e, make_float4(t1[0], t1[1], t1[2], t1[3]));
    nt_store4(m_w + bt.e, make_float4(m1[0], m1[1], m1[2], m1[3]));
    nt_store4(v_w + bt.e, make_float4(v1[0], v1[1], v1[2], v1[3]));
    if (B16) {
      ushort4 w16; w16.x = f32_to_bf16_rne(t1[0]); w16.y = f32_to_bf16_rne(t1[1]); w16.z = f32_to_bf16_rne(t1[2]); w16.w = f32_to_bf16_rne(t1[3]);
      __builtin_nontemporal_store(__builtin_bit_cast(unsigned long long, w16), reinterpret_cast<unsigned long long*>(b16_w + bt.e));
    }
  };
  Batch ring[DEPTH];
#pragma unroll
  for (int bb = 0; bb < DEPTH - 1; ++bb) load_batch(ring[bb], bb);
#pragma unroll
  for (int bb = 0; bb < NB; ++bb) {
    const int i = bb / 8, b = bb % 8;
    if (b == 0) {
      // scatter the accumulators of tile row i (earlier reads of the region are done: same wave, program order)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = (r >> 2) * 8 + lhalf * 4 + (r & 3), col = j * 32 + l32;
          gl[row * PR + col] = acc[i][j][r];
          hl[row * PR + col] = racc[i][j][r];
        }
    }
    if (bb + DEPTH - 1 < NB) load_batch(ring[(bb + DEPTH - 1) % DEPTH], bb + DEPTH - 1);
    __builtin_amdgcn_sched_barrier(0);
    finish_batch(ring[bb % DEPTH], b);
    asm volatile("" : "+v"(nsum));                          // the batch's terms are summed here, not kept for later
    __builtin_amdgcn_sched_barrier(0);
  }
  return nsum;
}

// One of several Hutchinson probes that is not the last: only z*Hz of the wave's tile is kept, added to (first
// probe: stored as) the running sum f.dacc; the parameters and moments are not touched.  Same LDS staging and
// 256-byte rows as above; racc, gl, wbase, ldc, row_base, col_base, zrow, lane as above.
template <int TM>
__device__ __forceinline__ void fused_probe_sum_wave_tile(const fu_floatx16 (&racc)[TM][2], float* gl, const FuseArgs& f,
                                                          int64_t wbase, int ldc, int row_base, int col_base,
                                                          const uint32_t* zrow, int lane) {
  const int l32 = lane & 31, lhalf = lane >> 5;
  constexpr int PR = 72;
  float* dacc_w = f.dacc + wbase;
  const int brow = lane >> 4, bcol = (lane & 15) * 4;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) gl[((r >> 2) * 8 + lhalf * 4 + (r & 3)) * PR + j * 32 + l32] = racc[i][j][r];
    uint32_t e[8], zw[8];
    float4 dd[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      e[b] = (uint32_t)(row_base + i * 32 + b * 4 + brow) * (uint32_t)ldc + (uint32_t)(col_base + bcol);
      zw[b] = zrow[e[b] >> 5];
      dd[b] = f.first ? make_float4(0.f, 0.f, 0.f, 0.f) : nt_load4(dacc_w + e[b]);
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const float4 h4 = *reinterpret_cast<const float4*>(gl + (b * 4 + brow) * PR + bcol);
      const uint32_t zb4 = zw[b] >> (e[b] & 31u);
      float4 o;
      o.x = dd[b].x + ((zb4 & 1u) ? h4.x : -h4.x); o.y = dd[b].y + ((zb4 & 2u) ? h4.y : -h4.y);
      o.z = dd[b].z + ((zb4 & 4u) ? h4.z : -h4.z); o.w = dd[b].w + ((zb4 & 8u) ? h4.w : -h4.w);
      nt_store4(dacc_w + e[b], o);
    }
  }
}

}  // namespace dw
