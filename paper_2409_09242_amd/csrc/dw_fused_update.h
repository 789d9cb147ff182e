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
//
// Two Hutchinson probes in one kernel (PROBES == 2): the wave holds a second R-accumulator, the Hessian-vector
// product along the earlier probe's z, and D = (z_p*Hz_p + z*Hz) / 2 needs no running sum in memory.  That kernel
// runs 8 waves per block, so the staging region holds 16 rows of the MFMA tile row at a time (three arrays).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dw_internal.h"
#include "dw_device_util.h"

namespace dw {

typedef float fu_floatx16 __attribute__((ext_vector_type(16)));

// floats of LDS one wave needs: g and Hz of one row of MFMA tiles, [32][72] each; two probes in one kernel: g and both
// Hz of half a row of tiles, [16][72] each
__host__ __device__ constexpr int fused_update_lds_floats(bool pair = false) { return pair ? 3 * 16 * 72 : 2 * 32 * 72; }

// The update of one wave's tile.  Constructor: wbase = the worker's offset in theta, m, v (and the bf16 copy); row_base,
// col_base: first row and column of the wave's tile in W_l; zrow: sign bits of z from the first parameter of the W
// block on.  run: acc, racc = the wave's accumulators (plain product = g, R-companion = Hz), MFMA 32x32 layout: lane
// holds column lane%32 of each tile, rows (r/4)*8 + (lane/32)*4 + r%4; gl: the wave's LDS region; ib1, ib2: the
// worker's 1/(1 - beta^t).  Returns this lane's share of the squared distance of the new parameters to the centre
// (0 unless f.dist).  (Issuing the first batch's loads under the kernel's last k-tile was tried: the one-probe kernel
// has no registers for it, the two-probe kernel gains nothing.)
// B16: also store the bf16 copy of the new parameters.  PROBES = 1: the diagonal estimate is the mean over several
// Hutchinson probes, D = (f.dacc + z*Hz) * f.d_scale, f.dacc holding the sum over the earlier probes.  PROBES = 2:
// the mean over two probes, the earlier one's product in raccp and its sign bits in zrowp (both unused otherwise).
template <int TM, bool B16, int PROBES = 0, int DEPTH_ = 3>
struct FusedUpdateTile {
  static constexpr int PR = 72;                             // floats per LDS row: both half-waves hit distinct banks
  static constexpr int SR = PROBES == 2 ? 16 : 32;          // rows staged at a time
  static constexpr int SB = SR / 4;                         // batches per staging
  static constexpr int NB = TM * 8, DEPTH = DEPTH_;        // DEPTH - 1 batches of loads are in flight
  struct Batch { uint32_t e, zw, zwp; float4 th, mm, vv, cc, dd; };

  const FuseArgs& f;
  float* th_w; float* m_w; float* v_w; uint16_t* b16_w; const float* dacc_w;
  const uint32_t* zrow; const uint32_t* zrowp;
  uint32_t e0;                                              // offset of the lane's float4 of batch 0 inside the W block
  uint32_t ldc;
  int lane;
  Batch ring[DEPTH];

  __device__ __forceinline__ FusedUpdateTile(const FuseArgs& fu, int64_t wbase, int ldc_, int row_base, int col_base,
                                             const uint32_t* zrow_, const uint32_t* zrowp_, int lane_)
      : f(fu), th_w(fu.theta + wbase), m_w(fu.m + wbase), v_w(fu.v + wbase), b16_w(B16 ? fu.wb16 + wbase : nullptr),
        dacc_w(PROBES == 1 ? fu.dacc + wbase : nullptr), zrow(zrow_), zrowp(zrowp_),
        e0((uint32_t)(row_base + (lane_ >> 4)) * (uint32_t)ldc_ + (uint32_t)(col_base + (lane_ & 15) * 4)),
        ldc((uint32_t)ldc_), lane(lane_) {}

  __device__ __forceinline__ void load_batch(Batch& bt, int bb) {
    bt.e = e0 + (uint32_t)(bb * 4) * ldc;                   // a multiple of 4
    bt.th = nt_load4(th_w + bt.e); bt.mm = nt_load4(m_w + bt.e);   // the state streams through once: no reuse in L2
    bt.vv = nt_load4(v_w + bt.e);
    bt.cc = f.dist ? *reinterpret_cast<const float4*>(f.centre + bt.e) : make_float4(0.f, 0.f, 0.f, 0.f);
    bt.zw = zrow[bt.e >> 5];
    if constexpr (PROBES == 1) bt.dd = nt_load4(dacc_w + bt.e);
    if constexpr (PROBES == 2) bt.zwp = zrowp[bt.e >> 5];
  }

  // b: the batch's place in the staged rows
  __device__ __forceinline__ void finish_batch(const Batch& bt, int b, const float* gl, float ib1, float ib2, float& nsum) {
    const int brow = lane >> 4, bcol = (lane & 15) * 4;
    const float* hl = gl + SR * PR;
    const float4 g4 = *reinterpret_cast<const float4*>(gl + (b * 4 + brow) * PR + bcol);
    const float4 h4 = *reinterpret_cast<const float4*>(hl + (b * 4 + brow) * PR + bcol);
    const float g[4] = {g4.x, g4.y, g4.z, g4.w}, hz[4] = {h4.x, h4.y, h4.z, h4.w};
    const float th[4] = {bt.th.x, bt.th.y, bt.th.z, bt.th.w}, mm[4] = {bt.mm.x, bt.mm.y, bt.mm.z, bt.mm.w};
    const float vv[4] = {bt.vv.x, bt.vv.y, bt.vv.z, bt.vv.w}, cc[4] = {bt.cc.x, bt.cc.y, bt.cc.z, bt.cc.w};
    const uint32_t zb4 = bt.zw >> (bt.e & 31u);
    float D[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) D[q] = ((zb4 >> q) & 1u) ? hz[q] : -hz[q];      // Hutchinson: z * Hz
    if constexpr (PROBES == 1) {
      const float dd[4] = {bt.dd.x, bt.dd.y, bt.dd.z, bt.dd.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) D[q] = (dd[q] + D[q]) * f.d_scale;
    }
    if constexpr (PROBES == 2) {
      const float4 p4 = *reinterpret_cast<const float4*>(hl + SR * PR + (b * 4 + brow) * PR + bcol);
      const float hp[4] = {p4.x, p4.y, p4.z, p4.w};
      const uint32_t zp4 = bt.zwp >> (bt.e & 31u);
#pragma unroll
      for (int q = 0; q < 4; ++q) D[q] = ((((zp4 >> q) & 1u) ? hp[q] : -hp[q]) + D[q]) * 0.5f;
    }
    if (f.avg_block == 2) {
      const float p0 = 0.5f * (D[0] + D[1]), p1 = 0.5f * (D[2] + D[3]);
      D[0] = D[1] = p0; D[2] = D[3] = p1;
    } else if (f.avg_block >= 4) {
      const int group_lanes = f.avg_block >> 2;             // lanes that share one averaging block
      float sD = (D[0] + D[1]) + (D[2] + D[3]);
#pragma unroll
      for (int off = 1; off < 8; off <<= 1) {
        const float t = __shfl_xor(sD, off);
        sD += off < group_lanes ? t : 0.f;
      }
      sD *= 1.0f / (float)f.avg_block;
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
  }

  __device__ __forceinline__ float run(const fu_floatx16 (&acc)[TM][2], const fu_floatx16 (&racc)[TM][2],
                                       const fu_floatx16 (&raccp)[TM][2], float* gl, float ib1, float ib2) {
    const int l32 = lane & 31, lhalf = lane >> 5;
    float* hl = gl + SR * PR;
    float* hlp = hl + SR * PR;                              // (two probes)
    float nsum = 0.f;
#pragma unroll
    for (int bb = 0; bb < DEPTH - 1; ++bb) load_batch(ring[bb], bb);
#pragma unroll
    for (int bb = 0; bb < NB; ++bb) {
      const int i = bb / 8, b = bb % 8;
      if (b % SB == 0) {
        // scatter the accumulators of the next SR rows of tile row i (earlier reads of the region are done: same
        // wave, program order); accumulator r of a lane is row (r/4)*8 + (lane/32)*4 + r%4 of the tile
        constexpr int R0 = SR / 2;                          // accumulators per lane and staging
        const int r_first = (b / SB) * R0;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int rr = 0; rr < R0; ++rr) {
            const int r = r_first + rr;
            const int row = (rr >> 2) * 8 + lhalf * 4 + (rr & 3), col = j * 32 + l32;
            gl[row * PR + col] = acc[i][j][r];
            hl[row * PR + col] = racc[i][j][r];
            if constexpr (PROBES == 2) hlp[row * PR + col] = raccp[i][j][r];
          }
      }
      if (bb + DEPTH - 1 < NB) load_batch(ring[(bb + DEPTH - 1) % DEPTH], bb + DEPTH - 1);
      __builtin_amdgcn_sched_barrier(0);
      finish_batch(ring[bb % DEPTH], b % SB, gl, ib1, ib2, nsum);
      asm volatile("" : "+v"(nsum));                        // the batch's terms are summed here, not kept for later
      __builtin_amdgcn_sched_barrier(0);
    }
    return nsum;
  }
};

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
