// Epilogue helper of the bf16 dual GEMMs: one wave's row of MFMA tiles (32 rows x TN*32 columns) of the two
// bf16 outputs C and RC is written to memory through a wave-private LDS region.
//
// The MFMA layout gives a lane one column and 16 rows, i.e. 2-byte stores of 64-byte row pieces.  Going through
// LDS ([row][TN*32 bf16 + 8] per output, conflict-free for the scatter) turns them into 16-byte stores, each
// instruction covering whole row pieces of the wave's tile (TN*64 bytes), and the ReLU mask of the data gradient
// into 16-byte loads.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dw_device_util.h"

namespace dw {

typedef float epi_floatx16 __attribute__((ext_vector_type(16)));

// 0xFFFF for each 16-bit half of m2 that holds a bf16 value > 0 (stored activation of a unit that is on)
__device__ __forceinline__ uint32_t epi_keep(uint32_t m2) {
  const uint32_t lo = m2 & 0xFFFFu, hi = m2 >> 16;
  return ((lo != 0 && !(lo & 0x8000u)) ? 0x0000FFFFu : 0u) | ((hi != 0 && !(hi & 0x8000u)) ? 0xFFFF0000u : 0u);
}

constexpr int epi_bf16_lds_bytes(int tn) { return 2 * 32 * (tn * 64 + 16); }     // per wave

// cv, rcv: the TN accumulator tiles of the row, already with bias / activation applied (fp32)
// out0: element offset of the tile row's first element in C and RC; rows_left, cols_left: valid extent from there
// MASK: keep an element only where mask[msk0 + row*ld_mask + col] > 0 (same shape as the outputs)
// STORE_C = false: only RC is written (cv is not read)
template <int TN, bool MASK, bool STORE_C = true>
__device__ __forceinline__ void epi_bf16_rows_out(char* wl, const epi_floatx16* cv, const epi_floatx16* rcv, int lane,
                                                  uint16_t* C, uint16_t* RC, int64_t out0, int ldc, int rows_left,
                                                  int cols_left, const uint16_t* msk, int64_t msk0, int ld_mask) {
  constexpr int RS = TN * 64 + 16;                            // bytes per LDS row
  const int l32 = lane & 31, lhalf = lane >> 5;
  char* wr = wl + 32 * RS;
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int off = ((r >> 2) * 8 + lhalf * 4 + (r & 3)) * RS + (j * 32 + l32) * 2;
      if (STORE_C) *reinterpret_cast<uint16_t*>(wl + off) = f32_to_bf16_rne(cv[j][r]);
      *reinterpret_cast<uint16_t*>(wr + off) = f32_to_bf16_rne(rcv[j][r]);
    }
  constexpr int LPR = TN * 4, RPP = 64 / LPR;                 // lanes per row, rows per pass
  const int prow = lane / LPR, ch = lane % LPR;
#pragma unroll
  for (int p = 0; p < 32 / RPP; ++p) {
    const int row = p * RPP + prow;
    uint4 v = STORE_C ? *reinterpret_cast<const uint4*>(wl + row * RS + ch * 16) : make_uint4(0u, 0u, 0u, 0u);
    uint4 rv = *reinterpret_cast<const uint4*>(wr + row * RS + ch * 16);
    if (row < rows_left && ch * 8 < cols_left) {
      if (MASK) {
        const uint4 mv = *reinterpret_cast<const uint4*>(msk + msk0 + (int64_t)row * ld_mask + ch * 8);
        const uint32_t k0 = epi_keep(mv.x), k1 = epi_keep(mv.y), k2 = epi_keep(mv.z), k3 = epi_keep(mv.w);
        v.x &= k0; v.y &= k1; v.z &= k2; v.w &= k3;
        rv.x &= k0; rv.y &= k1; rv.z &= k2; rv.w &= k3;
      }
      if (STORE_C) *reinterpret_cast<uint4*>(C + out0 + (int64_t)row * ldc + ch * 8) = v;
      *reinterpret_cast<uint4*>(RC + out0 + (int64_t)row * ldc + ch * 8) = rv;
    }
  }
}

}  // namespace dw
