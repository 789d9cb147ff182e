// bf16 dual GEMM of the output layer's forward pass: few columns (the classes), long contraction.
//
// S = A W^T + b and RS = RA W^T + A V^T + c (Section IV-B) with W [C][K], C <= 16: the product is a stream over the
// activations A and RA ([B][K] bf16 each); W and the sign bits of V are tiny and stay in cache.  A tile kernel gives
// this shape only B/256 blocks per worker, each walking the whole K with one tile in flight.  Here a block owns 16
// rows and its four waves a quarter of K each, every lane keeping eight 16-byte loads of A and of RA in flight;
// the 16 x 16 x 32 MFMA takes the lanes' loads as they come (8 consecutive k per lane, no LDS), and the four
// partial tiles are added in wave order through LDS, so the result does not depend on timing.
#include "dw_internal.h"

namespace dw {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace b16o {

constexpr int ROWS = 16, NT = 256, NW = NT / 64, KSTEP = 32, UNROLL = 8;

__device__ __forceinline__ uint32_t pm1_pair(uint32_t b_lo, uint32_t b_hi) {
  return 0xBF80BF80u ^ (b_lo << 15) ^ (b_hi << 31);     // bit set -> +1 (0x3F80), clear -> -1 (0xBF80)
}
__device__ __forceinline__ bf16x8 pm1_x8(uint32_t b) {
  uint4 o;
  o.x = pm1_pair(b & 1u, (b >> 1) & 1u); o.y = pm1_pair((b >> 2) & 1u, (b >> 3) & 1u);
  o.z = pm1_pair((b >> 4) & 1u, (b >> 5) & 1u); o.w = pm1_pair((b >> 6) & 1u, (b >> 7) & 1u);
  return __builtin_bit_cast(bf16x8, o);
}

// grid: (M / 16, active workers); requirements in gemm_bf16_out_ok
__global__ __launch_bounds__(NT) void out_layer_fwd_bf16(GemmArgs a) {
  const int worker = nth_active_worker(a.active_mask, blockIdx.y);
  const int row0 = blockIdx.x * ROWS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;              // operand row (A) or column (W), and which 8 of the 32 k
  const int kspan = a.K / NW;                             // this wave's share of the contraction
  const int kbeg = wave * kspan;

  const uint16_t* X = reinterpret_cast<const uint16_t*>(a.X) + (int64_t)worker * a.x_wstride +
                      (int64_t)(row0 + r16) * a.ldx + kg * 8;
  const uint16_t* RX = reinterpret_cast<const uint16_t*>(a.RX) + (int64_t)worker * a.x_wstride +
                       (int64_t)(row0 + r16) * a.ldx + kg * 8;
  const bool col_ok = r16 < a.N;
  const int wrow = col_ok ? r16 : 0;                      // lanes of padding columns read row 0 and multiply by zero
  const uint16_t* W = reinterpret_cast<const uint16_t*>(a.Y) + (int64_t)worker * a.y_wstride + (int64_t)wrow * a.ldy + kg * 8;
  const uint32_t* zb = a.zbits + (int64_t)worker * a.z_stride;
  const int64_t zbit0 = a.z_off + (int64_t)wrow * a.ldy + kg * 8;   // multiple of 8: the 8 bits sit in one byte

  floatx4 acc = {0.f, 0.f, 0.f, 0.f}, racc = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = kbeg; k0 < kbeg + kspan; k0 += KSTEP * UNROLL) {
    u32x4 xa[UNROLL], rxa[UNROLL], wb[UNROLL];
    uint32_t zw[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int k = k0 + u * KSTEP;
      xa[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(X + k));
      rxa[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(RX + k));
      wb[u] = *reinterpret_cast<const u32x4*>(W + k);
      const int64_t bi = zbit0 + k;
      zw[u] = (zb[bi >> 5] >> (bi & 31)) & 0xFFu;
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const bf16x8 x = __builtin_bit_cast(bf16x8, xa[u]), rx = __builtin_bit_cast(bf16x8, rxa[u]);
      const u32x4 zero = {0u, 0u, 0u, 0u};
      const bf16x8 w = __builtin_bit_cast(bf16x8, col_ok ? wb[u] : zero);
      const bf16x8 v = col_ok ? pm1_x8(zw[u]) : __builtin_bit_cast(bf16x8, zero);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, w, acc, 0, 0, 0);
      racc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rx, w, racc, 0, 0, 0);
      racc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, v, racc, 0, 0, 0);
    }
  }

  // partial tiles of the four waves: element (row, col) of a wave sits in lane col + 16*(row/4), register row%4
  __shared__ float part[NW][2][ROWS][ROWS + 1];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    part[wave][0][kg * 4 + r][r16] = acc[r];
    part[wave][1][kg * 4 + r][r16] = racc[r];
  }
  __syncthreads();
  const int m = tid >> 4, n = tid & 15;
  if (n < a.N && row0 + m < a.M) {
    float s = 0.f, rs = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) { s += part[w][0][m][n]; rs += part[w][1][m][n]; }
    const int64_t bi = a.zb_off + n;
    const float cz = ((zb[bi >> 5] >> (bi & 31)) & 1u) ? 1.f : -1.f;
    const int64_t o = (int64_t)worker * a.c_wstride + (int64_t)(row0 + m) * a.ldc + n;
    reinterpret_cast<float*>(a.C)[o] = s + a.bias[(int64_t)worker * a.bias_wstride + n];
    reinterpret_cast<float*>(a.RC)[o] = rs + cz;
  }
}

}  // namespace b16o

// the output layer's forward product (linear epilogue, at most 16 columns) with a contraction long enough to
// split over four waves in steps of 256, whole 16-row tiles, and operands that 16-byte loads can address
bool gemm_bf16_out_ok(const GemmArgs& a) {
  if (a.epi != EPI_LINEAR || !a.ry_bits || !a.RX || !a.x_kcontig || !a.y_kcontig) return false;
  if (a.N < 1 || a.N > b16o::ROWS || a.M % b16o::ROWS != 0) return false;
  if (a.K % (b16o::NW * b16o::KSTEP * b16o::UNROLL) != 0) return false;
  if (a.ldx % 8 != 0 || a.ldy % 8 != 0 || a.x_wstride % 8 != 0 || a.y_wstride % 8 != 0 || a.z_off % 8 != 0) return false;
  if ((reinterpret_cast<uintptr_t>(a.X) & 15u) || (reinterpret_cast<uintptr_t>(a.RX) & 15u) ||
      (reinterpret_cast<uintptr_t>(a.Y) & 15u))
    return false;
  return true;
}

hipError_t launch_gemm_bf16_out(const GemmArgs& a, hipStream_t s) {
  const dim3 grid((unsigned)(a.M / b16o::ROWS), (unsigned)active_count(a.active_mask, a.k));
  hipLaunchKernelGGL(b16o::out_layer_fwd_bf16, grid, dim3(b16o::NT), 0, s, a);
  return hipGetLastError();
}

}  // namespace dw
