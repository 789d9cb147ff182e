// fp32 output layer and softmax head in one kernel.
//
// S = A W^T + b and RS = RA W^T + A V^T + c (Section IV-B) with W [C][K], C <= 16 classes, followed at once by the
// softmax cross-entropy of the rows and its R-derivative (dw_head_math.h): the logits never go to memory.  For the
// small models this replaces three short launches in a row (a product with a handful of tiles, the sum of its slices,
// the head) by one.  A block owns 16 samples; its four waves take a quarter of the contraction each with the
// 16 x 16 x 4 MFMA, every lane loading 16 bytes (4 consecutive k) of A, RA and W per step, and the four partial tiles
// are added in wave order through LDS.  A 16-lane group then holds one sample's 16 logits, gathers them by shuffles
// and runs the head's arithmetic on them.  The loss of the block's samples goes to one slot per (worker, block);
// loss_sum_kernel adds a worker's slots in index order when the caller wants the loss.
#include "dw_internal.h"
#include "dw_head_math.h"

namespace dw {

typedef float f32o_x4 __attribute__((ext_vector_type(4)));

namespace f32o {

constexpr int ROWS = 16, NT = 256, NW = NT / 64, KSTEP = 16;
static_assert(DW_MAX_CLASSES == ROWS, "a 16-lane group holds one sample's logits, one class per lane");

// grid: (ceil(M / 16), active workers); requirements in out_head_f32_ok
__global__ __launch_bounds__(NT) void out_head_f32_kernel(GemmArgs a, HeadArgs h, float* loss_part) {
  const int worker = nth_active_worker(a.active_mask, blockIdx.y);
  const int row0 = blockIdx.x * ROWS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r16 = lane & 15, kg = lane >> 4;               // operand row (A) or column (W), and which 4 of the 16 k
  const int kspan = a.K / NW;                              // this wave's share of the contraction
  const int kbeg = wave * kspan;
  const int arow = row0 + r16 < a.M ? row0 + r16 : a.M - 1;   // rows past the end repeat the last one (never stored)

  const float* X = reinterpret_cast<const float*>(a.X) + (int64_t)worker * a.x_wstride + (int64_t)arow * a.ldx + kg * 4;
  const bool has_rx = a.RX != nullptr;
  const float* RX = has_rx ? reinterpret_cast<const float*>(a.RX) + (int64_t)worker * a.x_wstride + (int64_t)arow * a.ldx + kg * 4
                           : X;
  const bool col_ok = r16 < a.N;
  const int wrow = col_ok ? r16 : 0;                       // lanes of padding columns read row 0 and multiply by zero
  const float* W = reinterpret_cast<const float*>(a.Y) + (int64_t)worker * a.y_wstride + (int64_t)wrow * a.ldy + kg * 4;
  const uint32_t* zb = a.zbits + (int64_t)worker * a.z_stride;
  const int64_t zbit0 = a.z_off + (int64_t)wrow * a.ldy + kg * 4;    // multiple of 4: the 4 bits sit in one word

  f32o_x4 acc = {0.f, 0.f, 0.f, 0.f}, racc = {0.f, 0.f, 0.f, 0.f};

  for (int k0 = kbeg; k0 < kbeg + kspan; k0 += KSTEP) {
    const float4 x4 = *reinterpret_cast<const float4*>(X + k0);
    const float4 rx4 = has_rx ? *reinterpret_cast<const float4*>(RX + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 w4 = col_ok ? *reinterpret_cast<const float4*>(W + k0) : make_float4(0.f, 0.f, 0.f, 0.f);
    const int64_t bi = zbit0 + k0;
    const uint32_t bits = col_ok ? (zb[bi >> 5] >> (bi & 31)) & 0xFu : 0u;
    const float x[4] = {x4.x, x4.y, x4.z, x4.w}, rx[4] = {rx4.x, rx4.y, rx4.z, rx4.w}, w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float v = col_ok ? (((bits >> j) & 1u) ? 1.f : -1.f) : 0.f;
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x[j], w[j], acc, 0, 0, 0);
      racc = __builtin_amdgcn_mfma_f32_16x16x4f32(rx[j], w[j], racc, 0, 0, 0);
      racc = __builtin_amdgcn_mfma_f32_16x16x4f32(x[j], v, racc, 0, 0, 0);
    }
  }

  // partial tiles of the four waves: element (row, col) of a wave sits in lane col + 16*(row/4), register row%4
  __shared__ float part[NW][2][ROWS][ROWS + 1];
  __shared__ float row_loss[ROWS];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    part[wave][0][kg * 4 + r][r16] = acc[r];
    part[wave][1][kg * 4 + r][r16] = racc[r];
  }
  __syncthreads();
  const int m = tid >> 4, n = tid & 15;                   // one 16-lane group per sample, one lane per class
  float s = 0.f, rs = 0.f;
  if (n < a.N) {
#pragma unroll
    for (int w = 0; w < NW; ++w) { s += part[w][0][m][n]; rs += part[w][1][m][n]; }
    const int64_t bi = a.zb_off + n;
    s += a.bias[(int64_t)worker * a.bias_wstride + n];
    rs += ((zb[bi >> 5] >> (bi & 31)) & 1u) ? 1.f : -1.f;
  }
  // every lane of the group gathers the sample's logits and runs the head on them; it keeps its own class
  float sv[DW_MAX_CLASSES], rsv[DW_MAX_CLASSES], d[DW_MAX_CLASSES], rd[DW_MAX_CLASSES];
  const int base = lane & 48;
#pragma unroll
  for (int c = 0; c < DW_MAX_CLASSES; ++c) { sv[c] = __shfl(s, base + c); rsv[c] = __shfl(rs, base + c); }
  const int row = row0 + m;
  const int yrow = row < a.M ? row : a.M - 1;
  const int y = h.y[(int64_t)worker * h.B + yrow];
  const float lrow = head_row(sv, rsv, y, h.C, 1.0f / (float)h.B, d, rd);
  float dn = 0.f, rdn = 0.f;
#pragma unroll
  for (int c = 0; c < DW_MAX_CLASSES; ++c) { if (c == n) { dn = d[c]; rdn = rd[c]; } }
  if (row < a.M && n < h.ld) {
    const int64_t o = ((int64_t)worker * h.B + row) * h.ld + n;
    h.delta[o] = dn;
    h.Rdelta[o] = rdn;
  }
  if (n == 0) row_loss[m] = row < a.M ? lrow : 0.f;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
#pragma unroll
    for (int r = 0; r < ROWS; ++r) t += row_loss[r];
    loss_part[(int64_t)worker * gridDim.x + blockIdx.x] = t;
  }
}

// loss[i] = (sum of worker i's slots, in index order) / B
__global__ __launch_bounds__(64) void loss_sum_kernel(const float* loss_part, int n_slots, float* loss, int k, int B,
                                                      uint64_t active_mask) {
  const int i = threadIdx.x;
  if (i >= k || !((active_mask >> i) & 1ull)) return;
  float t = 0.f;
  for (int b = 0; b < n_slots; ++b) t += loss_part[(int64_t)i * n_slots + b];
  loss[i] = t / (float)B;
}

}  // namespace f32o

// the fp32 output layer's forward product (linear epilogue, at most 16 columns) with a contraction that four waves
// can share in steps of 16, operands that 16-byte loads can address and sign bits that come four to a word
bool out_head_f32_ok(const GemmArgs& a) {
  if (a.epi != EPI_LINEAR || !a.ry_bits || !a.x_kcontig || !a.y_kcontig || a.ksplit > 1) return false;
  if (a.N < 1 || a.N > f32o::ROWS || a.M < 1) return false;
  if (a.K < f32o::NW * f32o::KSTEP || a.K % (f32o::NW * f32o::KSTEP) != 0) return false;
  if (a.ldx % 4 != 0 || a.ldy % 4 != 0 || a.x_wstride % 4 != 0 || a.y_wstride % 4 != 0 || a.z_off % 4 != 0) return false;
  if ((reinterpret_cast<uintptr_t>(a.X) & 15u) || (reinterpret_cast<uintptr_t>(a.Y) & 15u) ||
      (a.RX && (reinterpret_cast<uintptr_t>(a.RX) & 15u)))
    return false;
  return true;
}

// loss_part: at least k * ceil(M / 16) floats; h.loss may be nullptr (then the slots are not added up)
hipError_t launch_out_head_f32(const GemmArgs& a, const HeadArgs& h, float* loss_part, hipStream_t s) {
  KernelScope ks(KC_HEAD, s);
  const int n_slots = (a.M + f32o::ROWS - 1) / f32o::ROWS;
  const dim3 grid((unsigned)n_slots, (unsigned)active_count(a.active_mask, a.k));
  hipLaunchKernelGGL(f32o::out_head_f32_kernel, grid, dim3(f32o::NT), 0, s, a, h, loss_part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !h.loss) return e;
  hipLaunchKernelGGL(f32o::loss_sum_kernel, dim3(1), dim3(64), 0, s, loss_part, n_slots, h.loss, a.k, h.B, a.active_mask);
  return hipGetLastError();
}

}  // namespace dw
