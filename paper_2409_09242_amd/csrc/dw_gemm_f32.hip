// fp32 "dual-number" GEMM for gfx950: C = X*Y and RC = RX*Y + X*RY in one pass over the tiles.
//
// Forward and backward propagation of the MLP (Section II eq.(2)) and the propagation of their
// directional derivatives along z, which yields the Hessian-vector product Hz of the Hutchinson estimate
// (Section IV-B), all have this product-rule shape:
//   forward      s  = a W^T,            Rs  = Ra W^T + a V^T            (V = z reshaped like W)
//   data grad    d' = d W,              Rd' = Rd W + d V
//   weight grad  gW = d^T a,            HzW = Rd^T a + d^T Ra
// so one kernel template serves the three, sharing every tile load between the plain product and its
// R-companion.  The +-1 operand V is never stored as a matrix: its tile is expanded from the sign bits of
// z while the W tile is staged.
//
// Tiling: 256 threads = 4 waves; block tile BM x BN x 16; tiles are staged k-major in LDS so that each
// lane's MFMA operand (v_mfma_f32_32x32x2_f32: lane l supplies A[l%32][l/32] and B[l/32][l%32]) is one
// conflict-free 32-bit LDS read; global loads are 16-byte and prefetched into registers one tile ahead.
#include <cstddef>

#include "dw_internal.h"
#include "dw_fused_update.h"

namespace dw {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;
constexpr int PAD = 4;
constexpr int NT = 256;

enum RyMode { RY_NONE = 0, RY_MEM = 1, RY_BITS = 2 };

template <int ROWS>                      // ROWS = extent of the non-contraction index in the tile (BM or BN)
struct TileLoader {
  static constexpr int CNT = ROWS * BK / 4;            // float4 per tile
  static constexpr int NL = (CNT + NT - 1) / NT;       // float4 per thread

  // position of float4 number idx inside the tile: (r = non-contraction index, kk = contraction index)
  template <bool KC>
  __device__ static __forceinline__ void pos(int idx, int& r, int& kk) {
    if (KC) { r = idx / (BK / 4); kk = (idx % (BK / 4)) * 4; }      // 4 consecutive kk at one r
    else    { kk = idx / (ROWS / 4); r = (idx % (ROWS / 4)) * 4; }  // 4 consecutive r at one kk
  }

  // Element offset of the float4 at row `row` (non-contraction index), contraction index `kq` of the operand, and
  // whether it exists: a matrix in memory (ld), or a view of a map (see OperandView)
  template <bool KC, int VIEW>
  __device__ static __forceinline__ int64_t offset(int row, int kq, int ld, const ConvView& cv, bool& ok) {
    if (VIEW == VIEW_NONE) return KC ? (int64_t)row * ld + kq : (int64_t)kq * ld + row;
    // the operand's own (row, column) whichever of them the product contracts
    const int mrow = KC ? row : kq, col = KC ? kq : row;
    if (VIEW == VIEW_PATCH) {
      const int Wo = cv.W - 2, Ho = cv.H - 2;
      const int x = mrow % Wo, t = mrow / Wo, y = t % Ho, b = t / Ho;
      const int tap = col / cv.Cin, ci = col - tap * cv.Cin, dy = tap / 3, dx = tap - dy * 3;
      return (((int64_t)b * cv.H + (y + dy)) * cv.W + (x + dx)) * cv.Cin + ci;
    }
    if (VIEW == VIEW_SHIFTED) {
      const int Wo = cv.W - 2, Ho = cv.H - 2;
      const int xx = mrow % cv.W, t = mrow / cv.W, yy = t % cv.H, b = t / cv.H;
      const int tap = col / cv.Cout, co = col - tap * cv.Cout, dy = tap / 3, dx = tap - dy * 3;
      const int y = yy - dy, x = xx - dx;
      ok = ok && y >= 0 && y < Ho && x >= 0 && x < Wo;
      return (((int64_t)b * Ho + y) * Wo + x) * cv.Cout + co;
    }
    // VIEW_TAPS: operand row = tap*Cout + co (the contraction index of the data gradient), column = ci
    const int tap = mrow / cv.Cout, co = mrow - tap * cv.Cout;
    return (int64_t)co * (9 * cv.Cin) + tap * cv.Cin + col;
  }

  template <bool KC, int VIEW = VIEW_NONE>
  __device__ static __forceinline__ void load(const float* __restrict__ src, int ld, int r0, int k0, int R, int K,
                                              float4 (&reg)[NL], const ConvView& cv = ConvView{}) {
#pragma unroll
    for (int it = 0; it < NL; ++it) {
      const int idx = it * NT + (int)threadIdx.x;
      int r, kk; pos<KC>(idx, r, kk);
      bool ok = idx < CNT && (r0 + r) < R && (k0 + kk) < K;
      const int64_t off = ok ? offset<KC, VIEW>(r0 + r, k0 + kk, ld, cv, ok) : 0;
      reg[it] = ok ? *reinterpret_cast<const float4*>(src + off) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }

  // sign bits of the four elements that load<KC> would read (0 when out of range)
  template <bool KC, int VIEW = VIEW_NONE>
  __device__ static __forceinline__ void load_bits(const uint32_t* __restrict__ zb, int64_t z_off, int ld, int r0,
                                                   int k0, int R, int K, uint32_t (&reg)[NL], const ConvView& cv = ConvView{}) {
#pragma unroll
    for (int it = 0; it < NL; ++it) {
      const int idx = it * NT + (int)threadIdx.x;
      int r, kk; pos<KC>(idx, r, kk);
      bool ok = idx < CNT && (r0 + r) < R && (k0 + kk) < K;
      const int64_t off = z_off + (ok ? offset<KC, VIEW>(r0 + r, k0 + kk, ld, cv, ok) : 0);
      reg[it] = ok ? (zb[off >> 5] >> (off & 31)) & 0xFu : 0u;
    }
  }

  template <bool KC>
  __device__ static __forceinline__ void store(float (*lds)[ROWS + PAD], const float4 (&reg)[NL]) {
#pragma unroll
    for (int it = 0; it < NL; ++it) {
      const int idx = it * NT + (int)threadIdx.x;
      if (idx < CNT) {
        int r, kk; pos<KC>(idx, r, kk);
        if (KC) {
          lds[kk + 0][r] = reg[it].x; lds[kk + 1][r] = reg[it].y;
          lds[kk + 2][r] = reg[it].z; lds[kk + 3][r] = reg[it].w;
        } else {
          *reinterpret_cast<float4*>(&lds[kk][r]) = reg[it];
        }
      }
    }
  }

  template <bool KC>
  __device__ static __forceinline__ void store_bits(float (*lds)[ROWS + PAD], const uint32_t (&reg)[NL]) {
#pragma unroll
    for (int it = 0; it < NL; ++it) {
      const int idx = it * NT + (int)threadIdx.x;
      if (idx < CNT) {
        int r, kk; pos<KC>(idx, r, kk);
        float4 v;
        v.x = (reg[it] & 1u) ? 1.f : -1.f; v.y = (reg[it] & 2u) ? 1.f : -1.f;
        v.z = (reg[it] & 4u) ? 1.f : -1.f; v.w = (reg[it] & 8u) ? 1.f : -1.f;
        if (KC) {
          lds[kk + 0][r] = v.x; lds[kk + 1][r] = v.y; lds[kk + 2][r] = v.z; lds[kk + 3][r] = v.w;
        } else {
          *reinterpret_cast<float4*>(&lds[kk][r]) = v;
        }
      }
    }
  }
};

// XV, YV: OperandView of X/RX and of Y/RY (convolutions without a patch matrix in memory)
template <int BM, int BN, int WM, int WN, bool X_KC, bool Y_KC, bool HAS_RX, int RYM, int EPI, int FM = 0, int XV = VIEW_NONE,
          int YV = VIEW_NONE>
__global__ __launch_bounds__(NT) void dual_gemm_f32(GemmArgs a) {
  static_assert(WM * WN == 4, "four waves per block");
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");
  const int worker = nth_active_worker(a.active_mask, blockIdx.y);    // grid y covers the active workers

  const int tiles_m = (a.M + BM - 1) / BM;
  const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
  const int row0 = tm * BM, col0 = tn * BN;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm0 = (wave % WM) * (BM / WM), wn0 = (wave / WM) * (BN / WN);
  const int l32 = lane & 31, lhalf = lane >> 5;

  __shared__ __attribute__((aligned(16))) float Xs[BK][BM + PAD];
  __shared__ __attribute__((aligned(16))) float RXs[HAS_RX ? BK : 1][BM + PAD];
  __shared__ __attribute__((aligned(16))) float Ys[BK][BN + PAD];
  __shared__ __attribute__((aligned(16))) float RYs[RYM != RY_NONE ? BK : 1][BN + PAD];

  const float* X = reinterpret_cast<const float*>(a.X) + (int64_t)worker * a.x_wstride;
  const float* RX = HAS_RX ? reinterpret_cast<const float*>(a.RX) + (int64_t)worker * a.x_wstride : nullptr;
  const float* Y = reinterpret_cast<const float*>(a.Y) + (int64_t)worker * a.y_wstride;
  const float* RY = RYM == RY_MEM ? reinterpret_cast<const float*>(a.RY) + (int64_t)worker * a.y_wstride : nullptr;
  const uint32_t* zb = a.zbits + (int64_t)worker * a.z_stride;

  using LX = TileLoader<BM>;
  using LY = TileLoader<BN>;
  float4 xr[LX::NL], rxr[LX::NL], yr[LY::NL], ryr[LY::NL];
  uint32_t zr[LY::NL];

  floatx16 acc[TM][TN], racc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0.f; racc[i][j][r] = 0.f; }

  float gb_acc = 0.f, hzb_acc = 0.f;     // EPI_WGRAD: column sums of X and RX (bias gradients)

  // the slice of the contraction this block covers (all of it unless the weight gradient is cut along k)
  const bool sliced = (EPI == EPI_WGRAD || EPI == EPI_RELU || EPI == EPI_LINEAR || EPI == EPI_MASK) && a.ksplit > 1;
  const int kchunk = sliced ? ((a.K + a.ksplit - 1) / a.ksplit + BK - 1) / BK * BK : a.K;
  const int kbeg = sliced ? (int)blockIdx.z * kchunk : 0;
  const int kend = sliced ? (kbeg + kchunk < a.K ? kbeg + kchunk : a.K) : a.K;
  const int nkt = kend > kbeg ? (kend - kbeg + BK - 1) / BK : 0;
  auto fetch = [&](int kt) {
    const int k0 = kbeg + kt * BK;
    LX::template load<X_KC, XV>(X, a.ldx, row0, k0, a.M, kend, xr, a.cv);
    if (HAS_RX) LX::template load<X_KC, XV>(RX, a.ldx, row0, k0, a.M, kend, rxr, a.cv);
    LY::template load<Y_KC, YV>(Y, a.ldy, col0, k0, a.N, kend, yr, a.cv);
    if (RYM == RY_MEM) LY::template load<Y_KC, YV>(RY, a.ldy, col0, k0, a.N, kend, ryr, a.cv);
    if (RYM == RY_BITS) LY::template load_bits<Y_KC, YV>(zb, a.z_off, a.ldy, col0, k0, a.N, kend, zr, a.cv);
  };

  if (nkt > 0) fetch(0);
  for (int kt = 0; kt < nkt; ++kt) {
    LX::template store<X_KC>(Xs, xr);
    if (HAS_RX) LX::template store<X_KC>(RXs, rxr);
    LY::template store<Y_KC>(Ys, yr);
    if (RYM == RY_MEM) LY::template store<Y_KC>(RYs, ryr);
    if (RYM == RY_BITS) LY::template store_bits<Y_KC>(RYs, zr);
    __syncthreads();
    if (kt + 1 < nkt) fetch(kt + 1);

    if ((EPI == EPI_WGRAD || EPI == EPI_WGRAD_FUSED) && tn == 0 && (int)threadIdx.x < BM) {
#pragma unroll
      for (int kk = 0; kk < BK; ++kk) {
        gb_acc += Xs[kk][threadIdx.x];
        if (HAS_RX) hzb_acc += RXs[kk][threadIdx.x];
      }
    }

#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const int ks = kk + lhalf;
      float xa[TM], rxa[TM], yb[TN], ryb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        xa[i] = Xs[ks][wm0 + i * 32 + l32];
        if (HAS_RX) rxa[i] = RXs[ks][wm0 + i * 32 + l32];
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        yb[j] = Ys[ks][wn0 + j * 32 + l32];
        if (RYM != RY_NONE) ryb[j] = RYs[ks][wn0 + j * 32 + l32];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          // (a Hutchinson probe before the last, FM == 1, only needs the R-products)
          if (FM != 1) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[i], yb[j], acc[i][j], 0, 0, 0);
          if (HAS_RX) racc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(rxa[i], yb[j], racc[i][j], 0, 0, 0);
          if (RYM != RY_NONE) racc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(xa[i], ryb[j], racc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();
  }

  if constexpr (EPI == EPI_WGRAD_FUSED) {
    // The update of Section IV-B applied to the tile instead of storing gW and HzW (see dw_fused_update.h): whole
    // 128 x 128 tiles, wave tiles of 64 x 64; a private LDS region per wave (dynamic shared memory; the operand
    // tiles above are static).
    static_assert(TM == 2 && TN == 2, "four waves of 64 x 64");
    extern __shared__ __attribute__((aligned(16))) float fused_lds[];
    const FuseArgs& f = a.fu;
    typedef const char __attribute__((address_space(4)))* karg_bytes;
    typedef const float __attribute__((address_space(4)))* karg_floats;
    const karg_bytes ka = (karg_bytes)__builtin_amdgcn_kernarg_segment_ptr();
    const karg_floats bc = (karg_floats)(ka + offsetof(GemmArgs, fu) + offsetof(FuseArgs, sc));
    const float ib1 = bc[worker], ib2 = bc[DW_MAX_K + worker];    // scalar loads from the kernel-argument block
    static_assert(offsetof(UpdateScalars, inv_bc2) == DW_MAX_K * sizeof(float), "inv_bc2 follows inv_bc1");
    // FM: 0 one Hutchinson probe; 1 a probe before the last (only the running sum of z*Hz is written); 2 the last
    // of several probes
    float nsum = 0.f;
    if constexpr (FM == 1)
      fused_probe_sum_wave_tile<TM>(racc, fused_lds + wave * fused_update_lds_floats(), f, (int64_t)worker * a.c_wstride,
                                    a.ldc, row0 + wm0, col0 + wn0, zb + (a.z_off >> 5), lane);
    else {
      FusedUpdateTile<TM, false, FM == 2 ? 1 : 0> upd(f, (int64_t)worker * a.c_wstride, a.ldc, row0 + wm0, col0 + wn0,
                                                     zb + (a.z_off >> 5), nullptr, lane);
      nsum = upd.run(acc, racc, racc, fused_lds + wave * fused_update_lds_floats(), ib1, ib2);
    }
    double ws = (double)nsum;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ws += __shfl_xor(ws, off);
    __shared__ double red[NT / 64];
    if (lane == 0) red[wave] = ws;
    __syncthreads();
    if (threadIdx.x == 0 && f.dist) {
      double t = 0.0;
#pragma unroll
      for (int w = 0; w < NT / 64; ++w) t += red[w];
      f.partials[(int64_t)worker * f.part_stride + f.part_base + blockIdx.x] = t;
    }
  }
  // epilogue: lane holds column n = l32 of each 32x32 tile, rows (r/4)*8 + lhalf*4 + r%4
  float* C = reinterpret_cast<float*>(a.C) + (int64_t)worker * a.c_wstride;
  float* RC = reinterpret_cast<float*>(a.RC) + (int64_t)worker * a.c_wstride;
  if (sliced) {
    C = a.part + (((int64_t)blockIdx.z * a.k + worker) * 2) * a.part_stride;
    RC = C + a.part_stride;
  }
#pragma unroll
  for (int j = 0; j < (EPI == EPI_WGRAD_FUSED ? 0 : TN); ++j) {
    const int n = col0 + wn0 + j * 32 + l32;
    const bool n_ok = n < a.N;
    float bias = 0.f, cz = 0.f;
    if ((EPI == EPI_RELU || EPI == EPI_LINEAR) && n_ok) {
      bias = a.bias[(int64_t)worker * a.bias_wstride + n];
      const int64_t bi = a.zb_off + n;
      cz = ((zb[bi >> 5] >> (bi & 31)) & 1u) ? 1.f : -1.f;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = row0 + wm0 + i * 32 + (r >> 2) * 8 + lhalf * 4 + (r & 3);
        if (!n_ok || m >= a.M) continue;
        float c = acc[i][j][r], rc = racc[i][j][r];
        const int64_t o = (int64_t)m * a.ldc + n;
        if (sliced) {                                 // raw partial products: the epilogue follows the sum of the slices
          C[o] = c; RC[o] = rc;
        } else if (EPI == EPI_RELU && FM == 1) {      // a later probe: the activation is in memory, only its R-companion is new
          RC[o] = C[o] > 0.f ? rc + cz : 0.f;
        } else if (EPI == EPI_RELU) {
          c += bias; rc += cz;
          const bool on = c > 0.f;
          C[o] = on ? c : 0.f;
          RC[o] = on ? rc : 0.f;
        } else if (EPI == EPI_LINEAR) {
          C[o] = c + bias;
          RC[o] = rc + cz;
        } else if (EPI == EPI_MASK) {
          const float* msk = reinterpret_cast<const float*>(a.mask_src) + (int64_t)worker * a.mask_wstride;
          const bool on = msk[(int64_t)m * a.ld_mask + n] > 0.f;
          if (FM != 1) C[o] = on ? c : 0.f;           // (a later probe: the plain data gradient is in memory already)
          RC[o] = on ? rc : 0.f;
        } else {
          C[o] = c;
          RC[o] = rc;
        }
      }
    }
  }
  if ((EPI == EPI_WGRAD || EPI == EPI_WGRAD_FUSED) && tn == 0 && (int)threadIdx.x < BM) {
    const int m = row0 + threadIdx.x;
    if (m < a.M) {
      if (sliced) {
        float* pb = a.part_b + (((int64_t)blockIdx.z * a.k + worker) * 2) * a.M;
        pb[m] = gb_acc; pb[a.M + m] = hzb_acc;
      } else {
        a.gb[(int64_t)worker * a.c_wstride + m] = gb_acc;
        a.hzb[(int64_t)worker * a.c_wstride + m] = hzb_acc;
      }
    }
  }
}

// adds the slices of a product cut along its contraction, in slice order, and applies the epilogue the main kernel
// left out: C, RC (M rows of ldc, columns < N) and, for a weight gradient, the bias sums gb, hzb (M)
__global__ __launch_bounds__(256) void sum_slices_kernel(GemmArgs a) {
  const int worker = nth_active_worker(a.active_mask, blockIdx.y);
  const int64_t n_out = (int64_t)a.M * a.ldc;
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int n = (int)(e % a.ldc);
  if (e < n_out && n < a.N) {
    float c = 0.f, rc = 0.f;
    for (int sl = 0; sl < a.ksplit; ++sl) {
      const float* p = a.part + (((int64_t)sl * a.k + worker) * 2) * a.part_stride;
      c += p[e]; rc += p[a.part_stride + e];
    }
    if (a.epi == EPI_RELU || a.epi == EPI_LINEAR) {
      const uint32_t* zb = a.zbits + (int64_t)worker * a.z_stride;
      const int64_t bi = a.zb_off + n;
      c += a.bias[(int64_t)worker * a.bias_wstride + n];
      rc += ((zb[bi >> 5] >> (bi & 31)) & 1u) ? 1.f : -1.f;
      if (a.epi == EPI_RELU && !(c > 0.f)) { c = 0.f; rc = 0.f; }
    } else if (a.epi == EPI_MASK) {
      const float* msk = reinterpret_cast<const float*>(a.mask_src) + (int64_t)worker * a.mask_wstride;
      if (!(msk[(e / a.ldc) * a.ld_mask + n] > 0.f)) { c = 0.f; rc = 0.f; }
    }
    reinterpret_cast<float*>(a.C)[(int64_t)worker * a.c_wstride + e] = c;
    reinterpret_cast<float*>(a.RC)[(int64_t)worker * a.c_wstride + e] = rc;
  }
  if (a.epi == EPI_WGRAD && e < a.M) {
    float b = 0.f, rb = 0.f;
    for (int sl = 0; sl < a.ksplit; ++sl) {
      const float* p = a.part_b + (((int64_t)sl * a.k + worker) * 2) * a.M;
      b += p[e]; rb += p[a.M + e];
    }
    a.gb[(int64_t)worker * a.c_wstride + e] = b;
    a.hzb[(int64_t)worker * a.c_wstride + e] = rb;
  }
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_shape(const GemmArgs& a, hipStream_t s) {
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  const bool sliced = (a.epi == EPI_WGRAD || a.epi == EPI_RELU || a.epi == EPI_LINEAR || a.epi == EPI_MASK) && a.ksplit > 1;
  const dim3 grid((unsigned)tiles, (unsigned)active_count(a.active_mask, a.k), (unsigned)(sliced ? a.ksplit : 1)), block(NT);
#define DW_LAUNCH(XKC, YKC, RX, RYM, EPI) \
  hipLaunchKernelGGL((dual_gemm_f32<BM, BN, WM, WN, XKC, YKC, RX, RYM, EPI>), grid, block, 0, s, a)
#define DW_LAUNCH_R(XKC, YKC, RX, RYM, EPI) \
  hipLaunchKernelGGL((dual_gemm_f32<BM, BN, WM, WN, XKC, YKC, RX, RYM, EPI, 1>), grid, block, 0, s, a)
#define DW_LAUNCH_V(XKC, YKC, RX, RYM, EPI, XV, YV) \
  hipLaunchKernelGGL((dual_gemm_f32<BM, BN, WM, WN, XKC, YKC, RX, RYM, EPI, 0, XV, YV>), grid, block, 0, s, a)
  const bool rx = a.RX != nullptr;
  if (a.x_view != VIEW_NONE || a.y_view != VIEW_NONE) {
    // a convolution on a map: forward (patches as X), weight gradient (patches as Y), data gradient (the gradient
    // map seen from the input positions as X, the taps of W in the contraction index)
    if (a.epi == EPI_RELU && rx && a.x_view == VIEW_PATCH && a.y_view == VIEW_NONE)
      DW_LAUNCH_V(true, true, true, RY_BITS, EPI_RELU, VIEW_PATCH, VIEW_NONE);
    else if (a.epi == EPI_WGRAD && a.RY && a.x_view == VIEW_NONE && a.y_view == VIEW_PATCH)
      DW_LAUNCH_V(false, false, true, RY_MEM, EPI_WGRAD, VIEW_NONE, VIEW_PATCH);
    else if (a.epi == EPI_MASK && a.x_view == VIEW_SHIFTED && a.y_view == VIEW_TAPS)
      DW_LAUNCH_V(true, false, true, RY_BITS, EPI_MASK, VIEW_SHIFTED, VIEW_TAPS);

    else
      return hipErrorInvalidValue;
  } else if (a.r_only && !sliced && a.epi == EPI_RELU) {
    // a later Hutchinson probe of the same minibatch: the plain product is in memory, only the R-products are computed
    if (rx) DW_LAUNCH_R(true, true, true, RY_BITS, EPI_RELU); else DW_LAUNCH_R(true, true, false, RY_BITS, EPI_RELU);
  } else if (a.r_only && !sliced && a.epi == EPI_MASK) {
    DW_LAUNCH_R(true, false, true, RY_BITS, EPI_MASK);
  } else if (a.epi == EPI_RELU) {              // forward, hidden layer
    if (rx) DW_LAUNCH(true, true, true, RY_BITS, EPI_RELU); else DW_LAUNCH(true, true, false, RY_BITS, EPI_RELU);
  } else if (a.epi == EPI_LINEAR) {            // forward, output layer
    if (rx) DW_LAUNCH(true, true, true, RY_BITS, EPI_LINEAR); else DW_LAUNCH(true, true, false, RY_BITS, EPI_LINEAR);
  } else if (a.epi == EPI_MASK) {              // data gradient
    DW_LAUNCH(true, false, true, RY_BITS, EPI_MASK);
  } else if (a.epi == EPI_PLAIN) {             // data gradient stored unmasked (the mask follows a col2im)
    DW_LAUNCH(true, false, true, RY_BITS, EPI_PLAIN);
  } else {                                     // weight gradient
    if (a.RY) DW_LAUNCH(false, false, true, RY_MEM, EPI_WGRAD); else DW_LAUNCH(false, false, true, RY_NONE, EPI_WGRAD);
  }
#undef DW_LAUNCH
#undef DW_LAUNCH_R
#undef DW_LAUNCH_V
  if (sliced) {
    const int64_t n_out = (int64_t)a.M * a.ldc;
    hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((n_out + 255) / 256), grid.y), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

// weight gradient that applies the update itself: 128 x 128 tiles, dynamic LDS for the epilogue's per-wave regions
template <int FM>
static hipError_t launch_fused_wgrad_mode(const GemmArgs& a, hipStream_t s) {
  const int tiles = (a.M / 128) * (a.N / 128);
  const dim3 grid((unsigned)tiles, (unsigned)active_count(a.active_mask, a.k)), block(NT);
  constexpr int smem = (NT / 64) * fused_update_lds_floats() * (int)sizeof(float);
  auto with_ry = dual_gemm_f32<128, 128, 2, 2, false, false, true, RY_MEM, EPI_WGRAD_FUSED, FM>;
  auto without_ry = dual_gemm_f32<128, 128, 2, 2, false, false, true, RY_NONE, EPI_WGRAD_FUSED, FM>;
  static LdsLimitOnce lim_with, lim_without;
  hipError_t e = lim_with.raise(reinterpret_cast<const void*>(with_ry), smem);
  if (e == hipSuccess) e = lim_without.raise(reinterpret_cast<const void*>(without_ry), smem);
  if (e != hipSuccess) return e;
  if (a.RY) hipLaunchKernelGGL(with_ry, grid, block, smem, s, a);
  else hipLaunchKernelGGL(without_ry, grid, block, smem, s, a);
  return hipGetLastError();
}

// several Hutchinson probes: own instances for the probes before the last and for the last one
static hipError_t launch_fused_wgrad(const GemmArgs& a, hipStream_t s) {
  if (a.fu.probe_mode == 1) return launch_fused_wgrad_mode<1>(a, s);
  if (a.fu.probe_mode == 2) return launch_fused_wgrad_mode<2>(a, s);
  return launch_fused_wgrad_mode<0>(a, s);
}

// The fp32 weight-gradient product of W[n_out][n_in] can apply the update in its epilogue when W is made of whole
// 128 x 128 tiles that fill the chip, an averaging block is at most 32 and the Hessian power is 1.
bool gemm_f32_wgrad_fusable(int n_out, int n_in, int k, int avg_block, float hpow, int64_t woff) {
  if (n_out % 128 != 0 || n_in % 128 != 0 || woff % 32 != 0 || avg_block > 32 || hpow != 1.0f) return false;
  if ((int64_t)n_out * n_in >= (1ll << 31)) return false;
  return (int64_t)(n_out / 128) * (n_in / 128) * k >= 512;
}
int gemm_f32_wgrad_tiles(int n_out, int n_in) { return (n_out / 128) * (n_in / 128); }

hipError_t launch_gemm_f32(const GemmArgs& a, hipStream_t s) {
  KernelScope ks(a.epi == EPI_WGRAD ? KC_GEMM_WGRAD : (a.epi == EPI_MASK || a.epi == EPI_PLAIN) ? KC_GEMM_DGRAD : KC_GEMM_FWD, s);
  if (a.epi == EPI_WGRAD && a.fu.on) return launch_fused_wgrad(a, s);
  if (a.N <= 32) return launch_shape<128, 32, 4, 1>(a, s);
  if (a.M <= 32) return launch_shape<32, 128, 1, 4>(a, s);
  if (a.N <= 64 && (int64_t)((a.M + 127) / 128) * a.k >= 512) return launch_shape<128, 64, 2, 2>(a, s);   // many rows, few columns
  const int64_t big_tiles = (int64_t)((a.M + 127) / 128) * ((a.N + 127) / 128) * a.k;
  if (big_tiles >= 512 && a.M > 64 && a.N > 64) return launch_shape<128, 128, 2, 2>(a, s);   // (a 128-wide tile on 64 rows is half empty)
  return launch_shape<64, 64, 2, 2>(a, s);
}

}  // namespace dw
