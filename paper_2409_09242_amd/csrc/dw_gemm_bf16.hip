// bf16 "dual-number" GEMM for gfx950: C = X*Y and RC = RX*Y + X*RY with bf16 operands and fp32 accumulation.
//
// Same product-rule structure as the fp32 kernel (forward, data gradient and weight gradient of the MLP
// together with their directional derivatives along z, which give the Hessian-vector product of the
// Hutchinson estimate, Section IV-B), on the bf16 matrix cores: v_mfma_f32_32x32x16_bf16, where lane l
// supplies 8 consecutive k of row l%32, k-chunk l/32, for both operands.
//
// Tiling: 256 threads = 4 waves; block tile BM x BN x 32, LDS tiles stored [row][k] with 8 k per 16 bytes
// (row stride 40 bf16 = 80 B, which makes the 16-byte operand reads conflict-free) and double-buffered, so
// one barrier per k-tile.  Operands whose contraction index is the slow one in memory (W in the data
// gradient, both operands of the weight gradient) are transposed in registers on their way into LDS:
// a thread loads a 4(row) x 8(k) patch as eight 8-byte loads and writes four 16-byte LDS rows.
// The +-1 operand V (z reshaped like W) is expanded from the sign bits of z in the loader.
#include "dw_internal.h"

namespace dw {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

namespace b16 {

constexpr int BK = 32;          // k per tile (two MFMA k-steps of 16)
constexpr int LDK = 40;         // LDS row stride in bf16 elements
constexpr int NT = 256;

enum RyMode { RY_NONE = 0, RY_MEM = 1, RY_BITS = 2 };

__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// two bf16 values +-1 from two sign bits (bit set -> +1 = 0x3F80, clear -> -1 = 0xBF80)
__device__ __forceinline__ uint32_t pm1_pair(uint32_t b_lo, uint32_t b_hi) {
  return 0xBF80BF80u ^ (b_lo << 15) ^ (b_hi << 31);
}

// One operand tile of R rows x BK k, loaded by NTH threads (thread index tl in [0, NTH)).
//   KC = true : source rows are k-contiguous; unit = 8 k of one row (one 16-byte load, one 16-byte LDS store)
//   KC = false: source is k-major ([k][row]); unit = patch of 4 rows x 8 k (eight 8-byte loads, register
//               transpose, four 16-byte LDS stores)
template <int R, int NTH, bool KC>
struct Loader {
  static constexpr int UNITS = KC ? R * (BK / 8) : (R / 4) * (BK / 8);
  static constexpr int UPT = (UNITS + NTH - 1) / NTH;
  static constexpr int REGS = KC ? UPT : UPT * 4;          // uint4 registers per thread

  __device__ static __forceinline__ void load(const uint16_t* __restrict__ src, int ld, int r0, int k0, int Rmax,
                                              int K, int tl, uint4 (&reg)[REGS]) {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = u * NTH + tl;
      if (KC) {
        const int row = unit / (BK / 8), kc = (unit % (BK / 8)) * 8;
        const bool ok = unit < UNITS && (r0 + row) < Rmax && (k0 + kc) < K;
        reg[u] = ok ? *reinterpret_cast<const uint4*>(src + (int64_t)(r0 + row) * ld + (k0 + kc))
                    : make_uint4(0, 0, 0, 0);
      } else {
        const int rq = (unit % (R / 4)) * 4, kq = (unit / (R / 4)) * 8;
        const bool okr = unit < UNITS && (r0 + rq) < Rmax;
        uint2 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const bool ok = okr && (k0 + kq + i) < K;
          v[i] = ok ? *reinterpret_cast<const uint2*>(src + (int64_t)(k0 + kq + i) * ld + (r0 + rq)) : make_uint2(0, 0);
        }
        reg[u * 4 + 0] = make_uint4(v[0].x, v[0].y, v[1].x, v[1].y);
        reg[u * 4 + 1] = make_uint4(v[2].x, v[2].y, v[3].x, v[3].y);
        reg[u * 4 + 2] = make_uint4(v[4].x, v[4].y, v[5].x, v[5].y);
        reg[u * 4 + 3] = make_uint4(v[6].x, v[6].y, v[7].x, v[7].y);
      }
    }
  }

  // sign bits of the elements load() would read: KC: 8 bits per unit; !KC: 8 nibbles (k rows) per unit
  __device__ static __forceinline__ void load_bits(const uint32_t* __restrict__ zb, int64_t z_off, int ld, int r0,
                                                   int k0, int Rmax, int K, int tl, uint32_t (&reg)[UPT]) {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = u * NTH + tl;
      if (KC) {
        const int row = unit / (BK / 8), kc = (unit % (BK / 8)) * 8;
        const bool ok = unit < UNITS && (r0 + row) < Rmax && (k0 + kc) < K;
        const int64_t off = z_off + (int64_t)(r0 + row) * ld + (k0 + kc);
        reg[u] = ok ? (zb[off >> 5] >> (off & 31)) & 0xFFu : 0u;
      } else {
        const int rq = (unit % (R / 4)) * 4, kq = (unit / (R / 4)) * 8;
        const bool okr = unit < UNITS && (r0 + rq) < Rmax;
        uint32_t packed = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const bool ok = okr && (k0 + kq + i) < K;
          const int64_t off = z_off + (int64_t)(k0 + kq + i) * ld + (r0 + rq);
          const uint32_t nib = ok ? (zb[off >> 5] >> (off & 31)) & 0xFu : 0u;
          packed |= nib << (4 * i);
        }
        reg[u] = packed;
      }
    }
  }

  // v[i] = (elements of rows rq..rq+3 at k = kq+i) as two dwords; writes rows rq+j, j = 0..3
  __device__ static __forceinline__ void store_patch(uint16_t (*lds)[LDK], int rq, int kq, const uint32_t (&lo)[8],
                                                     const uint32_t (&hi)[8]) {
    // lo[i] holds rows (rq, rq+1) at k_i, hi[i] rows (rq+2, rq+3)
    uint4 o0, o1, o2, o3;
    o0.x = __builtin_amdgcn_perm(lo[1], lo[0], 0x05040100u); o1.x = __builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u);
    o0.y = __builtin_amdgcn_perm(lo[3], lo[2], 0x05040100u); o1.y = __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u);
    o0.z = __builtin_amdgcn_perm(lo[5], lo[4], 0x05040100u); o1.z = __builtin_amdgcn_perm(lo[5], lo[4], 0x07060302u);
    o0.w = __builtin_amdgcn_perm(lo[7], lo[6], 0x05040100u); o1.w = __builtin_amdgcn_perm(lo[7], lo[6], 0x07060302u);
    o2.x = __builtin_amdgcn_perm(hi[1], hi[0], 0x05040100u); o3.x = __builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u);
    o2.y = __builtin_amdgcn_perm(hi[3], hi[2], 0x05040100u); o3.y = __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u);
    o2.z = __builtin_amdgcn_perm(hi[5], hi[4], 0x05040100u); o3.z = __builtin_amdgcn_perm(hi[5], hi[4], 0x07060302u);
    o2.w = __builtin_amdgcn_perm(hi[7], hi[6], 0x05040100u); o3.w = __builtin_amdgcn_perm(hi[7], hi[6], 0x07060302u);
    *reinterpret_cast<uint4*>(&lds[rq + 0][kq]) = o0;
    *reinterpret_cast<uint4*>(&lds[rq + 1][kq]) = o1;
    *reinterpret_cast<uint4*>(&lds[rq + 2][kq]) = o2;
    *reinterpret_cast<uint4*>(&lds[rq + 3][kq]) = o3;
  }

  __device__ static __forceinline__ void store(uint16_t (*lds)[LDK], int tl, const uint4 (&reg)[REGS]) {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = u * NTH + tl;
      if (unit >= UNITS) continue;
      if (KC) {
        const int row = unit / (BK / 8), kc = (unit % (BK / 8)) * 8;
        *reinterpret_cast<uint4*>(&lds[row][kc]) = reg[u];
      } else {
        const int rq = (unit % (R / 4)) * 4, kq = (unit / (R / 4)) * 8;
        const uint32_t lo[8] = {reg[u * 4 + 0].x, reg[u * 4 + 0].z, reg[u * 4 + 1].x, reg[u * 4 + 1].z,
                                reg[u * 4 + 2].x, reg[u * 4 + 2].z, reg[u * 4 + 3].x, reg[u * 4 + 3].z};
        const uint32_t hi[8] = {reg[u * 4 + 0].y, reg[u * 4 + 0].w, reg[u * 4 + 1].y, reg[u * 4 + 1].w,
                                reg[u * 4 + 2].y, reg[u * 4 + 2].w, reg[u * 4 + 3].y, reg[u * 4 + 3].w};
        store_patch(lds, rq, kq, lo, hi);
      }
    }
  }

  __device__ static __forceinline__ void store_bits(uint16_t (*lds)[LDK], int tl, const uint32_t (&reg)[UPT]) {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int unit = u * NTH + tl;
      if (unit >= UNITS) continue;
      if (KC) {
        const int row = unit / (BK / 8), kc = (unit % (BK / 8)) * 8;
        const uint32_t b = reg[u];
        uint4 o;
        o.x = pm1_pair(b & 1u, (b >> 1) & 1u); o.y = pm1_pair((b >> 2) & 1u, (b >> 3) & 1u);
        o.z = pm1_pair((b >> 4) & 1u, (b >> 5) & 1u); o.w = pm1_pair((b >> 6) & 1u, (b >> 7) & 1u);
        *reinterpret_cast<uint4*>(&lds[row][kc]) = o;
      } else {
        const int rq = (unit % (R / 4)) * 4, kq = (unit / (R / 4)) * 8;
        uint32_t lo[8], hi[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t nib = (reg[u] >> (4 * i)) & 0xFu;
          lo[i] = pm1_pair(nib & 1u, (nib >> 1) & 1u);
          hi[i] = pm1_pair((nib >> 2) & 1u, (nib >> 3) & 1u);
        }
        store_patch(lds, rq, kq, lo, hi);
      }
    }
  }
};

template <int BM, int BN, int WM, int WN, bool X_KC, bool Y_KC, bool HAS_RX, int RYM, int EPI>
__global__ __launch_bounds__(NT) void dual_gemm_bf16(GemmArgs a) {
  static_assert(WM * WN == 4, "four waves per block");
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");
  const int worker = blockIdx.y;
  if (!((a.active_mask >> worker) & 1ull)) return;

  const int tiles_m = (a.M + BM - 1) / BM;
  const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % WM) * (BM / WM), wn0 = (wave / WM) * (BN / WN);
  const int l32 = lane & 31, lhalf = lane >> 5;

  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  // per stage: Xs[BM], RXs[BM] (if HAS_RX), Ys[BN], RYs[BN] (if RYM), each [rows][LDK]
  constexpr int X_ROWS = BM * (HAS_RX ? 2 : 1);
  constexpr int Y_ROWS = BN * (RYM != RY_NONE ? 2 : 1);
  constexpr int STAGE = (X_ROWS + Y_ROWS) * LDK;
  auto Xs = [&](int st) { return reinterpret_cast<uint16_t(*)[LDK]>(smem + st * STAGE); };
  auto RXs = [&](int st) { return reinterpret_cast<uint16_t(*)[LDK]>(smem + st * STAGE + BM * LDK); };
  auto Ys = [&](int st) { return reinterpret_cast<uint16_t(*)[LDK]>(smem + st * STAGE + X_ROWS * LDK); };
  auto RYs = [&](int st) { return reinterpret_cast<uint16_t(*)[LDK]>(smem + st * STAGE + (X_ROWS + BN) * LDK); };

  const uint16_t* X = reinterpret_cast<const uint16_t*>(a.X) + (int64_t)worker * a.x_wstride;
  const uint16_t* RX = HAS_RX ? reinterpret_cast<const uint16_t*>(a.RX) + (int64_t)worker * a.x_wstride : nullptr;
  const uint16_t* Y = reinterpret_cast<const uint16_t*>(a.Y) + (int64_t)worker * a.y_wstride;
  const uint16_t* RY = RYM == RY_MEM ? reinterpret_cast<const uint16_t*>(a.RY) + (int64_t)worker * a.y_wstride : nullptr;
  const uint32_t* zb = a.zbits + (int64_t)worker * a.z_stride;

  // X and RX are loaded by one half of the block each (the halves are whole waves); Y and RY by all threads
  constexpr int XTH = HAS_RX ? NT / 2 : NT;
  using LX = Loader<BM, XTH, X_KC>;
  using LY = Loader<BN, NT, Y_KC>;
  const bool second_half = HAS_RX && tid >= XTH;
  const int xtl = second_half ? tid - XTH : tid;
  const uint16_t* xsrc = second_half ? RX : X;
  uint4 xr[LX::REGS], yr[LY::REGS], ryr[LY::REGS];
  uint32_t zr[LY::UPT];

  floatx16 acc[TM][TN], racc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0.f; racc[i][j][r] = 0.f; }
  float gb_acc = 0.f, hzb_acc = 0.f;

  const int nkt = (a.K + BK - 1) / BK;
  auto fetch = [&](int kt) {
    const int k0 = kt * BK;
    LX::load(xsrc, a.ldx, row0, k0, a.M, a.K, xtl, xr);
    LY::load(Y, a.ldy, col0, k0, a.N, a.K, tid, yr);
    if (RYM == RY_MEM) LY::load(RY, a.ldy, col0, k0, a.N, a.K, tid, ryr);
    if (RYM == RY_BITS) LY::load_bits(zb, a.z_off, a.ldy, col0, k0, a.N, a.K, tid, zr);
  };
  auto stash = [&](int st) {
    LX::store(second_half ? RXs(st) : Xs(st), xtl, xr);
    LY::store(Ys(st), tid, yr);
    if (RYM == RY_MEM) LY::store(RYs(st), tid, ryr);
    if (RYM == RY_BITS) LY::store_bits(RYs(st), tid, zr);
  };

  fetch(0);
  stash(0);
  if (nkt > 1) fetch(1);
  __syncthreads();

  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nkt) stash(cur ^ 1);
    if (kt + 2 < nkt) fetch(kt + 2);

    if (EPI == EPI_WGRAD && tn == 0 && tid < BM) {
      const uint16_t(*xs)[LDK] = Xs(cur);
      const uint16_t(*rxs)[LDK] = RXs(cur);
#pragma unroll
      for (int kk = 0; kk < BK; ++kk) {
        gb_acc += bf2f(xs[tid][kk]);
        if (HAS_RX) hzb_acc += bf2f(rxs[tid][kk]);
      }
    }

#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int kc = ks * 16 + lhalf * 8;
      bf16x8 xa[TM], rxa[TM], yb[TN], ryb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        xa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&Xs(cur)[wm0 + i * 32 + l32][kc]));
        if (HAS_RX)
          rxa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&RXs(cur)[wm0 + i * 32 + l32][kc]));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        yb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&Ys(cur)[wn0 + j * 32 + l32][kc]));
        if (RYM != RY_NONE)
          ryb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&RYs(cur)[wn0 + j * 32 + l32][kc]));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[i], yb[j], acc[i][j], 0, 0, 0);
          if (HAS_RX) racc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rxa[i], yb[j], racc[i][j], 0, 0, 0);
          if (RYM != RY_NONE) racc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[i], ryb[j], racc[i][j], 0, 0, 0);
        }
    }
    __syncthreads();
  }

  // epilogue: lane holds column n = l32 of each 32x32 tile, rows (r/4)*8 + lhalf*4 + r%4
#pragma unroll
  for (int j = 0; j < TN; ++j) {
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
        const int64_t o = (int64_t)worker * a.c_wstride + (int64_t)m * a.ldc + n;
        if (EPI == EPI_RELU) {
          c += bias; rc += cz;
          const bool on = c > 0.f;
          reinterpret_cast<uint16_t*>(a.C)[o] = f2bf(on ? c : 0.f);
          reinterpret_cast<uint16_t*>(a.RC)[o] = f2bf(on ? rc : 0.f);
        } else if (EPI == EPI_LINEAR) {
          reinterpret_cast<float*>(a.C)[o] = c + bias;
          reinterpret_cast<float*>(a.RC)[o] = rc + cz;
        } else if (EPI == EPI_MASK) {
          const uint16_t* msk = reinterpret_cast<const uint16_t*>(a.mask_src) + (int64_t)worker * a.mask_wstride;
          const uint16_t mv = msk[(int64_t)m * a.ld_mask + n];
          const bool on = mv != 0 && !(mv & 0x8000u);     // stored activation > 0
          reinterpret_cast<uint16_t*>(a.C)[o] = f2bf(on ? c : 0.f);
          reinterpret_cast<uint16_t*>(a.RC)[o] = f2bf(on ? rc : 0.f);
        } else {
          reinterpret_cast<float*>(a.C)[o] = c;
          reinterpret_cast<float*>(a.RC)[o] = rc;
        }
      }
    }
  }
  if (EPI == EPI_WGRAD && tn == 0 && tid < BM) {
    const int m = row0 + tid;
    if (m < a.M) {
      a.gb[(int64_t)worker * a.c_wstride + m] = gb_acc;
      a.hzb[(int64_t)worker * a.c_wstride + m] = hzb_acc;
    }
  }
}

template <int BM, int BN, bool HAS_RX, int RYM>
constexpr int smem_bytes() {
  return 2 * (BM * (HAS_RX ? 2 : 1) + BN * (RYM != RY_NONE ? 2 : 1)) * LDK * 2;
}

template <int BM, int BN, int WM, int WN, bool XKC, bool YKC, bool RX, int RYM, int EPI>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s) {
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  const dim3 grid((unsigned)tiles, (unsigned)a.k), block(NT);
  constexpr int smem = smem_bytes<BM, BN, RX, RYM>();
  auto kern = dual_gemm_bf16<BM, BN, WM, WN, XKC, YKC, RX, RYM, EPI>;
  static bool configured = false;        // raise the dynamic LDS limit once per instantiation
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    configured = true;
  }
  hipLaunchKernelGGL(kern, grid, block, smem, s, a);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN>
static hipError_t launch_shape(const GemmArgs& a, hipStream_t s) {
  const bool rx = a.RX != nullptr;
  if (a.epi == EPI_RELU) {
    return rx ? launch_one<BM, BN, WM, WN, true, true, true, RY_BITS, EPI_RELU>(a, s)
              : launch_one<BM, BN, WM, WN, true, true, false, RY_BITS, EPI_RELU>(a, s);
  } else if (a.epi == EPI_LINEAR) {
    return rx ? launch_one<BM, BN, WM, WN, true, true, true, RY_BITS, EPI_LINEAR>(a, s)
              : launch_one<BM, BN, WM, WN, true, true, false, RY_BITS, EPI_LINEAR>(a, s);
  } else if (a.epi == EPI_MASK) {
    return launch_one<BM, BN, WM, WN, true, false, true, RY_BITS, EPI_MASK>(a, s);
  }
  return a.RY ? launch_one<BM, BN, WM, WN, false, false, true, RY_MEM, EPI_WGRAD>(a, s)
              : launch_one<BM, BN, WM, WN, false, false, true, RY_NONE, EPI_WGRAD>(a, s);
}

}  // namespace b16

hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  KernelScope ks(a.epi == EPI_WGRAD ? KC_GEMM_WGRAD : a.epi == EPI_MASK ? KC_GEMM_DGRAD : KC_GEMM_FWD, s);
  if (a.N <= 32) return b16::launch_shape<128, 32, 4, 1>(a, s);
  if (a.M <= 32) return b16::launch_shape<32, 128, 1, 4>(a, s);
  const int64_t big_tiles = (int64_t)((a.M + 127) / 128) * ((a.N + 255) / 256) * a.k;
  if (big_tiles >= 256) return b16::launch_shape<128, 256, 2, 2>(a, s);
  return b16::launch_shape<64, 64, 2, 2>(a, s);
}

}  // namespace dw
