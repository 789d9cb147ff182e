// bf16 "dual-number" GEMM for gfx950: C = X*Y and RC = RX*Y + X*RY with bf16 operands and fp32 accumulation.
//
// Same product-rule structure as the fp32 kernel (forward, data gradient and weight gradient of the MLP
// together with their directional derivatives along z, which give the Hessian-vector product of the
// Hutchinson estimate, Section IV-B), on the bf16 matrix cores: v_mfma_f32_32x32x16_bf16, where lane l
// supplies 8 consecutive k of row l%32, k-chunk l/32, for both operands.
//
// Tiling: 512 threads = 8 waves (two per SIMD, so one wave's LDS reads hide behind the other's MFMAs);
// block tile BM x BN x 32, double-buffered in LDS with one barrier per k-tile.  Every global load and LDS
// store is a plain 16-byte copy along the axis that is contiguous in memory:
//   - an operand whose contraction index k is contiguous is staged [row][k] (row stride 40 bf16 = 80 B, so
//     the 16-byte operand reads are conflict-free);
//   - an operand stored k-major (W in the data gradient, both operands of the weight gradient) is staged
//     [k][row] as it lies in memory and transposed by the LDS itself on the way out (ds_read_b64_tr_b16:
//     within 16 lanes, lane i receives element i%4 of the 8-byte rows addressed by lanes i/4, 4+i/4, 8+i/4,
//     12+i/4), which hands each lane its 4 consecutive k for one row.
// The +-1 operand V (z reshaped like W) is expanded from the sign bits of z in the loader.
#include <cstddef>

#include "dw_internal.h"
#include "dw_device_util.h"
#include "dw_gemm_epi.h"
#include "dw_fused_update.h"

namespace dw {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short v4i16 __attribute__((ext_vector_type(4)));

namespace b16 {

constexpr int BK = 32;          // k per tile (two MFMA k-steps of 16)
constexpr int LDK = 40;         // row stride (elements) of a [row][k] tile
constexpr int KPAD = 32;        // row padding (elements) of a [k][row] tile
[[maybe_unused]] constexpr int NT = 512;   // block size of every shape but the fused weight gradient's

enum RyMode { RY_NONE = 0, RY_MEM = 1, RY_BITS = 2 };

__device__ __forceinline__ float bf2f(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// two bf16 values +-1 from two sign bits (bit set -> +1 = 0x3F80, clear -> -1 = 0xBF80)
__device__ __forceinline__ uint32_t pm1_pair(uint32_t b_lo, uint32_t b_hi) {
  return 0xBF80BF80u ^ (b_lo << 15) ^ (b_hi << 31);
}
__device__ __forceinline__ uint4 pm1_x8(uint32_t b) {
  uint4 o;
  o.x = pm1_pair(b & 1u, (b >> 1) & 1u); o.y = pm1_pair((b >> 2) & 1u, (b >> 3) & 1u);
  o.z = pm1_pair((b >> 4) & 1u, (b >> 5) & 1u); o.w = pm1_pair((b >> 6) & 1u, (b >> 7) & 1u);
  return o;
}

// One operand tile: R rows (the non-contraction index) x BK, moved by NTH threads in 16-byte units.
//   KC = true : memory is [row][k]; unit u = 8 k of row u/4; LDS [R][LDK]
//   KC = false: memory is [k][row]; unit u = 8 rows at k = u/(R/8); LDS [BK][R+KPAD]
//   BKT: k per tile (BK, or 16 for [k][row] tiles of the two-probe weight gradient)
template <int R, int NTH, bool KC, int BKT = BK>
struct Tile {
  static_assert(BKT == BK || (!KC && BKT == 16), "[row][k] tiles have the row stride of BK = 32");
  static constexpr int UNITS = R * BKT / 8;
  static constexpr int UPT = (UNITS + NTH - 1) / NTH;
  static constexpr int LDS_ELEMS = KC ? R * LDK : BKT * (R + KPAD);
  static constexpr int LDR = R + KPAD;

  // Unit u of this thread is unit number u*NTH + tl of the tile; a thread's units differ by constants, so
  // only the first one's offsets are kept.
  static constexpr bool FULL = UNITS % NTH == 0;                          // every thread owns UPT units
  static constexpr int ROWS_PER_PASS = KC ? NTH / (BKT / 8) : 0;          // KC: rows between a thread's units
  static constexpr int K_PER_PASS = KC ? 0 : (NTH >= R / 8 ? NTH / (R / 8) : 0);   // !KC: k rows between them
  int goff0;              // element offset of unit 0 in the source at k0 = 0 (an operand has < 2^31 elements)
  int loff0;              // element offset of unit 0 in the LDS tile
  int kk0;                // k index of unit 0 inside the tile
  unsigned okmask;        // bit u: unit u exists and its row (KC) / column group (!KC) is inside the operand

  __device__ __forceinline__ void init(int tl, int ld, int r0, int Rmax) {
    okmask = 0;
    if (KC) {
      const int row = tl / (BKT / 8), kc = (tl % (BKT / 8)) * 8;
      goff0 = (r0 + row) * ld + kc; loff0 = row * LDK + kc; kk0 = kc;
#pragma unroll
      for (int u = 0; u < UPT; ++u)
        if ((FULL || u * NTH + tl < UNITS) && (r0 + row + u * ROWS_PER_PASS) < Rmax) okmask |= 1u << u;
    } else {
      const int krow = tl / (R / 8), c = (tl % (R / 8)) * 8;
      goff0 = krow * ld + (r0 + c); loff0 = krow * LDR + c; kk0 = krow;
#pragma unroll
      for (int u = 0; u < UPT; ++u)
        if ((FULL || u * NTH + tl < UNITS) && (r0 + c) < Rmax) okmask |= 1u << u;
    }
  }
  __device__ __forceinline__ int kk(int u) const { return KC ? kk0 : kk0 + u * K_PER_PASS; }
  __device__ __forceinline__ int loff(int u) const {
    return KC ? loff0 + u * ROWS_PER_PASS * LDK : loff0 + u * K_PER_PASS * LDR;
  }
  __device__ __forceinline__ bool ok(int u, int k0, int K) const { return ((okmask >> u) & 1u) && (k0 + kk(u)) < K; }
  __device__ __forceinline__ int64_t at(int u, int k0, int ld) const {
    return KC ? (int64_t)goff0 + (int64_t)u * ROWS_PER_PASS * ld + k0
              : (int64_t)goff0 + (int64_t)(u * K_PER_PASS + k0) * ld;
  }
  // Loads are unconditional (a unit outside the operand reads the operand's first elements instead), so the
  // prefetch is free of branches and of waits; such a unit is zeroed when it is copied into LDS.
  // WHOLE: every unit of the tile lies inside the operand (whole tiles, a contraction of whole k-tiles): no selects
  template <bool WHOLE = false>
  __device__ __forceinline__ void load(const uint16_t* __restrict__ src, int ld, int k0, int K, uint4 (&reg)[UPT]) const {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int64_t o = (WHOLE || ok(u, k0, K)) ? at(u, k0, ld) : 0;
      reg[u] = *reinterpret_cast<const uint4*>(src + o);
    }
  }
  // the raw 32-bit word holding the unit's 8 sign bits; the bits are extracted when the tile is stored
  __device__ __forceinline__ void load_bits(const uint32_t* __restrict__ zb, int64_t z_off, int ld, int k0, int K,
                                            uint32_t (&reg)[UPT]) const {
#pragma unroll
    for (int u = 0; u < UPT; ++u) {
      const int64_t off = z_off + (ok(u, k0, K) ? at(u, k0, ld) : 0);
      reg[u] = zb[off >> 5];
    }
  }
  template <bool WHOLE = false>
  __device__ __forceinline__ void store(uint16_t* lds, const uint4 (&reg)[UPT], int tl, int k0, int K) const {
#pragma unroll
    for (int u = 0; u < UPT; ++u)
      if (FULL || u * NTH + tl < UNITS)
        *reinterpret_cast<uint4*>(lds + loff(u)) = (WHOLE || ok(u, k0, K)) ? reg[u] : make_uint4(0, 0, 0, 0);
  }
  __device__ __forceinline__ void store_bits(uint16_t* lds, const uint32_t (&reg)[UPT], int tl, int64_t z_off,
                                             int k0, int ld) const {
#pragma unroll
    for (int u = 0; u < UPT; ++u)
      if (FULL || u * NTH + tl < UNITS) {
        const int sh = (int)((z_off + at(u, k0, ld)) & 31);
        *reinterpret_cast<uint4*>(lds + loff(u)) = pm1_x8((reg[u] >> sh) & 0xFFu);
      }
  }
};

// MFMA operand of one lane: 8 consecutive k (k-step ks, chunk lane/32) of tile row `row0 + lane%32`
template <int R, bool KC>
__device__ __forceinline__ bf16x8 frag(const uint16_t* lds, int row0, int ks, int lane) {
  if (KC) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(
        lds + (row0 + (lane & 31)) * LDK + ks * 16 + (lane >> 5) * 8));
  } else {
    constexpr int LDR = R + KPAD;
    const int s = lane & 15;
    const uint16_t* p = lds + (ks * 16 + (lane >> 5) * 8 + (s >> 2)) * LDR + row0 + ((lane >> 4) & 1) * 16 + (s & 3) * 4;
    typedef __attribute__((address_space(3))) v4i16 lds_v4;
    struct { v4i16 a, b; } r;
    r.a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4*)(p));
    r.b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4*)(p + 4 * LDR));
    return __builtin_bit_cast(bf16x8, r);
  }
}

// KWHOLE (fused weight gradient): the minibatch is made of whole k-tiles, so every load and LDS store of the main loop is
// unconditional (the tiles of a fused layer are whole anyway)
template <int BM, int BN, int WM, int WN, bool X_KC, bool Y_KC, bool HAS_RX, int RYM, int EPI, int FM = 0, int NTH = 512,
          bool KWHOLE = false>
__global__ __launch_bounds__(NTH, NTH == 256 ? 2 : 1) void dual_gemm_bf16(GemmArgs a) {   // (two waves per SIMD either way)
  constexpr int NT = NTH;                                   // threads per block: 512, or 256 (see launch_fused_wgrad)
  static_assert(WM * WN == NT / 64, "one wave tile per wave");
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  static_assert(TM >= 1 && TN >= 1, "wave tile must hold at least one 32x32 MFMA tile");
  // Workgroups are handed to the 8 XCDs round-robin by their index.  The index is remapped so that each XCD
  // works through a contiguous range of (worker, tile) pairs: the blocks that share a W tile or a worker's
  // activations then run on the same XCD at about the same time and meet in its L2.
  const int tiles_m = (a.M + BM - 1) / BM;
  const int tiles = tiles_m * ((a.N + BN - 1) / BN);
  const int per_xcd = gridDim.x >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  const int slot = logical / tiles;                         // which of the active workers
  if (slot >= active_count(a.active_mask, a.k)) return;
  const int worker = nth_active_worker(a.active_mask, slot);
  const int tile = logical - slot * tiles;
  if (EPI == EPI_WGRAD && NTH == 256 && FM != 1 && blockIdx.x < 256 * 8) {
    // Fused update: a block alternates between a compute-bound main loop and an HBM-bound epilogue of about twice
    // its length.  Blocks that start together stay in step, leaving HBM idle while everybody multiplies, so the
    // first block of every compute unit starts with one of 16 delays spread over about one block period.
    const int ph = (blockIdx.x >> 3) & 15;
    if (blockIdx.x < 256)
      for (int i = 0; i < ph; ++i) __builtin_amdgcn_s_sleep(127);
  }
  int tm = tile % tiles_m, tn = tile / tiles_m;
  if (EPI == EPI_WGRAD && tiles_m % 8 == 0) {
    // Weight gradient: both operands are panels of the minibatch (512 k x 128 or 256 columns, with their
    // R-companions 256 KB and 512 KB).  The blocks an XCD runs at a time (32 of 128 x 256, or 64 of 128 x 128) are
    // 8 row tiles x 4 or 8 column tiles (2 + 2 MB of panels, which its 4 MB L2 can hold) instead of a column of
    // row tiles (8 MB and more).
    const int tiles_n = tiles / tiles_m;
    const int g = tile / (8 * tiles_n), r = tile - g * (8 * tiles_n);
    tn = r / 8; tm = g * 8 + r % 8;
  }
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % WM) * (BM / WM), wn0 = (wave / WM) * (BN / WN);
  const int l32 = lane & 31, lhalf = lane >> 5;

  // X and RX are each moved by one half of the block (whole waves); Y and RY by all threads
  constexpr int XTH = HAS_RX ? NT / 2 : NT;
  using TX = Tile<BM, XTH, X_KC>;
  using TY = Tile<BN, NT, Y_KC>;
  constexpr int X_ELEMS = TX::LDS_ELEMS, Y_ELEMS = TY::LDS_ELEMS;
  constexpr int STAGE = X_ELEMS * (HAS_RX ? 2 : 1) + Y_ELEMS * (RYM != RY_NONE ? 2 : 1);
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  auto Xs = [&](int st) { return smem + st * STAGE; };
  auto RXs = [&](int st) { return smem + st * STAGE + X_ELEMS; };
  auto Ys = [&](int st) { return smem + st * STAGE + X_ELEMS * (HAS_RX ? 2 : 1); };
  auto RYs = [&](int st) { return smem + st * STAGE + X_ELEMS * (HAS_RX ? 2 : 1) + Y_ELEMS; };

  const bool second_half = HAS_RX && tid >= XTH;
  const int xtl = second_half ? tid - XTH : tid;
  const uint16_t* xsrc = reinterpret_cast<const uint16_t*>(second_half ? a.RX : a.X) + (int64_t)worker * a.x_wstride;
  const uint16_t* Y = reinterpret_cast<const uint16_t*>(a.Y) + (int64_t)worker * a.y_wstride;
  const uint16_t* RY = RYM == RY_MEM ? reinterpret_cast<const uint16_t*>(a.RY) + (int64_t)worker * a.y_wstride : nullptr;
  const uint32_t* zb = a.zbits + (int64_t)worker * a.z_stride;

  TX tx; TY ty;
  tx.init(xtl, a.ldx, row0, a.M);
  ty.init(tid, a.ldy, col0, a.N);
  uint4 xr[TX::UPT], yr[TY::UPT], ryr[TY::UPT];
  uint32_t zr[TY::UPT];

  floatx16 acc[TM][TN], racc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0.f; racc[i][j][r] = 0.f; }
  float gb_acc = 0.f, hzb_acc = 0.f;

  // launch_fused_wgrad's instances apply the update of Section IV-B to the tile (FM: 0 one Hutchinson probe; 1 a probe
  // before the last, only the running sum of z*Hz is written; 2 the last of several probes)
  constexpr bool FUSED = EPI == EPI_WGRAD && NTH == 256 && TN == 2;

  const int nkt = (a.K + BK - 1) / BK;
  auto fetch = [&](int kt) {
    const int k0 = kt * BK;
    tx.template load<KWHOLE>(xsrc, a.ldx, k0, a.K, xr);
    ty.template load<KWHOLE>(Y, a.ldy, k0, a.K, yr);
    if (RYM == RY_MEM) ty.template load<KWHOLE>(RY, a.ldy, k0, a.K, ryr);
    if (RYM == RY_BITS) ty.load_bits(zb, a.z_off, a.ldy, k0, a.K, zr);
  };
  auto stash = [&](int st, int kt) {       // kt: the k-tile held in the registers
    tx.template store<KWHOLE>(second_half ? RXs(st) : Xs(st), xr, xtl, kt * BK, a.K);
    ty.template store<KWHOLE>(Ys(st), yr, tid, kt * BK, a.K);
    if (RYM == RY_MEM) ty.template store<KWHOLE>(RYs(st), ryr, tid, kt * BK, a.K);
    if (RYM == RY_BITS) ty.store_bits(RYs(st), zr, tid, a.z_off, kt * BK, a.ldy);
  };

  // operand registers of one k-step; two sets alternate so that the LDS reads of the next k-step are in
  // flight while the matrix cores work on the current one
  struct Frags { bf16x8 xa[TM], rxa[TM], yb[TN], ryb[TN]; };
  auto read_frags = [&](Frags& f, int st, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      f.xa[i] = frag<BM, X_KC>(Xs(st), wm0 + i * 32, ks, lane);
      if (HAS_RX) f.rxa[i] = frag<BM, X_KC>(RXs(st), wm0 + i * 32, ks, lane);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      f.yb[j] = frag<BN, Y_KC>(Ys(st), wn0 + j * 32, ks, lane);
      if (RYM != RY_NONE) f.ryb[j] = frag<BN, Y_KC>(RYs(st), wn0 + j * 32, ks, lane);
    }
  };
  auto mfma_step = [&](const Frags& f) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        if (FM != 1)                                         // (a probe before the last only needs the R-products)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.xa[i], f.yb[j], acc[i][j], 0, 0, 0);
    if (HAS_RX) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          racc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.rxa[i], f.yb[j], racc[i][j], 0, 0, 0);
    }
    if (RYM != RY_NONE) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          racc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.xa[i], f.ryb[j], racc[i][j], 0, 0, 0);
    }
  };
  static_assert(BK == 32, "the loop below is written for two k-steps per tile");

  auto compute_tile = [&](int cur) {
    if (EPI == EPI_WGRAD && tn == 0 && tid < BM) {       // bias gradients: sums over the minibatch (X is [k][m])
      const uint16_t* xs = Xs(cur);
      const uint16_t* rxs = RXs(cur);
#pragma unroll
      for (int kq = 0; kq < BK; ++kq) {
        gb_acc += bf2f(xs[kq * TX::LDR + tid]);
        if (HAS_RX) hzb_acc += bf2f(rxs[kq * TX::LDR + tid]);
      }
    }
    Frags f0, f1;
    read_frags(f0, cur, 0);
    read_frags(f1, cur, 1);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);                           // the wave feeding the matrix cores issues first
    mfma_step(f0);
    mfma_step(f1);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto move_tiles = [&](int kt, int cur) {
    if (kt + 1 < nkt) stash(cur ^ 1, kt + 1);            // registers -> the other LDS stage
    if (kt + 2 < nkt) fetch(kt + 2);                     // global -> registers, for the iteration after next
  };

  fetch(0);
  stash(0, 0);
  if (nkt > 1) fetch(1);
  __syncthreads();

  // The two waves that share a SIMD (w and w+4) run the two halves of an iteration in opposite order: one
  // feeds the matrix cores while the other waits for its global loads and copies them into LDS, then they
  // swap.  Both read LDS stage `cur` and write stage `cur^1`, so one barrier per k-tile is enough.
  const bool compute_first = wave < (NT / 64) / 2;
  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1;
    if (compute_first) {
      compute_tile(cur);
      move_tiles(kt, cur);
    } else {
      move_tiles(kt, cur);
      compute_tile(cur);
    }
    __syncthreads();
  }

  // epilogue: lane holds column n = l32 of each 32x32 tile, rows (r/4)*8 + lhalf*4 + r%4
  if constexpr (FUSED) {
    // The update applied to the tile while g and Hz are still in registers (same arithmetic as update_kernel, Hessian
    // power 1).  Element (m, n) is parameter m*ldc + n of the layer's W block; W is made of whole tiles, so no
    // element is out of range, and offsets inside the block fit 32 bits.
    const FuseArgs& f = a.fu;
    // bias corrections of this worker, read from the kernel-argument block by a scalar load (indexing the by-value
    // argument with a variable would copy it to scratch memory)
    typedef const char __attribute__((address_space(4)))* karg_bytes;
    typedef const float __attribute__((address_space(4)))* karg_floats;
    const karg_bytes ka = (karg_bytes)__builtin_amdgcn_kernarg_segment_ptr();
    const karg_floats bc = (karg_floats)(ka + offsetof(GemmArgs, fu) + offsetof(FuseArgs, sc));
    const float ib1 = bc[worker], ib2 = bc[DW_MAX_K + worker];
    static_assert(offsetof(UpdateScalars, inv_bc2) == DW_MAX_K * sizeof(float), "inv_bc2 follows inv_bc1");
    float* gl = reinterpret_cast<float*>(smem) + wave * fused_update_lds_floats();     // free after the main loop
    float nsum = 0.f;
    if constexpr (FM == 1)
      fused_probe_sum_wave_tile<TM>(racc, gl, f, (int64_t)worker * a.c_wstride, a.ldc, row0 + wm0, col0 + wn0,
                                    zb + (a.z_off >> 5), lane);
    else {
      FusedUpdateTile<TM, true, FM == 2 ? 1 : 0> upd(f, (int64_t)worker * a.c_wstride, a.ldc, row0 + wm0, col0 + wn0,
                                                    zb + (a.z_off >> 5), nullptr, lane);
      nsum = upd.run(acc, racc, racc, gl, ib1, ib2);
    }
    // squared distance of the tile's new parameters to the centre: one slot per (worker, tile)
    double ws = (double)nsum;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) ws += __shfl_xor(ws, off);
    __syncthreads();                                          // everybody is done with the operand tiles in LDS
    double* red = reinterpret_cast<double*>(smem);
    if (lane == 0) red[wave] = ws;
    __syncthreads();
    if (tid == 0 && f.dist) {
      double t = 0.0;
#pragma unroll
      for (int w = 0; w < NT / 64; ++w) t += red[w];
      f.partials[(int64_t)worker * f.part_stride + f.part_base + tile] = t;
    }
  } else if (EPI == EPI_WGRAD && TN == 2 && BM == 128 && BN == 256 && a.M % BM == 0 && a.N % BN == 0) {
    // Large weight gradient stored as it is (gW and HzW, fp32): through the same per-wave LDS regions as the fused
    // epilogue, so that the stores are float4 of 256-byte row pieces; non-temporal, the update kernel reads
    // them once.
    constexpr int PR = 72;
    float* gl = reinterpret_cast<float*>(smem) + wave * (2 * 32 * PR);
    float* hl = gl + 32 * PR;
    const int brow = lane >> 4, bcol = (lane & 15) * 4;
    float* Cw = reinterpret_cast<float*>(a.C) + (int64_t)worker * a.c_wstride;
    float* RCw = reinterpret_cast<float*>(a.RC) + (int64_t)worker * a.c_wstride;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = (r >> 2) * 8 + lhalf * 4 + (r & 3), col = j * 32 + l32;
          gl[row * PR + col] = acc[i][j][r];
          hl[row * PR + col] = racc[i][j][r];
        }
#pragma unroll
      for (int b = 0; b < 8; ++b) {
        const int64_t e = (int64_t)(row0 + wm0 + i * 32 + b * 4 + brow) * a.ldc + (col0 + wn0 + bcol);
        nt_store4(Cw + e, *reinterpret_cast<const float4*>(gl + (b * 4 + brow) * PR + bcol));
        nt_store4(RCw + e, *reinterpret_cast<const float4*>(hl + (b * 4 + brow) * PR + bcol));
      }
    }
  } else if (EPI == EPI_RELU || EPI == EPI_MASK) {
    // bf16 outputs: through LDS, 16-byte stores of whole row pieces (see dw_gemm_epi.h)
    char* wl = reinterpret_cast<char*>(smem) + wave * epi_bf16_lds_bytes(TN);
    const uint16_t* msk = EPI == EPI_MASK ? reinterpret_cast<const uint16_t*>(a.mask_src) + (int64_t)worker * a.mask_wstride : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      floatx16 cv[TN], rcv[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if (EPI == EPI_RELU) {
          const int n = col0 + wn0 + j * 32 + l32;
          float bias = 0.f, cz = 0.f;
          if (n < a.N) {
            bias = a.bias[(int64_t)worker * a.bias_wstride + n];
            const int64_t bi = a.zb_off + n;
            cz = ((zb[bi >> 5] >> (bi & 31)) & 1u) ? 1.f : -1.f;
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float c = acc[i][j][r] + bias, rc = racc[i][j][r] + cz;
            const bool on = c > 0.f;
            cv[j][r] = on ? c : 0.f; rcv[j][r] = on ? rc : 0.f;
          }
        } else {
          cv[j] = acc[i][j]; rcv[j] = racc[i][j];
        }
      }
      const int rbase = row0 + wm0 + i * 32, cbase = col0 + wn0;
      epi_bf16_rows_out<TN, EPI == EPI_MASK>(wl, cv, rcv, lane, reinterpret_cast<uint16_t*>(a.C), reinterpret_cast<uint16_t*>(a.RC),
                                             (int64_t)worker * a.c_wstride + (int64_t)rbase * a.ldc + cbase, a.ldc,
                                             a.M - rbase, a.N - cbase, msk, (int64_t)rbase * a.ld_mask + cbase, a.ld_mask);
    }
  } else {
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
          reinterpret_cast<uint16_t*>(a.C)[o] = f32_to_bf16_rne(on ? c : 0.f);
          reinterpret_cast<uint16_t*>(a.RC)[o] = f32_to_bf16_rne(on ? rc : 0.f);
        } else if (EPI == EPI_LINEAR) {
          reinterpret_cast<float*>(a.C)[o] = c + bias;
          reinterpret_cast<float*>(a.RC)[o] = rc + cz;
        } else if (EPI == EPI_MASK) {
          const uint16_t* msk = reinterpret_cast<const uint16_t*>(a.mask_src) + (int64_t)worker * a.mask_wstride;
          const uint16_t mv = msk[(int64_t)m * a.ld_mask + n];
          const bool on = mv != 0 && !(mv & 0x8000u);     // stored activation > 0
          reinterpret_cast<uint16_t*>(a.C)[o] = f32_to_bf16_rne(on ? c : 0.f);
          reinterpret_cast<uint16_t*>(a.RC)[o] = f32_to_bf16_rne(on ? rc : 0.f);
        } else {
          reinterpret_cast<float*>(a.C)[o] = c;
          reinterpret_cast<float*>(a.RC)[o] = rc;
        }
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

// Weight gradient of a layer for two Hutchinson probes of one minibatch at once, with the update in its epilogue:
// g = X^T Y as above, Hz_p = RXp^T Y + X^T RYp along the earlier probe's z and Hz = RX^T Y + X^T RY along the later
// one's, D = (z_p*Hz_p + z*Hz) / 2 (Section IV-B with two samples of the estimate).  X = d_l and Y = a_{l-1} are
// staged once for both probes and the parameters, moments and bf16 copy are moved once, where one launch per probe
// reads the operands twice and carries the first probe's z*Hz through memory.  Tiles of BM x 128 with BM/32 x 2 waves
// of 32 x 64 (three accumulator sets of 32 registers), six operand tiles of PK k per stage.  Launched with BM = 128,
// PK = 32: 8 waves, 120 KB of LDS, one block per compute unit.  KWHOLE: a minibatch of whole k-tiles, unconditional
// loads and LDS stores in the main loop.  Measured on a 4096 x 4096 layer of 16 workers, bounds checks still in: 2.38 ms, the multiplications alone 1.36 ms (1.37 Tflop: 40 % of the matrix cores' peak; operand reads from LDS take
// as many cycles as the MFMAs) and the update alone 1.39 ms, so the two phases of a block mostly follow each other;
// BM = 64, PK = 16 puts two blocks of 4 waves on a unit, which do overlap, but with more LDS traffic per product the
// launch takes 2.64 ms.
template <bool HAS_RY, int BM, int PK, bool KWHOLE>
__global__ __launch_bounds__(BM * 4, BM == 128 ? 1 : 2) void fused_wgrad_pair_bf16(GemmArgs a) {
  constexpr int NT = BM * 4, BN = 128, WM = BM / 32, KS = PK / 16;
  const int tiles_m = a.M / BM, tiles_n = a.N / BN;
  const int tiles = tiles_m * tiles_n;
  const int per_xcd = gridDim.x >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);     // an XCD walks a contiguous range
  const int slot = logical / tiles;
  if (slot >= active_count(a.active_mask, a.k)) return;
  const int worker = nth_active_worker(a.active_mask, slot);
  const int tile = logical - slot * tiles;
  if (blockIdx.x < 256) {                                    // first block of every compute unit: staggered start
    const int ph = (blockIdx.x >> 3) & 15;
    for (int i = 0; i < ph; ++i) __builtin_amdgcn_s_sleep(127);
  }
  int tm = tile % tiles_m, tn = tile / tiles_m;
  constexpr int GR = 1024 / BM;                              // groups of 1024 x 1024 share their operand panels in L2
  if (tiles_m % GR == 0) {
    const int g = tile / (GR * tiles_n), r = tile - g * (GR * tiles_n);
    tn = r / GR; tm = g * GR + r % GR;
  }
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % WM) * 32, wn0 = (wave / WM) * 64;

  using TX = Tile<BM, NT, false, PK>;                        // every operand is [k][row]; a thread moves at most one
  using TY = Tile<BN, NT, false, PK>;                        // 16-byte unit of each tile
  static_assert(TX::UPT == 1 && TY::UPT == 1, "one unit per thread and tile");
  constexpr int X_ELEMS = TX::LDS_ELEMS, Y_ELEMS = TY::LDS_ELEMS, STAGE = 3 * X_ELEMS + 3 * Y_ELEMS;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  // tiles of a stage: X, RXp, RX, then Y, RYp, RY
  auto xt = [&](int st, int t) { return smem + st * STAGE + t * X_ELEMS; };
  auto yt = [&](int st, int t) { return smem + st * STAGE + 3 * X_ELEMS + t * Y_ELEMS; };

  const int64_t xo = (int64_t)worker * a.x_wstride, yo = (int64_t)worker * a.y_wstride;
  const uint16_t* xsrc[3] = {reinterpret_cast<const uint16_t*>(a.X) + xo, reinterpret_cast<const uint16_t*>(a.RXp) + xo,
                             reinterpret_cast<const uint16_t*>(a.RX) + xo};
  const uint16_t* ysrc[3] = {reinterpret_cast<const uint16_t*>(a.Y) + yo,
                             HAS_RY ? reinterpret_cast<const uint16_t*>(a.RYp) + yo : nullptr,
                             HAS_RY ? reinterpret_cast<const uint16_t*>(a.RY) + yo : nullptr};
  TX tx; TY ty;
  tx.init(tid, a.ldx, row0, a.M);
  ty.init(tid, a.ldy, col0, a.N);
  constexpr int NY = HAS_RY ? 3 : 1;
  uint4 xr[3][1], yr[NY][1];

  floatx16 acc[1][2], raccp[1][2], racc[1][2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[0][j][r] = 0.f; raccp[0][j][r] = 0.f; racc[0][j][r] = 0.f; }
  float gb_acc = 0.f, hzb_acc = 0.f;

  const int nkt = (a.K + PK - 1) / PK;
  auto fetch = [&](int kt) {
#pragma unroll
    for (int t = 0; t < 3; ++t) tx.template load<KWHOLE>(xsrc[t], a.ldx, kt * PK, a.K, xr[t]);
#pragma unroll
    for (int t = 0; t < NY; ++t) ty.template load<KWHOLE>(ysrc[t], a.ldy, kt * PK, a.K, yr[t]);
  };
  auto stash = [&](int st, int kt) {
#pragma unroll
    for (int t = 0; t < 3; ++t) tx.template store<KWHOLE>(xt(st, t), xr[t], tid, kt * PK, a.K);
#pragma unroll
    for (int t = 0; t < NY; ++t) ty.template store<KWHOLE>(yt(st, t), yr[t], tid, kt * PK, a.K);
  };
  struct Frags { bf16x8 x, rxp, rx, y[2], ryp[2], ry[2]; };
  auto compute_tile = [&](int cur) {
    if (tn == 0 && tid < BM) {                               // bias gradients of the later probe (X is [k][m])
      const uint16_t* xs = xt(cur, 0);
      const uint16_t* rxs = xt(cur, 2);
#pragma unroll
      for (int kq = 0; kq < PK; ++kq) {
        gb_acc += bf2f(xs[kq * TX::LDR + tid]);
        hzb_acc += bf2f(rxs[kq * TX::LDR + tid]);
      }
    }
    Frags f[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      f[ks].x = frag<BM, false>(xt(cur, 0), wm0, ks, lane);
      f[ks].rxp = frag<BM, false>(xt(cur, 1), wm0, ks, lane);
      f[ks].rx = frag<BM, false>(xt(cur, 2), wm0, ks, lane);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        f[ks].y[j] = frag<BN, false>(yt(cur, 0), wn0 + j * 32, ks, lane);
        if (HAS_RY) {
          f[ks].ryp[j] = frag<BN, false>(yt(cur, 1), wn0 + j * 32, ks, lane);
          f[ks].ry[j] = frag<BN, false>(yt(cur, 2), wn0 + j * 32, ks, lane);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        acc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[ks].x, f[ks].y[j], acc[0][j], 0, 0, 0);
        raccp[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[ks].rxp, f[ks].y[j], raccp[0][j], 0, 0, 0);
        racc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[ks].rx, f[ks].y[j], racc[0][j], 0, 0, 0);
      }
      if (HAS_RY) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          raccp[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[ks].x, f[ks].ryp[j], raccp[0][j], 0, 0, 0);
          racc[0][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[ks].x, f[ks].ry[j], racc[0][j], 0, 0, 0);
        }
      }
    }
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto move_tiles = [&](int kt, int cur) {
    if (kt + 1 < nkt) stash(cur ^ 1, kt + 1);
    if (kt + 2 < nkt) fetch(kt + 2);
  };

  fetch(0);
  stash(0, 0);
  if (nkt > 1) fetch(1);
  __syncthreads();
  const bool compute_first = wave < NT / 128;                // half of the waves multiply first, half move first
  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1;
    if (compute_first) {
      compute_tile(cur);
      move_tiles(kt, cur);
    } else {
      move_tiles(kt, cur);
      compute_tile(cur);
    }
    __syncthreads();
  }

  const FuseArgs& f = a.fu;
  typedef const char __attribute__((address_space(4)))* karg_bytes;
  typedef const float __attribute__((address_space(4)))* karg_floats;
  const karg_bytes ka = (karg_bytes)__builtin_amdgcn_kernarg_segment_ptr();
  const karg_floats bc = (karg_floats)(ka + offsetof(GemmArgs, fu) + offsetof(FuseArgs, sc));
  const float ib1 = bc[worker], ib2 = bc[DW_MAX_K + worker];   // scalar loads from the kernel-argument block
  float* gl = reinterpret_cast<float*>(smem) + wave * fused_update_lds_floats(true);   // free after the main loop
  const int64_t zw0 = (int64_t)worker * a.z_stride + (a.z_off >> 5);
  FusedUpdateTile<1, true, 2> upd(f, (int64_t)worker * a.c_wstride, a.ldc, row0 + wm0, col0 + wn0, a.zbits + zw0,
                                  a.zbits_p + zw0, lane);
  const float nsum = upd.run(acc, racc, raccp, gl, ib1, ib2);
  double ws = (double)nsum;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) ws += __shfl_xor(ws, off);
  __syncthreads();                                           // everybody is done with the staging regions
  double* red = reinterpret_cast<double*>(smem);
  if (lane == 0) red[wave] = ws;
  __syncthreads();
  if (tid == 0 && f.dist) {
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < NT / 64; ++w) t += red[w];
    f.partials[(int64_t)worker * f.part_stride + f.part_base + tile] = t;
  }
  if (tn == 0 && tid < BM) {
    a.gb[(int64_t)worker * a.c_wstride + row0 + tid] = gb_acc;
    a.hzb[(int64_t)worker * a.c_wstride + row0 + tid] = hzb_acc;
  }
}

template <bool HAS_RY, bool KWHOLE>
static hipError_t launch_pair(const GemmArgs& a, hipStream_t s) {
  constexpr int BM = 128, PK = 32, NT = BM * 4;
  const int tiles = (a.M / BM) * (a.N / 128);
  const dim3 grid((unsigned)((tiles * active_count(a.active_mask, a.k) + 7) / 8 * 8)), block(NT);
  constexpr int tiles_b = 2 * 2 * 3 * (Tile<BM, NT, false, PK>::LDS_ELEMS + Tile<128, NT, false, PK>::LDS_ELEMS);
  constexpr int epi_b = (NT / 64) * fused_update_lds_floats(true) * 4;
  constexpr int smem = tiles_b > epi_b ? tiles_b : epi_b;
  static_assert(smem <= 160 * 1024, "LDS budget");
  auto kern = fused_wgrad_pair_bf16<HAS_RY, BM, PK, KWHOLE>;
  static LdsLimitOnce lds_limit;
  { const hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), smem); if (e != hipSuccess) return e; }
  hipLaunchKernelGGL(kern, grid, block, smem, s, a);
  return hipGetLastError();
}

template <int BM, int BN, int WM, int WN, bool XKC, bool YKC, bool RX, int RYM, int EPI, int FM = 0, int NTH = 512,
          bool KWHOLE = false>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s) {
  constexpr int NT = NTH;
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  const dim3 grid((unsigned)((tiles * active_count(a.active_mask, a.k) + 7) / 8 * 8)), block(NT);
  constexpr int XTH = RX ? NT / 2 : NT;
  constexpr int tiles_b = 2 * 2 * (Tile<BM, XTH, XKC>::LDS_ELEMS * (RX ? 2 : 1) +
                                   Tile<BN, NT, YKC>::LDS_ELEMS * (RYM != RY_NONE ? 2 : 1));
  // the fused weight-gradient epilogue passes g and Hz through LDS: per wave two arrays of 32 rows x 72 floats
  constexpr int epi_b = (EPI == EPI_WGRAD && BM == 128 && (BN == 256 || BN == 128)) ? (NT / 64) * 2 * 32 * 72 * 4 : 0;
  constexpr int out_b = (EPI == EPI_RELU || EPI == EPI_MASK) ? (NT / 64) * epi_bf16_lds_bytes(BN / WN / 32) : 0;
  constexpr int smem = tiles_b > epi_b ? (tiles_b > out_b ? tiles_b : out_b) : (epi_b > out_b ? epi_b : out_b);
  static_assert(smem <= 160 * 1024, "LDS budget");
  auto kern = dual_gemm_bf16<BM, BN, WM, WN, XKC, YKC, RX, RYM, EPI, FM, NTH, KWHOLE>;
  static LdsLimitOnce lds_limit;
  { const hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), smem); if (e != hipSuccess) return e; }
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

// Weight gradient that applies the update itself: 128 x 128 tiles and 256 threads (four waves of 64 x 64), two blocks
// per compute unit (2 x 80 KB of LDS, one wave of each per SIMD), so that one block's state traffic runs under the
// other's multiplications and neither's start-up and drain leaves the unit idle.  Own instances for the steps of
// several Hutchinson probes (FM 1: a probe before the last, 2: the last), so that the one-probe kernel keeps its
// registers.
static hipError_t launch_fused_wgrad(const GemmArgs& a, hipStream_t s) {
  if (a.fu.probe_mode == 3) {
    if (a.K % BK == 0) return a.RY ? launch_pair<true, true>(a, s) : launch_pair<false, true>(a, s);
    return a.RY ? launch_pair<true, false>(a, s) : launch_pair<false, false>(a, s);
  }
  if (a.fu.probe_mode == 1)
    return a.RY ? launch_one<128, 128, 2, 2, false, false, true, RY_MEM, EPI_WGRAD, 1, 256>(a, s)
                : launch_one<128, 128, 2, 2, false, false, true, RY_NONE, EPI_WGRAD, 1, 256>(a, s);
  if (a.fu.probe_mode == 2)
    return a.RY ? launch_one<128, 128, 2, 2, false, false, true, RY_MEM, EPI_WGRAD, 2, 256>(a, s)
                : launch_one<128, 128, 2, 2, false, false, true, RY_NONE, EPI_WGRAD, 2, 256>(a, s);
  if (a.K % BK == 0)                  // (the usual case: the one-probe kernel without bounds checks in its main loop)
    return a.RY ? launch_one<128, 128, 2, 2, false, false, true, RY_MEM, EPI_WGRAD, 0, 256, true>(a, s)
                : launch_one<128, 128, 2, 2, false, false, true, RY_NONE, EPI_WGRAD, 0, 256, true>(a, s);
  return a.RY ? launch_one<128, 128, 2, 2, false, false, true, RY_MEM, EPI_WGRAD, 0, 256>(a, s)
              : launch_one<128, 128, 2, 2, false, false, true, RY_NONE, EPI_WGRAD, 0, 256>(a, s);
}

}  // namespace b16

// The weight-gradient product of W[n_out][n_in] can apply the update in its epilogue (128 x 128 tiles, see
// launch_fused_wgrad) when W is made of whole tiles (rows are then whole 32-lane segments and sign-bit words),
// an averaging block is at most one segment and the Hessian power is 1.
bool gemm_bf16_wgrad_fusable(int n_out, int n_in, int k, int avg_block, float hpow, int64_t woff) {
  if (n_out % 128 != 0 || n_in % 128 != 0 || woff % 32 != 0 || avg_block > 32 || hpow != 1.0f) return false;
  if ((int64_t)n_out * n_in >= (1ll << 31)) return false;
  return (int64_t)(n_out / 128) * (n_in / 128) * k >= 512;
}
int gemm_bf16_wgrad_tiles(int n_out, int n_in, int /*n_samples*/) { return ((n_out + 127) / 128) * ((n_in + 127) / 128); }

hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  KernelScope ks(a.epi == EPI_WGRAD ? KC_GEMM_WGRAD : a.epi == EPI_MASK ? KC_GEMM_DGRAD : KC_GEMM_FWD, s);
  if (gemm_bf16_dma_ok(a)) return launch_gemm_bf16_dma(a, s);
  if (gemm_bf16_out_ok(a)) return launch_gemm_bf16_out(a, s);
  if (a.epi == EPI_WGRAD && a.fu.on) return b16::launch_fused_wgrad(a, s);
  if (a.N <= 32) return b16::launch_shape<256, 32, 8, 1>(a, s);
  if (a.M <= 32) return b16::launch_shape<32, 256, 1, 8>(a, s);
  const int64_t big_tiles = (int64_t)((a.M + 127) / 128) * ((a.N + 255) / 256) * a.k;
  if (big_tiles >= 256) return b16::launch_shape<128, 256, 2, 4>(a, s);
  return b16::launch_shape<64, 128, 2, 4>(a, s);
}

}  // namespace dw
