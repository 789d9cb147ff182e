// bf16 dual GEMM of the forward pass, large-tile path: tiles travel global -> LDS without passing through
// registers, and one wave per SIMD owns a 128 x 64 output tile with all 512 registers of its lanes.
//
// Same computation as dual_gemm_bf16 for the forward product of one layer and its directional derivative along
// z (Section IV-B): S = A W^T, RS = RA W^T + A V^T with V = z's W-part as +-1.  Block tile 128 x 256 x 32, four
// waves side by side along N: the two accumulator sets of a wave (4 x 2 MFMA tiles each) are 256 registers, which
// the compiler keeps in the accumulation registers, leaving the 256 vector registers to operands and addresses.
// A wave tile of 128 x 64 needs 20 LDS reads of 16 bytes per lane and k-tile against 24 for two waves of 64 x 64,
// and half as many +-1 expansions as 64 x 128 would.  With a single wave per SIMD nothing else hides a stall, so
// the k-loop is written as two straight-line regions per k-tile (one per k-step of 16) in which the multiplies of
// one k-step are interleaved, by scheduling groups, with the LDS reads, the sign expansions and the global loads
// that feed the next one; the loop body has no branch except a uniform one around the sign-bit fetch, placed right
// after the barrier, and the last STAGES k-tiles (nothing left to fetch) run in a loop of their own.
// `global_load_lds_dwordx4` writes each lane's 16 bytes straight into LDS (lane l of a wave lands at base + 16 l),
// so tiles in flight cost no registers and four k-tiles are in flight or resident.  Because a wave's 64 x 16
// bytes land contiguously, tiles cannot be padded; bank conflicts are avoided by an XOR swizzle applied when
// choosing which 16 bytes a lane fetches: rows are 64 bytes, 16-byte slot = k-chunk ^ ((row >> 2) & 3).
// The +-1 operand V is never staged as a matrix: every fourth k-tile the sign bits of the next 128 k (16 bytes per
// row, 4 KB per block) are fetched into a two-deep ring; a lane reads its 32 bits of a k-tile one k-tile ahead and
// expands 8 of them to bf16 +-1 in registers just before the multiply.
//
// Requirements (otherwise the caller uses dual_gemm_bf16): see gemm_bf16_dma_ok.  Rows beyond M are clamped to the
// last valid row (their products are discarded).
#include <type_traits>

#include "dw_internal.h"
#include "dw_gemm_epi.h"

namespace dw {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

namespace b16d {

constexpr int BM = 128, BN = 256, BK = 32, NT = 256, NW = NT / 64;
constexpr int WM = 1, WN = 4, TM = 4, TN = 2;           // wave tile 128 x 64
constexpr int STAGES = 4;
constexpr int ZGROUP = 4;                               // k-tiles covered by one fetch of sign bits (16 bytes per row)

// cache policy of the weight-tile loads: non-temporal.  A weight panel is read by the four row tiles of its column
// tile at about the same time and never again in the launch, while the activation panels are re-read by every
// column tile: keeping the weights from displacing them is worth 3 % (measured).
constexpr int kStreamed = 2;

typedef __attribute__((address_space(3))) void* lds_void;
typedef __attribute__((address_space(3))) const char* lds_char;
typedef __attribute__((address_space(1))) const void* glb_void;

// eight bf16 values +-1 from the eight sign bits of b (b < 256; bit set -> +1 = 0x3F80, clear -> -1 = 0xBF80).  Two
// values share a dword: bit 2q of b goes to bit 15 and bit 2q+1 to bit 31 by two shifts of the whole byte (no other
// bit of b can land on 15 or 31; the compiler makes one multiply of the two), which one AND-XOR then folds into the
// pattern of two -1.  (Measured in this loop, each against this form on one box: a form with fewer and cheaper
// instructions, the loads' addresses as scalar base + 32-bit lane offset, and the pointer arithmetic moved into the
// first k-step were all 2 to 5 % slower: once the vector instructions are spread over both k-steps, see `expand`,
// their count is not what limits the loop, and the schedule is touchy.)
__device__ __forceinline__ bf16x8 pm1_x8(uint32_t b) {
  uint4 o;
  o.x = 0xBF80BF80u ^ (((b << 15) | (b << 30)) & 0x80008000u);
  o.y = 0xBF80BF80u ^ (((b << 13) | (b << 28)) & 0x80008000u);
  o.z = 0xBF80BF80u ^ (((b << 11) | (b << 26)) & 0x80008000u);
  o.w = 0xBF80BF80u ^ (((b << 9) | (b << 24)) & 0x80008000u);
  return __builtin_bit_cast(bf16x8, o);
}

// wait until at most n of this wave's vector-memory operations are outstanding (n < 64) and all of its LDS
// reads have returned (so that, after the barrier that follows, the stage they read may be overwritten)
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
}

// wait until all of this wave's LDS reads have returned (vector-memory operations are not waited for)
__device__ __forceinline__ void wait_lds() {
  __builtin_amdgcn_s_waitcnt((63 & 15) | ((63 >> 4) << 14) | (0x7 << 4) | (0x0 << 8));
}

// ---- one operand tile of R rows x 32 k, memory [row][k] -> LDS rows of 64 bytes, chunk c (1 KB) = rows 16c..16c+15
template <int R>
struct DmaTile {
  static constexpr int BYTES = R * BK * 2;
  static constexpr int CPW = BYTES / 1024 / NW;           // chunks per wave
  static_assert(BYTES % (1024 * NW) == 0, "every wave moves the same number of chunks");
  __device__ static __forceinline__ int swz(int row) { return (row >> 2) & 3; }
  // global element offset (at k0 = 0) of the 16 bytes lane `lane` moves for chunk c (they land at c*1024 + 16*lane)
  __device__ static __forceinline__ int64_t map(int c, int lane, int r0, int Rmax, int ld) {
    const int row = c * 16 + (lane >> 2), p = lane & 3;
    const int q = p ^ swz(row);                           // logical k-chunk stored in physical slot p
    int gr = r0 + row; gr = gr < Rmax ? gr : Rmax - 1;
    return (int64_t)gr * ld + q * 8;
  }
  // MFMA operand: 8 consecutive k of row row0 + lane%32, k-chunk ks*2 + lane/32
  __device__ static __forceinline__ bf16x8 frag(const char* lds, int row0, int ks, int lane) {
    const int row = row0 + (lane & 31), q = ks * 2 + (lane >> 5);
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(lds + row * 64 + ((q ^ swz(row)) << 4)));
  }
};

// ---- one operand tile of 32 k x R rows stored k-major in memory ([k][row], the weight matrix in the data gradient):
// LDS keeps it as it lies, 32 k-rows of R*2 bytes, chunk c (1 KB) = k-rows 2c and 2c+1 (R = 256).  The MFMA operand
// (8 consecutive k of one row) is produced by the LDS transpose read `ds_read_b64_tr_b16`: within 16 lanes, lane i
// receives element i%4 of the 8-byte pieces addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4.  The four k-rows a
// 16-lane group addresses are a multiple of 256 bytes apart, so the 32-byte piece ("pair" of 16-byte slots) a group
// reads is XOR-swizzled by 2*(k%4): the 32 lanes of a pass then cover 256 consecutive bytes of bank space.
template <int R>
struct DmaTileK {
  static_assert(R == 256, "two k-rows per 1 KB chunk");
  static constexpr int BYTES = R * BK * 2;
  static constexpr int CPW = BYTES / 1024 / NW;
  // global element offset (at k0 = 0) of the 16 bytes lane `lane` moves for chunk c (they land at c*1024 + 16*lane)
  __device__ static __forceinline__ int64_t map(int c, int lane, int r0, int ld) {
    const int k = 2 * c + (lane >> 5), ps = lane & 31;      // k-row, physical slot
    const int lp = (ps >> 1) ^ ((k & 3) << 1);              // logical pair held by physical pair ps/2
    return (int64_t)k * ld + r0 + ((lp << 1) | (ps & 1)) * 8;
  }
  // The transpose reads are written as inline assembly: behind the compiler's intrinsic they would be preceded by a
  // wait for every outstanding global -> LDS load (it cannot tell that they read other stages), which serialises the
  // pipeline.  The price: the compiler does not know when their results arrive.  The kernel waits for its LDS reads
  // explicitly (the waits it needs anyway before a barrier or a multiply) and then passes the registers through
  // `settle`, which pins every use behind that wait.  Between the read and `settle` the two halves stay the
  // read's own output registers (Raw): nothing is computed from them, not even the 16-byte operand they form, so
  // the compiler has no reason to copy a register whose value has not arrived yet.
  struct Raw { uint2 lo, hi; };
  __device__ static __forceinline__ Raw frag_raw(const char* lds, int row0, int ks, int lane) {
    const int s = lane & 15, kq = s >> 2;
    const int k = ks * 16 + (lane >> 5) * 8 + kq;           // k%4 == kq; the second read is 4 k-rows further on
    const int lp = (row0 >> 4) + ((lane >> 4) & 1);
    const uint32_t addr = (uint32_t)(uintptr_t)(lds_char)(lds + k * (R * 2) + ((lp ^ (kq << 1)) << 5) + (s & 3) * 8);
    Raw r;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r.lo) : "v"(addr));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(4 * R * 2));
    return r;
  }
  __device__ static __forceinline__ bf16x8 settle(Raw& r) {  // after the wait for this wave's LDS reads
    asm volatile("" : "+v"(r.lo), "+v"(r.hi));
    return __builtin_bit_cast(bf16x8, make_uint4(r.lo.x, r.lo.y, r.hi.x, r.hi.y));
  }
};

// DGRAD = false: forward product, Y = W stored [n][k], epilogue bias + ReLU.
// DGRAD = true: data gradient, Y = W stored [k][n] (k = the layer's outputs), sign bits from the transposed copy of
// z's W-part (bit (n, k) at z_off + n*K + k), epilogue = the ReLU mask of the layer below.
// RONLY: only the R-companion RC is computed and stored (a later Hutchinson probe of the same minibatch: the plain
// product C is in memory already, and its stored sign is the forward product's ReLU mask).
template <bool HAS_RX, bool DGRAD, bool RONLY = false>
__global__ __launch_bounds__(NT) void dual_gemm_bf16_dma(GemmArgs a) {
  // the R-only form of a layer without an R-operand (the first layer) is X V^T alone: W is not even loaded
  constexpr bool NO_Y = RONLY && !HAS_RX;
  using TX = DmaTile<BM>;
  using TY = typename std::conditional<DGRAD, DmaTileK<BN>, DmaTile<BN>>::type;
  constexpr int X_B = TX::BYTES, Y_B = TY::BYTES;
  constexpr int OFF_RX = X_B;
  constexpr int OFF_Y = X_B * (HAS_RX ? 2 : 1);
  constexpr int STAGE_B = OFF_Y + Y_B;
  constexpr int OFF_Z = STAGE_B * STAGES;                   // ring of two sign-bit groups, [256 rows][16 bytes] each
  constexpr int Z_B = BN * 16;
  // vector-memory operations every wave issues per k-tile; the sign-bit fetches (one more operation per wave every
  // fourth k-tile) are left out: counts are only used as "at most n outstanding", operations complete in order, so
  // an uncounted operation makes a wait slightly longer, never too short
  constexpr int LPT = TX::CPW * (HAS_RX ? 2 : 1) + (NO_Y ? 0 : TY::CPW);

  const int tiles_m = (a.M + BM - 1) / BM;
  const int tiles = tiles_m * (a.N / BN);
  const int per_xcd = gridDim.x >> 3;                       // XCD-aware order, see dual_gemm_bf16
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  const int slot = logical / tiles;                         // which of the active workers
  if (slot >= active_count(a.active_mask, a.k)) return;
  const int worker = nth_active_worker(a.active_mask, slot);
  const int tile = logical - slot * tiles;
  const int tm = tile % tiles_m, tn = tile / tiles_m;
  const int row0 = tm * BM, col0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % WM) * (BM / WM), wn0 = (wave / WM) * (BN / WN);
  const int l32 = lane & 31, lhalf = lane >> 5;

  extern __shared__ __attribute__((aligned(1024))) char smem[];

  const uint16_t* X = reinterpret_cast<const uint16_t*>(a.X) + (int64_t)worker * a.x_wstride;
  const uint16_t* RX = HAS_RX ? reinterpret_cast<const uint16_t*>(a.RX) + (int64_t)worker * a.x_wstride : nullptr;
  const uint16_t* Y = reinterpret_cast<const uint16_t*>(a.Y) + (int64_t)worker * a.y_wstride;
  const uint32_t* zb = DGRAD ? a.zbits_t + (int64_t)worker * a.zt_stride : a.zbits + (int64_t)worker * a.z_stride;

  // per-wave source pointers (k0 = 0) of the chunks this wave moves
  const uint16_t* gx[TX::CPW]; const uint16_t* grx[TX::CPW]; const uint16_t* gy[TY::CPW];
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);  // wave index as a scalar: LDS targets are per wave
#pragma unroll
  for (int c = 0; c < TX::CPW; ++c) {
    const int64_t go = TX::map(wave * TX::CPW + c, lane, row0, a.M, a.ldx);
    gx[c] = X + go; grx[c] = HAS_RX ? RX + go : nullptr;
  }
#pragma unroll
  for (int c = 0; c < TY::CPW; ++c) {
    if constexpr (DGRAD) gy[c] = Y + DmaTileK<BN>::map(wave * TY::CPW + c, lane, col0, a.ldy);
    else gy[c] = Y + DmaTile<BN>::map(wave * TY::CPW + c, lane, col0, a.N, a.ldy);
  }
  const int64_t y_step = DGRAD ? (int64_t)BK * a.ldy : BK;  // elements from one k-tile of Y to the next
  // sign bits: wave w fetches rows 64w..64w+63 of the tile, 16 bytes (128 k) per row and group
  const uint32_t* gz = zb + ((a.z_off + (int64_t)(col0 + (wave & 3) * 64 + lane) * a.K) >> 5);

  auto issue = [&](int kt, int st) {                        // start the loads of k-tile kt into LDS stage st
    char* base = smem + st * STAGE_B;
#pragma unroll
    for (int c = 0; c < TX::CPW; ++c) {
      __builtin_amdgcn_global_load_lds((glb_void)(gx[c] + (int64_t)kt * BK), (lds_void)(base + (wave_u * TX::CPW + c) * 1024), 16, 0, 0);
      if (HAS_RX)
        __builtin_amdgcn_global_load_lds((glb_void)(grx[c] + (int64_t)kt * BK), (lds_void)(base + OFF_RX + (wave_u * TX::CPW + c) * 1024), 16, 0, 0);
    }
    if constexpr (!NO_Y) {
#pragma unroll
      for (int c = 0; c < TY::CPW; ++c)
        __builtin_amdgcn_global_load_lds((glb_void)(gy[c] + kt * y_step), (lds_void)(base + OFF_Y + (wave_u * TY::CPW + c) * 1024), 16, 0, kStreamed);
    }
  };

  floatx16 acc[TM][TN], racc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc[i][j][r] = 0.f; racc[i][j][r] = 0.f; }

  struct Frags { bf16x8 xa[TM], rxa[TM], yb[TN], ryb[TN]; typename DmaTileK<BN>::Raw yraw[TN]; };
  uint32_t zw[TN], zn[TN];                                  // this lane's 32 sign bits of the current and of the next k-tile, per column tile
  auto read_frags = [&](Frags& f, int st, int ks) {
    const char* base = smem + st * STAGE_B;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      f.xa[i] = TX::frag(base, wm0 + i * 32, ks, lane);
      if (HAS_RX) f.rxa[i] = TX::frag(base + OFF_RX, wm0 + i * 32, ks, lane);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if constexpr (DGRAD) f.yraw[j] = TY::frag_raw(base + OFF_Y, wn0 + j * 32, ks, lane);
      else if constexpr (!NO_Y) f.yb[j] = TY::frag(base + OFF_Y, wn0 + j * 32, ks, lane);
    }
  };
  auto settle = [&](Frags& f) {                             // after a wait for this wave's LDS reads
    if constexpr (DGRAD) {
#pragma unroll
      for (int j = 0; j < TN; ++j) f.yb[j] = TY::settle(f.yraw[j]);
    }
  };
  auto read_bits = [&](int kt) {
    const char* zbase = smem + OFF_Z + ((kt / ZGROUP) & 1) * Z_B + (kt & (ZGROUP - 1)) * 4;
#pragma unroll
    for (int j = 0; j < TN; ++j) zn[j] = *reinterpret_cast<const uint32_t*>(zbase + (wn0 + j * 32 + l32) * 16);
  };
  auto take_bits = [&]() {
#pragma unroll
    for (int j = 0; j < TN; ++j) zw[j] = zn[j];
  };
  auto expand = [&](Frags& f, int ks) {                     // V operand of k-step ks: byte ks*2 + lane/32 of the tile's word
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      f.ryb[j] = pm1_x8((zw[j] >> ((ks * 2 + lhalf) * 8)) & 0xFFu);
      // the expansion stays where it is written: left alone, the compiler moves it down to the multiplies that use it,
      // past the barrier, where all of a k-tile's vector arithmetic then crowds one k-step's issue slots
      uint4 pin = __builtin_bit_cast(uint4, f.ryb[j]);
      asm volatile("" : "+v"(pin.x), "+v"(pin.y), "+v"(pin.z), "+v"(pin.w));
      f.ryb[j] = __builtin_bit_cast(bf16x8, pin);
    }
  };
  auto multiply = [&](Frags& f) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        if (!RONLY) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.xa[i], f.yb[j], acc[i][j], 0, 0, 0);
    if (HAS_RX) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          racc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.rxa[i], f.yb[j], racc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        racc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.xa[i], f.ryb[j], racc[i][j], 0, 0, 0);
  };

  const int nkt = a.K / BK;                                 // a multiple of 4, at least 4
  __builtin_amdgcn_global_load_lds((glb_void)gz, (lds_void)(smem + OFF_Z + wave_u * 1024), 16, 0, 0);   // bits of k-tiles 0..3
#pragma unroll
  for (int t = 0; t < STAGES; ++t) issue(t, t);
  wait_vm<LPT * (STAGES - 1)>();
  __syncthreads();
  Frags f0, f1;
  read_bits(0);
  read_frags(f0, 0, 0);
  __builtin_amdgcn_s_waitcnt(15 | (3 << 14) | (0x7 << 4) | (0x0 << 8));
  settle(f0);
  take_bits();
  expand(f0, 0);
  read_bits(1);
  __builtin_amdgcn_s_waitcnt(15 | (3 << 14) | (0x7 << 4) | (0x0 << 8));

  // Scheduling groups: after every multiply, one LDS read or one global load (while there are any) and two vector
  // instructions (address arithmetic, sign expansion) of the code that prepares the next k-step.
  constexpr int N_MFMA = TM * TN * ((HAS_RX ? 3 : 2) - (RONLY ? 1 : 0));   // multiplies per k-step
  constexpr int N_DS = TM * (HAS_RX ? 2 : 1) + (NO_Y ? 0 : TN);   // operand reads from LDS per k-step
  auto interleave = [&](auto n_vmem_, auto n_ds_) {
    constexpr int n_vmem = decltype(n_vmem_)::value, n_ds = decltype(n_ds_)::value;
#pragma unroll
    for (int q = 0; q < N_MFMA; ++q) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      if (q < n_vmem) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
      else if (q < n_vmem + n_ds) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
    }
  };
  using no_vmem = std::integral_constant<int, 0>;
  using tile_vmem = std::integral_constant<int, LPT>;
  using frag_ds = std::integral_constant<int, N_DS>;
  using frag_bits_ds = std::integral_constant<int, N_DS + TN>;
  int st = 0, kt = 0;
  for (; kt + STAGES < nkt; ++kt) {
    const int st_next = st + 1 == STAGES ? 0 : st + 1;
    read_frags(f1, st, 1);
    expand(f1, 1);
    multiply(f0);
    interleave(no_vmem{}, frag_ds{});
    __builtin_amdgcn_sched_barrier(0);
    wait_vm<LPT * (STAGES - 2)>();
    settle(f1);
    __syncthreads();
    if (((kt + STAGES) & (ZGROUP - 1)) == 0) {              // k-tile kt+STAGES opens a group of sign bits
      const int zg = (kt + STAGES) / ZGROUP;
      __builtin_amdgcn_global_load_lds((glb_void)(gz + zg * 4), (lds_void)(smem + OFF_Z + (zg & 1) * Z_B + wave_u * 1024), 16, 0, 0);
    }
    issue(kt + STAGES, st);
    take_bits(); read_bits(kt + 2); read_frags(f0, st_next, 0); expand(f0, 0);
    multiply(f1);
    interleave(tile_vmem{}, frag_bits_ds{});
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (DGRAD) { wait_lds(); settle(f0); }
    st = st_next;
  }
  for (; kt < nkt; ++kt) {                                  // the last STAGES k-tiles: nothing left to fetch
    const int st_next = st + 1 == STAGES ? 0 : st + 1;
    read_frags(f1, st, 1);
    expand(f1, 1);
    multiply(f0);
    __builtin_amdgcn_sched_barrier(0);
    wait_vm<0>();
    settle(f1);
    __syncthreads();
    if (kt + 1 < nkt) { take_bits(); if (kt + 2 < nkt) read_bits(kt + 2); read_frags(f0, st_next, 0); expand(f0, 0); }
    multiply(f1);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (DGRAD) { wait_lds(); settle(f0); }
    st = st_next;
  }
  __syncthreads();                                          // the epilogue reuses the stages as its staging area

  // epilogue.  Forward: bias, R-bias (the bias part of z), ReLU.  Data gradient: the ReLU mask of the layer below,
  // applied while the rows leave.  The two bf16 outputs go through LDS (free after the barrier above) so that they
  // leave as 16-byte stores of whole row pieces (see dw_gemm_epi.h)
  char* wl = smem + wave * epi_bf16_lds_bytes(TN);
  const uint16_t* msk = DGRAD ? reinterpret_cast<const uint16_t*>(a.mask_src) + (int64_t)worker * a.mask_wstride
                        : RONLY ? reinterpret_cast<const uint16_t*>(a.C) + (int64_t)worker * a.c_wstride : nullptr;
  const int ld_msk = DGRAD ? a.ld_mask : a.ldc;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    floatx16 cv[TN], rcv[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if constexpr (DGRAD) {
        cv[j] = acc[i][j]; rcv[j] = racc[i][j];
      } else {
        const int n = col0 + wn0 + j * 32 + l32;
        const float bias = a.bias[(int64_t)worker * a.bias_wstride + n];
        const int64_t bi = a.zb_off + n;
        const float cz = ((zb[bi >> 5] >> (bi & 31)) & 1u) ? 1.f : -1.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float c = acc[i][j][r] + bias, rc = racc[i][j][r] + cz;
          const bool on = RONLY || c > 0.f;                 // (R-only: masked by the stored activation as the row leaves)
          cv[j][r] = on ? c : 0.f; rcv[j][r] = on ? rc : 0.f;
        }
      }
    }
    const int rbase = row0 + wm0 + i * 32, cbase = col0 + wn0;
    epi_bf16_rows_out<TN, DGRAD || RONLY, !RONLY>(wl, cv, rcv, lane, reinterpret_cast<uint16_t*>(a.C),
                                                  reinterpret_cast<uint16_t*>(a.RC),
                                                  (int64_t)worker * a.c_wstride + (int64_t)rbase * a.ldc + cbase, a.ldc,
                                                  a.M - rbase, a.N - cbase, msk, (int64_t)rbase * ld_msk + cbase, ld_msk);
  }
}

template <bool RX, bool DGRAD, bool RONLY = false>
static hipError_t launch_one(const GemmArgs& a, hipStream_t s) {
  const int tiles = ((a.M + BM - 1) / BM) * (a.N / BN);
  const dim3 grid((unsigned)((tiles * active_count(a.active_mask, a.k) + 7) / 8 * 8)), block(NT);
  constexpr int smem = (BM * BK * 2 * (RX ? 2 : 1) + BN * BK * 2) * STAGES + 2 * BN * 16;
  static_assert(smem <= 160 * 1024, "LDS budget");
  auto kern = dual_gemm_bf16_dma<RX, DGRAD, RONLY>;
  static LdsLimitOnce lds_limit;
  { const hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(kern), smem); if (e != hipSuccess) return e; }
  hipLaunchKernelGGL(kern, grid, block, smem, s, a);
  return hipGetLastError();
}

}  // namespace b16d

bool gemm_bf16_dgrad_dma_shape_ok(int batch, int n_out, int n_in, int k, int64_t woff) {
  if (batch < 128 || n_in % 256 != 0 || n_out % 128 != 0 || woff % 128 != 0) return false;
  return (int64_t)((batch + 127) / 128) * (n_in / 256) * k >= 256;
}

// true when the large-tile DMA kernel can take this product: the forward product of a hidden layer (ReLU
// epilogue) or the data gradient through a layer (mask epilogue) that fills the chip, with whole 256-column tiles
// and rows of z (for the data gradient: of its transposed copy) that 16-byte loads can address
bool gemm_bf16_dma_ok(const GemmArgs& a) {
  const bool fwd = a.epi == EPI_RELU && a.y_kcontig && a.K == a.ldy;
  const bool dgrad = a.epi == EPI_MASK && !a.y_kcontig && a.RX && a.zbits_t && a.N == a.ldy && a.ld_mask % 8 == 0 &&
                     a.zt_stride % 4 == 0 && (reinterpret_cast<uintptr_t>(a.zbits_t) & 15u) == 0;
  if (!(fwd || dgrad) || !a.ry_bits || !a.x_kcontig) return false;
  if (a.M < 128 || a.N % 256 != 0 || a.K % 128 != 0) return false;
  if (a.ldx % 32 != 0 || a.ldc % 8 != 0) return false;
  if ((int64_t)((a.M + 127) / 128) * (a.N / 256) * a.k < 256) return false;
  if (a.z_off % 128 != 0 || a.z_stride % 4 != 0 || (reinterpret_cast<uintptr_t>(a.zbits) & 15u) != 0) return false;
  return true;
}

hipError_t launch_gemm_bf16_dma(const GemmArgs& a, hipStream_t s) {
  if (a.epi == EPI_MASK) return a.r_only ? b16d::launch_one<true, true, true>(a, s) : b16d::launch_one<true, true>(a, s);
  if (a.RX) return a.r_only ? b16d::launch_one<true, false, true>(a, s) : b16d::launch_one<true, false>(a, s);
  return a.r_only ? b16d::launch_one<false, false, true>(a, s) : b16d::launch_one<false, false>(a, s);
}

}  // namespace dw
