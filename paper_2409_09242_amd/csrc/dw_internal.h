// Internal declarations shared by the host API and the kernel translation units of libdw.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "dw.h"

namespace dw {

constexpr int kUpdThreads = 256;      // threads per block of the streaming update / pull kernels
constexpr int kUpdQuads = 4;          // float4 groups per thread and worker
constexpr int64_t kUpdChunk = (int64_t)kUpdThreads * kUpdQuads * 4;   // parameters per block

// per-launch scalars of the fused AdaHessian update (Section IV-B), one entry per worker
struct UpdateScalars {
  float inv_bc1[DW_MAX_K];            // 1 / (1 - beta1^t_i)
  float inv_bc2[DW_MAX_K];            // 1 / (1 - beta2^t_i)
};

// where biases sit in the canonical layout (they are excluded from spatial averaging)
struct BiasRanges {
  int n;
  int64_t begin[DW_MAX_LAYERS];
  int64_t end[DW_MAX_LAYERS];
};

// parameter ranges whose update is applied elsewhere (inside the weight-gradient kernel): the streaming update
// skips them for active workers and only measures the distance to the centre for frozen ones
struct FusedRanges {
  int n;
  int64_t begin[DW_MAX_LAYERS];
  int64_t end[DW_MAX_LAYERS];
};

struct UpdateArgs {
  float* theta; float* m; float* v;   // [k][Pp]
  const float* g; const float* hz;    // [k][g_stride]
  const float* centre;                // [Pp]
  const uint32_t* zbits;              // [k][z_stride] sign bits of z
  uint16_t* wb16;                     // [k][Pp] bf16 copy of theta or nullptr
  double* partials;                   // [k][n_blocks] squared-distance partial sums
  int64_t P;                          // parameters per worker; only groups of four below P are touched
  int64_t Pp;                         // padded parameter count (multiple of 64), row stride of theta, m, v
  int64_t g_stride, z_stride;
  int k;
  int avg_block;                      // power of two, 1..256
  float lr, beta1, beta2, eps, hpow;
  int optimizer;                      // DW_OPT_*: AdaHessian, or a baseline's first-order step on g alone
  float momentum;                     // DW_OPT_MOMENTUM: the velocity lives in m
  float d_scale;                      // 0: D = z*hz (one probe); > 0: hz holds the sum of z_j*Hz_j, D = hz * d_scale
  uint64_t active_mask;               // bit i: worker i takes the step (others only report their distance)
  BiasRanges bias;
  FusedRanges fused;
  UpdateScalars sc;
  // several probes per step with fused weight gradients (see FuseArgs): mode, first probe, running sum [k][Pp]
  int probe_mode, probe_first;
  float* dacc;
  // filled by launch_update: the launch covers all n_blocks chunks (n_list == 0) or only the listed ones
  int n_blocks, n_list;
  int block_list[64];
};

struct WeightArgs {                   // dynamic-weight scalars of one communication round (Section V-B)
  const double* partials;             // [k][n_blocks]
  int n_blocks;
  const double* partials_f;           // [k][n_blocks_f] partial sums written by fused weight-gradient kernels
  int n_blocks_f;
  double* u_ring;                     // [k][DW_MAX_P+1]
  double* score;                      // [k][4] = u, a, h1, h2
  float* omh1;                        // [k] 1 - h1_i   (0 pull for absent workers is handled by the mask)
  float* h2;                          // [k]
  int k, p, mode;
  int slot;                           // ring slot receiving this round's u
  int n_valid;                        // values of u in the ring after the push (<= p+1)
  float alpha, kappa;
  float c[DW_MAX_P];
  float man_h1[DW_MAX_K], man_h2[DW_MAX_K];
};

struct PullArgs {
  float* theta; float* centre;        // [k][Pp], [Pp]
  uint16_t* wb16;                     // bf16 copy of theta or nullptr
  const float* omh1; const float* h2; // [k] device scalars written by the weight kernel
  int64_t Pp;
  int k;
  uint64_t part_mask;                 // bit i: worker i communicates in this round
  int sequential;                     // 1: exchanges one after the other in index order, the centre moves in between
};

hipError_t launch_update(const UpdateArgs& a, int n_blocks, hipStream_t s);
hipError_t launch_weights(const WeightArgs& a, hipStream_t s);
hipError_t launch_pull(const PullArgs& a, hipStream_t s);
// weights and pull of one round in a single launch, for models with few distance partial sums per worker
bool sync_fusable(const WeightArgs& w, const PullArgs& p);
hipError_t launch_weights_and_pull(const WeightArgs& w, const PullArgs& p, hipStream_t s);
hipError_t launch_rademacher(uint32_t* zbits, int64_t z_stride, int64_t n_words64, const uint64_t* keys_host,
                             int k, uint64_t active_mask, hipStream_t s);
// dacc = (first ? 0 : dacc) + z*hz for the active workers: the running sum of a step's Hutchinson probes
hipError_t launch_probe_sum(float* dacc, const float* hz, const uint32_t* zbits, int64_t Pp, int64_t z_stride, int k,
                            uint64_t active_mask, int first, const FusedRanges& skip, hipStream_t s);
// zt = z with the bits of one layer's W-part [R][C] transposed (bit (r, c) at woff + r*C + c goes to woff + c*R + r);
// R, C and woff must be multiples of 128, both strides multiples of 4 words, both arrays 16-byte aligned
hipError_t launch_transpose_bits(const uint32_t* z, int64_t z_stride, uint32_t* zt, int64_t zt_stride, int64_t woff, int R, int C, int k,
                                 uint64_t active_mask, hipStream_t s);
hipError_t launch_broadcast(float* theta, const float* centre, uint16_t* wb16, int64_t Pp, int k, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_refresh_bf16(const float* theta, uint16_t* wb16, int64_t n, hipStream_t s);
// out[i][c] = sum over the B rows of src[i][.][c] (bf16 [k][B][n], n a multiple of 8, 16-byte aligned) for the
// active workers: the bias part of a weight gradient when the product itself is left to another launch
hipError_t launch_col_sums_bf16(const uint16_t* src, int B, int n, float* out, int64_t out_wstride, int k,
                                uint64_t active_mask, hipStream_t s);

// records a failed HIP call for dw_last_hip_error (this thread) and returns DW_ERR_HIP
int note_hip_error(hipError_t e);

// ---- data side ---------------------------------------------------------------------------------------
size_t partition_scratch_bytes(int64_t n);
// index [k][o + s], s = floor((n-o)/k): row j = the shared points then worker j's own, in permutation order
hipError_t launch_partition(int64_t n, int64_t o, int k, uint64_t seed, int32_t* index, void* scratch, hipStream_t s);
// x [k][B][row_bytes], y [k][B]: draw b of worker j is row index[j][floor(u*m/2^64)], u = mix(key_j + GAMMA*(b+1))
hipError_t launch_gather(const void* data, const int32_t* labels, const int32_t* index, int64_t n, int64_t m,
                         int row_bytes, int B, int k, const uint64_t* keys_host, uint64_t active_mask, void* x,
                         int32_t* y, hipStream_t s);

// ---- network part ------------------------------------------------------------------------------------

// AdaHessian update applied in the epilogue of a weight-gradient GEMM (same arithmetic as update_kernel):
// element (m, n) of the product is parameter woff + m*ldc + n of the worker
struct FuseArgs {
  int on;
  int dist;                           // 1: also read the centre and report the tile's squared distance to it
  float* theta; float* m; float* v;   // worker 0's W block of the layer; worker stride = the product's c_wstride
  const float* centre;                // the layer's W block of the centre
  uint16_t* wb16;                     // bf16 copy of theta (W block), worker stride c_wstride; nullptr in fp32
  double* partials;                   // [k][part_stride] squared-distance partial sums, one slot per tile
  int part_stride, part_base;         // slot of tile t of worker i: i*part_stride + part_base + t
  int avg_block;                      // power of two, 1..32
  float lr, beta1, beta2, eps, hpow;
  UpdateScalars sc;
  // several Hutchinson probes.  0: one probe.  1: a probe that is not the last, only
  // dacc (+)= z*Hz is written (first: stored, not added).  2: the last probe, D = (dacc + z*Hz) * d_scale.
  // 3: both of two probes in this kernel (GemmArgs::RXp, RYp, zbits_p), D = (z_p*Hz_p + z*Hz) / 2
  int probe_mode, first;
  float* dacc;                        // the layer's W block of worker 0 in the running sum, worker stride c_wstride
  float d_scale;
};

enum GemmKind { GEMM_FWD = 0, GEMM_DGRAD = 1, GEMM_WGRAD = 2 };

// An operand of the fp32 GEMM that is a view of a channels-last map instead of a matrix in memory (3 x 3 convolution,
// stride 1, no padding, as a linear layer on patches; Section VI's model):
//   VIEW_PATCH    the patch matrix of the input map [B][H][W][Cin]: row m = output position (b, y, x) of the
//                 (H-2) x (W-2) grid, column c = tap*Cin + ci, tap = dy*3 + dx  ->  map entry (b, y+dy, x+dx, ci)
//   VIEW_SHIFTED  the gradient map [B][H-2][W-2][Cout] seen from the input positions: row q = (b, yy, xx) of the
//                 H x W grid, column c = tap*Cout + co  ->  entry (b, yy-dy, xx-dx, co), zero outside the output grid
//   VIEW_TAPS     the weight matrix W[Cout][9*Cin] with the taps moved to the contraction index: row k = tap*Cout + co,
//                 column ci  ->  W[co][tap*Cin + ci] (the sign bits of V likewise)
// Channel counts are multiples of 4, so four consecutive columns are four consecutive floats of the map (of W).
enum OperandView { VIEW_NONE = 0, VIEW_PATCH = 1, VIEW_SHIFTED = 2, VIEW_TAPS = 3 };
struct ConvView { int H, W, Cin, Cout; };   // the convolution's input map and channel counts (its output map is (H-2) x (W-2) x Cout)
// PLAIN: a data gradient stored as it is.  WGRAD_FUSED: template instance of the fp32 kernel for EPI_WGRAD with fu.on
enum Epilogue { EPI_RELU = 0, EPI_LINEAR = 1, EPI_MASK = 2, EPI_WGRAD = 3, EPI_PLAIN = 4, EPI_WGRAD_FUSED = 5 };

// One "dual-number" GEMM: C = X*Y and RC = RX*Y + X*RY for all workers (grid y = worker).
// Element strides describe how the logical operands X[M][K], Y[K][N] sit in memory.
struct GemmArgs {
  const void* X; const void* RX;      // RX == nullptr: that term is absent
  const void* Y; const void* RY;      // RY == nullptr and ry_bits == 0: absent
  int ry_bits;                        // RY is the +-1 direction z, read from zbits at z_off + element offset in Y
  const uint32_t* zbits; int64_t z_stride; int64_t z_off;
  const uint32_t* zbits_t;            // optional: z with the W-part of this layer transposed (bit (n, k) at z_off + n*K + k)
  int64_t zt_stride;                  // its per-worker stride in words
  int64_t x_wstride, y_wstride;       // per-worker element strides of X/RX and Y/RY
  int x_kcontig, y_kcontig;           // 1: contraction index is the contiguous one
  int ldx, ldy;
  int M, N, K;
  void* C; void* RC; int ldc; int64_t c_wstride;      // outputs [M][ldc]
  const void* mask_src; int ld_mask; int64_t mask_wstride;   // EPI_MASK: keep where mask_src > 0
  const float* bias; int64_t bias_wstride;            // EPI_RELU / EPI_LINEAR: theta + b_off
  int64_t zb_off;                                     // bit offset of the bias part of z
  float* gb; float* hzb;                              // EPI_WGRAD: bias-gradient outputs (g + b_off, hz + b_off)
  FuseArgs fu;                                        // EPI_WGRAD: fu.on != 0 replaces the stores of C and RC by the update
  // fp32 forward (EPI_RELU, EPI_LINEAR) or weight gradient with a long contraction and few output tiles: the contraction is cut into ksplit slices
  // (grid z), slice s of worker i writes its partial products to part + ((s*k + i)*2 + {0,1})*part_stride and its
  // partial bias sums (weight gradient) to part_b + ((s*k + i)*2 + {0,1})*M; a second kernel adds the slices in order and
  // applies the epilogue (bias, ReLU) into C, RC, gb, hzb
  int ksplit; float* part; int64_t part_stride; float* part_b;
  int x_view, y_view;                 // fp32 kernels: OperandView of X/RX and of Y/RY (and of the sign bits of V)
  ConvView cv;
  int r_only;                         // 1: C is in memory already (an earlier probe of this minibatch); kernels may compute RC alone
  // EPI_WGRAD with fu.probe_mode == 3 (two Hutchinson probes in one kernel): the earlier probe's R-companions of X
  // and Y (laid out like RX and RY; RYp == nullptr with RY) and its sign bits (strides and offsets as zbits)
  const void* RXp; const void* RYp; const uint32_t* zbits_p;
  int epi;
  int k;
  uint64_t active_mask;
};

// The argument structs travel by value in the kernel-argument segment (4 KB at most)
static_assert(sizeof(GemmArgs) <= 4096 && sizeof(UpdateArgs) <= 4096, "kernel arguments must fit the kernel-argument segment");

// The GEMM grids cover the active workers only: block group j works for the j-th set bit of active_mask.
__host__ __device__ inline int active_count(uint64_t mask, int k) {
  const uint64_t low = k >= 64 ? ~0ull : ((1ull << k) - 1ull);
  return __builtin_popcountll(mask & low);
}
__device__ __forceinline__ int nth_active_worker(uint64_t mask, int j) {
  while (j-- > 0) mask &= mask - 1;                   // drop the j lowest set bits (uniform scalar work)
  return __builtin_ctzll(mask);
}

// Raises the dynamic-LDS limit of a kernel the first time it is launched on a device (the attribute belongs to the
// device's code object).  One instance per kernel instantiation, as a function-local static of its launcher.  Host
// threads may race to the first launch: the flag is atomic and setting the attribute twice is harmless.
struct LdsLimitOnce {
  std::atomic<bool> done[64] = {};
  hipError_t raise(const void* kern, int bytes) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done[dev].store(true, std::memory_order_release);
    return e;
  }
};

hipError_t launch_gemm_f32(const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s);
// can the bf16 weight-gradient kernel of a layer W[n_out][n_in] (bit/parameter offset woff) apply the update itself,
// and how many partial-sum slots (tiles) does it then write per worker when a step has n_samples Hutchinson probes?
bool gemm_bf16_wgrad_fusable(int n_out, int n_in, int k, int avg_block, float hpow, int64_t woff);
int gemm_bf16_wgrad_tiles(int n_out, int n_in, int n_samples);
bool gemm_f32_wgrad_fusable(int n_out, int n_in, int k, int avg_block, float hpow, int64_t woff);   // same for fp32 (128 x 128 tiles)
int gemm_f32_wgrad_tiles(int n_out, int n_in);
// would the data gradient through W[n_out][n_in] of a minibatch of `batch` samples take the large-tile kernel
// (given the transposed sign bits)?
bool gemm_bf16_dgrad_dma_shape_ok(int batch, int n_out, int n_in, int k, int64_t woff);
bool gemm_bf16_dma_ok(const GemmArgs& a);                        // large-tile forward path usable for this product?
hipError_t launch_gemm_bf16_dma(const GemmArgs& a, hipStream_t s);
bool gemm_bf16_out_ok(const GemmArgs& a);                        // output-layer forward kernel usable for this product?
hipError_t launch_gemm_bf16_out(const GemmArgs& a, hipStream_t s);

struct HeadArgs {                     // softmax cross-entropy on the output layer and its R-derivative
  const float* s; const float* Rs;    // [k][B][ld] logits and their directional derivative
  float* delta; float* Rdelta;        // [k][B][ld] outputs (padding columns zeroed)
  uint16_t* delta_b16; uint16_t* Rdelta_b16;   // optional bf16 copies
  const int32_t* y;                   // [k][B]
  float* loss;                        // [k] or nullptr
  int B, C, ld, k;
  uint64_t active_mask;
};
hipError_t launch_head(const HeadArgs& a, hipStream_t s);
// fp32 output layer and head in one kernel (dw_out_head_f32.hip): `a` as for the output layer's forward product
// (its C and RC are not written), loss_part: k * ceil(M / 16) floats of scratch
bool out_head_f32_ok(const GemmArgs& a);
hipError_t launch_out_head_f32(const GemmArgs& a, const HeadArgs& h, float* loss_part, hipStream_t s);

struct Layout {            // byte offsets into the workspace, all multiples of 256
  int64_t P = 0, Pp = 0, z_stride = 0, n_upd_blocks = 0;
  int64_t woff[DW_MAX_LAYERS] = {0}, boff[DW_MAX_LAYERS] = {0};
  size_t theta = 0, m = 0, v = 0, g = 0, hz = 0, centre = 0, wb16 = 0, zbits = 0;
  size_t act[DW_MAX_LAYERS] = {0}, ract[DW_MAX_LAYERS] = {0};   // a_l, Ra_l for l = 1..L-1 (index l)
  size_t delta[DW_MAX_LAYERS] = {0}, rdelta[DW_MAX_LAYERS] = {0}; // d_l, Rd_l of the hidden layers l = 1..L-1 (index l)
  size_t sL = 0, rsL = 0, dL = 0, rdL = 0, dL16 = 0, rdL16 = 0;  // output layer, fp32 [k][B][16] (+ bf16 copies)
  size_t zbits_t = 0;                 // [k][z_stride] words: z with the W-parts of the layers in zt_layer transposed
  bool zt_layer[DW_MAX_LAYERS] = {false};   // index l-1: the data gradient through W_l reads the transposed bits
  size_t dacc = 0;                    // [k][Pp] floats, n_samples > 1 only: sum over the probes of z_j*Hz_j
  // two probes per step with fused bf16 weight gradients: those kernels take both probes at once, so the earlier
  // probe's z, Ra_l and Rd_l (hidden layers, index l) are kept in buffers of their own until the later probe's are there
  bool pair = false;
  size_t zbits_p = 0, ract_p[DW_MAX_LAYERS] = {0}, rdelta_p[DW_MAX_LAYERS] = {0};
  int fwdSplit[DW_MAX_LAYERS] = {0};   // fp32: slices of layer l+1's forward contraction (0 or 1: not cut)
  int dgSplit[DW_MAX_LAYERS] = {0};    // fp32: slices of the data gradient through W_{l+1} (0 or 1: not cut)
  bool overlap_wgrad = false;          // small model without fused layers: weight gradients on the handle's side stream
  int fuse_base[DW_MAX_LAYERS] = {0};  // first partial-sum slot of layer l+1's fused weight gradient, -1: not fused
  int n_fuse_slots = 0;
  size_t partials_f = 0;              // [k][n_fuse_slots] doubles
  // convolutional front end (index j = convolution j+1): geometry, parameter offsets, per-stage buffers
  int n_conv = 0;
  int cH[DW_MAX_CONV + 1] = {0}, cW[DW_MAX_CONV + 1] = {0}, cC[DW_MAX_CONV + 1] = {0};   // maps: input, then each output
  int cK[DW_MAX_CONV] = {0};                                    // padded row length of W_j: 9*C_in rounded up to 4
  int64_t cwoff[DW_MAX_CONV] = {0}, cboff[DW_MAX_CONV] = {0};
  size_t cP[DW_MAX_CONV] = {0};                                 // patches [k][M_0][K_0] of the first convolution
  size_t cA[DW_MAX_CONV] = {0}, cRA[DW_MAX_CONV] = {0};         // outputs a_j, Ra_j [k][M_j][C_j]
  size_t cD[DW_MAX_CONV] = {0}, cRD[DW_MAX_CONV] = {0};         // their gradients
  int cSplit[DW_MAX_CONV] = {0};                                // slices of the weight gradient's contraction (1: none)
  size_t cPart = 0, cPartB = 0;                                 // scratch of the sliced weight gradients
  size_t pool = 0, rpool = 0, dpool = 0, rdpool = 0, pidx = 0;  // pooled map [k][B][d_0] (+R, gradients), selection bytes
  size_t partials = 0, u_ring = 0, score = 0, omh1 = 0, h2 = 0, loss = 0;
  size_t total = 0;
};

// A second stream of a handle for launches that do not depend on each other: the weight gradients of a small model
// run beside its chain of data gradients (each launch fills a fraction of the chip and lasts about as long as the
// gap to the next one).  Forked from and joined to the caller's stream by events; the host never waits.
struct SideStream {
  hipStream_t s;
  hipEvent_t fork[DW_MAX_LAYERS + 1];   // index l: d_l and Rd_l are there
  hipEvent_t join;
};

// Enqueue forward, R-forward, backward and R-backward of all layers for the active workers; leaves the mean
// gradient in the g buffer and the Hessian-vector product in the hz buffer (returns a dw_status).  With `fuse`
// (the arguments of this step's update) the layers marked in lay.fuse_base are updated by their weight-gradient
// kernels instead, and their W-parts of g and hz are not written.  All data gradients are launched before the
// weight gradients (a fused weight gradient overwrites the W_l its layer's data gradient reads).
int run_network(const dw_config& cfg, char* ws, const Layout& lay, const void* d_x, const int32_t* d_y,
                const uint32_t* zbits, int64_t z_stride, uint64_t active, float* d_loss, const UpdateArgs* fuse,
                bool fuse_dist, hipStream_t s, const void* in_ract = nullptr, void* d_in = nullptr,
                void* rd_in = nullptr, bool r_only = false, int pair_phase = 0, const SideStream* side = nullptr);
// `r_only`: the same minibatch went through the network before (an earlier Hutchinson probe of this step), so the
// activations and the plain data gradients are in the workspace; kernels that can then compute the R-parts alone.
// `pair_phase` (lay.pair): 1 = the earlier of two probes: its R-quantities go to the buffers kept for it, the fused
// layers' weight gradients are left to the later probe's launch and only their bias parts of hz are written;
// 2 = the later probe: the fused weight-gradient kernels take both probes (zbits of the earlier one: lay.zbits_p).
// `side` (lay.overlap_wgrad): the weight gradients of the layers above the first are launched on that stream as soon
// as their d_l is there; the call returns with the caller's stream waiting for them.
// `in_ract` above: directional derivative of the input (nullptr: the input does not depend on the parameters).
// `d_in`, `rd_in`: when given, the gradient with respect to the input and its R-companion ([k][B][d_0], zero where
// the input is not positive: the input is then the ReLU output of a layer in front).
//
// The same for a model with a convolutional front end: convolutions, pooling, then run_network on the pooled map,
// then back through the pooling and the convolutions (fp32 only).
int run_network_cnn(const dw_config& cfg, char* ws, const Layout& lay, const void* d_x, const int32_t* d_y,
                    const uint32_t* zbits, int64_t z_stride, uint64_t active, float* d_loss, hipStream_t s);
// A small fp32 model's whole worker step in one kernel (dw_tiny.hip): can this configuration take it, and the launch.
// `u`: the update's arguments of this step (step counts already advanced), keys_host: the workers' stream keys.
bool tiny_step_ok(const dw_config& cfg, const Layout& lay);
hipError_t launch_tiny_step(const dw_config& cfg, char* ws, const Layout& lay, const void* d_x, const int32_t* d_y,
                            const uint32_t* d_zbits, const UpdateArgs& u, const uint64_t* keys_host, float* d_loss,
                            hipStream_t s);
// hz <- z * (mean over each 3x3 window of z * hz) on the kernels of the convolutions (Section IV-B averaging)
hipError_t launch_conv_window_mean(float* hz, const uint32_t* zbits, int64_t Pp, int64_t z_stride, const Layout& lay,
                                   int k, uint64_t active, hipStream_t s);

}  // namespace dw

// ---- optional per-kernel timing (HIP events on the caller's stream) ------------------------------------
namespace dw {

enum KernelClass {
  KC_RADEMACHER = 0, KC_GEMM_FWD = 1, KC_HEAD = 2, KC_GEMM_WGRAD = 3, KC_GEMM_DGRAD = 4,
  KC_UPDATE = 5, KC_WEIGHTS = 6, KC_PULL = 7, KC_GATHER = 8, KC_STEP = 9, KC_COUNT = 10
};

struct Profiler {
  static constexpr int kMaxLaunches = 8192;
  hipEvent_t start[kMaxLaunches];
  hipEvent_t stop[kMaxLaunches];
  int cls[kMaxLaunches];
  int created = 0;        // event pairs created so far
  int used = 0;           // pairs recorded since the last read
  int dropped = 0;
};

extern thread_local Profiler* tl_profiler;     // set by the API entry points while profiling is enabled

struct KernelScope {                            // records an event before and after one kernel launch
  Profiler* p; int slot; hipStream_t s;
  KernelScope(int kclass, hipStream_t stream);
  ~KernelScope();
};

}  // namespace dw
