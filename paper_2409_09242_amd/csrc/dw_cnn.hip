// Convolutional front end of the classifier (the paper's experiments use a small CNN, Section VI) and its
// directional derivative along z, in fp32.
//
// A 3x3 convolution (stride 1, no padding) over a channels-last map is a linear layer applied to every 3x3 patch,
// so it runs on the dual GEMM of the linear layers: the patches of a map [B][H][W][C] become a matrix
// [B*(H-2)*(W-2)][K], K = 9*C rounded up to 4, column (dy*3 + dx)*C + ci holding input (y+dy, x+dx, ci) (channels
// innermost, as in the map, so that patches are cut and put back with contiguous accesses), and
//   forward      S  = P W^T + b,          RS  = RP W^T + P V^T + c         (P patches, V = z reshaped like W)
//   weight grad  gW = D^T P,              HzW = RD^T P + D^T RP
//   data grad    dP = D W,                RdP = RD W + D V,   then summed back onto the map ("col2im")
// are the three products of Section IV-B's Hessian-vector product with B*(H-2)*(W-2) rows instead of B.  ReLU and
// max-pool pass the directional derivative through their selections (their curvature is zero almost everywhere).
// Only the first convolution (one input channel in the paper's model: 9 columns) has its patch matrix in memory.
// The others read the map itself: the GEMM's loader takes the patch matrix as a view of the map (OperandView), and
// the data gradient is the same product written from the input positions' side, dA = sum over taps of the shifted
// gradient map times W's tap, so that the nine contributions of a map entry are added inside the contraction and
// no patch-shaped gradient is ever stored.
// This file holds the data movement around those products (patch extraction for the first convolution, pooling and
// its adjoint, the 3x3 window mean of the Hutchinson estimate) and the order of the launches.
#include "dw_internal.h"

namespace dw {

namespace {

// patches of value map `in` and, when given, of its R-companion `rin`: one thread per V consecutive patch entries
// (V = 4 when the channel count allows 16-byte accesses, else 1)
template <int V>
__global__ __launch_bounds__(256) void im2col3x3_kernel(const float* in, const float* rin, float* P, float* RP, int B, int H,
                                                        int W, int C, int K, uint64_t active_mask) {
  const int worker = blockIdx.y;
  if (!((active_mask >> worker) & 1ull)) return;
  const int Ho = H - 2, Wo = W - 2, KV = K / V;
  const int64_t rows = (int64_t)B * Ho * Wo, total = rows * K, groups = rows * KV;
  const int64_t in_w = (int64_t)B * H * W * C;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < groups; e += (int64_t)gridDim.x * 256) {
    const int64_t m = e / KV;
    const int kk = (int)(e - m * KV) * V;
    float v[V], rv[V];
#pragma unroll
    for (int q = 0; q < V; ++q) { v[q] = 0.f; rv[q] = 0.f; }
    if (kk < 9 * C) {                                  // V consecutive channels of one tap (C % V == 0)
      const int tap = kk / C, ci = kk - tap * C, dy = tap / 3, dx = tap - dy * 3;
      const int x = (int)(m % Wo), y = (int)((m / Wo) % Ho);
      const int64_t b = m / ((int64_t)Wo * Ho);
      const int64_t src = worker * in_w + ((b * H + (y + dy)) * W + (x + dx)) * C + ci;
      if (V == 4) {
        const float4 t = *reinterpret_cast<const float4*>(in + src);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        if (rin) { const float4 r = *reinterpret_cast<const float4*>(rin + src); rv[0] = r.x; rv[1] = r.y; rv[2] = r.z; rv[3] = r.w; }
      } else {
        v[0] = in[src];
        if (rin) rv[0] = rin[src];
      }
    }
    const int64_t dst = worker * total + m * K + kk;
    if (V == 4) {
      *reinterpret_cast<float4*>(P + dst) = make_float4(v[0], v[1], v[2], v[3]);
      if (RP) *reinterpret_cast<float4*>(RP + dst) = make_float4(rv[0], rv[1], rv[2], rv[3]);
    } else {
      P[dst] = v[0];
      if (RP) RP[dst] = rv[0];
    }
  }
}

// 2x2 max-pool of a map and the same selection applied to its R-companion; which[...] = 0..3 in the order
// (0,0), (0,1), (1,0), (1,1), the first one on ties; one thread per four consecutive channels of a pooled entry
__global__ __launch_bounds__(256) void maxpool2_kernel(const float* A, const float* RA, float* Pm, float* RPm,
                                                       uint8_t* which, int B, int H, int W, int C, uint64_t active_mask) {
  const int worker = blockIdx.y;
  if (!((active_mask >> worker) & 1ull)) return;
  const int Hp = H / 2, Wp = W / 2, C4 = C / 4;
  const int64_t total = (int64_t)B * Hp * Wp * C, groups = total / 4, a_w = (int64_t)B * H * W * C;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < groups; e += (int64_t)gridDim.x * 256) {
    const int c = (int)(e % C4) * 4;
    const int j = (int)((e / C4) % Wp), i = (int)((e / ((int64_t)C4 * Wp)) % Hp);
    const int64_t b = e / ((int64_t)C4 * Wp * Hp);
    float best[4] = {0.f, 0.f, 0.f, 0.f}, rbest[4] = {0.f, 0.f, 0.f, 0.f};
    uint32_t sel[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t src = worker * a_w + ((b * H + (2 * i + (q >> 1))) * W + (2 * j + (q & 1))) * C + c;
      const float4 v4 = *reinterpret_cast<const float4*>(A + src), r4 = *reinterpret_cast<const float4*>(RA + src);
      const float v[4] = {v4.x, v4.y, v4.z, v4.w}, r[4] = {r4.x, r4.y, r4.z, r4.w};
#pragma unroll
      for (int t = 0; t < 4; ++t)
        if (q == 0 || v[t] > best[t]) { best[t] = v[t]; rbest[t] = r[t]; sel[t] = (uint32_t)q; }
    }
    *reinterpret_cast<float4*>(Pm + worker * total + e * 4) = make_float4(best[0], best[1], best[2], best[3]);
    *reinterpret_cast<float4*>(RPm + worker * total + e * 4) = make_float4(rbest[0], rbest[1], rbest[2], rbest[3]);
    *reinterpret_cast<uint32_t*>(which + worker * total + e * 4) = sel[0] | (sel[1] << 8) | (sel[2] << 16) | (sel[3] << 24);
  }
}

// adjoint of the pooling: the gradient of a pooled entry goes to the input that was selected, zero to the others;
// one thread per four consecutive channels of a map entry (channel counts are multiples of 4)
__global__ __launch_bounds__(256) void unpool2_kernel(const float* dPm, const float* RdPm, const uint8_t* which, float* D,
                                                      float* RD, int B, int H, int W, int C, uint64_t active_mask) {
  const int worker = blockIdx.y;
  if (!((active_mask >> worker) & 1ull)) return;
  const int Hp = H / 2, Wp = W / 2, C4 = C / 4;
  const int64_t total = (int64_t)B * H * W * C, groups = total / 4, p_w = (int64_t)B * Hp * Wp * C;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < groups; e += (int64_t)gridDim.x * 256) {
    const int c = (int)(e % C4) * 4;
    const int x = (int)((e / C4) % W), y = (int)((e / ((int64_t)C4 * W)) % H);
    const int64_t b = e / ((int64_t)C4 * W * H);
    const int64_t src = worker * p_w + ((b * Hp + (y >> 1)) * Wp + (x >> 1)) * C + c;
    const uint32_t w4 = *reinterpret_cast<const uint32_t*>(which + src);       // the selections of the four channels
    const uint32_t mine = (uint32_t)((y & 1) * 2 + (x & 1));
    const float4 d = *reinterpret_cast<const float4*>(dPm + src), rd = *reinterpret_cast<const float4*>(RdPm + src);
    const bool m0 = (w4 & 0xFFu) == mine, m1 = ((w4 >> 8) & 0xFFu) == mine, m2 = ((w4 >> 16) & 0xFFu) == mine, m3 = (w4 >> 24) == mine;
    *reinterpret_cast<float4*>(D + worker * total + e * 4) = make_float4(m0 ? d.x : 0.f, m1 ? d.y : 0.f, m2 ? d.z : 0.f, m3 ? d.w : 0.f);
    *reinterpret_cast<float4*>(RD + worker * total + e * 4) = make_float4(m0 ? rd.x : 0.f, m1 ? rd.y : 0.f, m2 ? rd.z : 0.f, m3 ? rd.w : 0.f);
  }
}

// Section IV-B averaging for a convolution kernel: D = z * Hz is replaced by its mean over the 3x3 window of every
// (output, input) channel pair.  The update multiplies hz by z again, so the window mean is stored times z.
__global__ __launch_bounds__(256) void conv_window_mean_kernel(float* hz, const uint32_t* zbits, int64_t Pp, int64_t z_stride,
                                                               int64_t woff, int C_out, int C_in, int K, uint64_t active_mask) {
  const int worker = blockIdx.y;
  if (!((active_mask >> worker) & 1ull)) return;
  const int pair = blockIdx.x * 256 + threadIdx.x;
  if (pair >= C_out * C_in) return;
  const int co = pair / C_in, ci = pair - co * C_in;
  const int64_t j0 = woff + (int64_t)co * K + ci;           // tap t of the pair sits C_in entries further on each time
  float* h = hz + worker * Pp;
  const uint32_t* zb = zbits + worker * z_stride;
  float sign[9], s = 0.f;
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    const int64_t j = j0 + (int64_t)t * C_in;
    sign[t] = ((zb[j >> 5] >> (j & 31)) & 1u) ? 1.f : -1.f;
    s += sign[t] * h[j];
  }
  s *= 1.0f / 9.0f;
#pragma unroll
  for (int t = 0; t < 9; ++t) h[j0 + (int64_t)t * C_in] = sign[t] * s;
}

inline unsigned blocks_for(int64_t n) {
  const int64_t b = (n + 255) / 256;
  return (unsigned)(b < 1 ? 1 : b > 16384 ? 16384 : b);
}

}  // namespace

hipError_t launch_conv_window_mean(float* hz, const uint32_t* zbits, int64_t Pp, int64_t z_stride, const Layout& lay,
                                   int k, uint64_t active, hipStream_t s) {
  KernelScope ks(KC_UPDATE, s);
  for (int j = 0; j < lay.n_conv; ++j) {
    const int pairs = lay.cC[j + 1] * lay.cC[j];
    hipLaunchKernelGGL(conv_window_mean_kernel, dim3((unsigned)((pairs + 255) / 256), (unsigned)k), dim3(256), 0, s, hz,
                       zbits, Pp, z_stride, lay.cwoff[j], lay.cC[j + 1], lay.cC[j], lay.cK[j], active);
  }
  return hipGetLastError();
}

int run_network_cnn(const dw_config& cfg, char* ws, const Layout& lay, const void* d_x, const int32_t* d_y,
                    const uint32_t* zbits, int64_t z_stride, uint64_t active, float* d_loss, hipStream_t s) {
  const int nc = lay.n_conv, k = cfg.k, B = cfg.batch;
  float* theta = reinterpret_cast<float*>(ws + lay.theta);
  float* g = reinterpret_cast<float*>(ws + lay.g);
  float* hz = reinterpret_cast<float*>(ws + lay.hz);
  auto f = [&](size_t off) { return reinterpret_cast<float*>(ws + off); };
  auto rows = [&](int j) { return (int64_t)B * lay.cH[j + 1] * lay.cW[j + 1]; };   // patches / output positions of convolution j
  hipError_t e;

  // forward through the convolutions
  for (int j = 0; j < nc; ++j) {
    const float* in = j == 0 ? reinterpret_cast<const float*>(d_x) : f(lay.cA[j - 1]);
    const float* rin = j == 0 ? nullptr : f(lay.cRA[j - 1]);
    const int64_t M = rows(j);
    const int64_t in_stride = (int64_t)B * lay.cH[j] * lay.cW[j] * lay.cC[j];
    if (j == 0) {
      KernelScope ks(KC_GEMM_FWD, s);
      if (lay.cC[j] % 4 == 0)
        hipLaunchKernelGGL(im2col3x3_kernel<4>, dim3(blocks_for(M * lay.cK[j] / 4), (unsigned)k), dim3(256), 0, s, in, rin,
                           f(lay.cP[j]), nullptr, B, lay.cH[j], lay.cW[j], lay.cC[j], lay.cK[j], active);
      else
        hipLaunchKernelGGL(im2col3x3_kernel<1>, dim3(blocks_for(M * lay.cK[j]), (unsigned)k), dim3(256), 0, s, in, rin,
                           f(lay.cP[j]), nullptr, B, lay.cH[j], lay.cW[j], lay.cC[j], lay.cK[j], active);
      if ((e = hipGetLastError()) != hipSuccess) return DW_ERR_HIP;
    }
    GemmArgs a{};
    if (j == 0) {
      a.X = f(lay.cP[j]); a.RX = nullptr; a.x_wstride = M * lay.cK[j];
    } else {                                             // the patches of the map below, read in place
      a.X = in; a.RX = rin; a.x_wstride = in_stride; a.x_view = VIEW_PATCH;
      a.cv.H = lay.cH[j]; a.cv.W = lay.cW[j]; a.cv.Cin = lay.cC[j]; a.cv.Cout = lay.cC[j + 1];
    }
    a.x_kcontig = 1; a.ldx = lay.cK[j];
    a.Y = theta + lay.cwoff[j]; a.RY = nullptr; a.ry_bits = 1; a.y_wstride = lay.Pp; a.y_kcontig = 1; a.ldy = lay.cK[j];
    a.zbits = zbits; a.z_stride = z_stride; a.z_off = lay.cwoff[j]; a.zb_off = lay.cboff[j];
    a.M = (int)M; a.N = lay.cC[j + 1]; a.K = lay.cK[j];
    a.bias = theta + lay.cboff[j]; a.bias_wstride = lay.Pp;
    a.C = f(lay.cA[j]); a.RC = f(lay.cRA[j]); a.ldc = lay.cC[j + 1]; a.c_wstride = M * lay.cC[j + 1];
    a.epi = EPI_RELU; a.k = k; a.active_mask = active;
    if ((e = launch_gemm_f32(a, s)) != hipSuccess) return DW_ERR_HIP;
  }
  // pooling
  {
    KernelScope ks(KC_GEMM_FWD, s);
    const int64_t total = (int64_t)B * cfg.dims[0];
    hipLaunchKernelGGL(maxpool2_kernel, dim3(blocks_for(total / 4), (unsigned)k), dim3(256), 0, s, f(lay.cA[nc - 1]),
                       f(lay.cRA[nc - 1]), f(lay.pool), f(lay.rpool), reinterpret_cast<uint8_t*>(ws + lay.pidx), B,
                       lay.cH[nc], lay.cW[nc], lay.cC[nc], active);
    if ((e = hipGetLastError()) != hipSuccess) return DW_ERR_HIP;
  }
  // the linear layers, forward and backward, down to the gradient with respect to the pooled map
  const int st = run_network(cfg, ws, lay, f(lay.pool), d_y, zbits, z_stride, active, d_loss, nullptr, true, s,
                             f(lay.rpool), f(lay.dpool), f(lay.rdpool));
  if (st != DW_OK) return st;
  // back through the pooling (the ReLU of the last convolution is already in the mask of that gradient: a pooled
  // entry is positive exactly when the input it selected is).  (Reading the pooled gradient through the selections in
  // the loaders of the last convolution's products instead was measured slower: its weight gradient 0.37 -> 0.49 ms
  // for the 0.10 ms of this kernel.)
  {
    KernelScope ks(KC_GEMM_DGRAD, s);
    const int64_t total = rows(nc - 1) * lay.cC[nc];
    hipLaunchKernelGGL(unpool2_kernel, dim3(blocks_for(total / 4), (unsigned)k), dim3(256), 0, s, f(lay.dpool), f(lay.rdpool),
                       reinterpret_cast<const uint8_t*>(ws + lay.pidx), f(lay.cD[nc - 1]), f(lay.cRD[nc - 1]), B,
                       lay.cH[nc], lay.cW[nc], lay.cC[nc], active);
    if ((e = hipGetLastError()) != hipSuccess) return DW_ERR_HIP;
  }
  // back through the convolutions: weight gradient (contraction over all output positions of the minibatch), then
  // the data gradient onto the map below with that map's ReLU mask
  for (int j = nc - 1; j >= 0; --j) {
    const int64_t M = rows(j);
    const int64_t in_stride = (int64_t)B * lay.cH[j] * lay.cW[j] * lay.cC[j];
    {
      GemmArgs a{};
      a.X = f(lay.cD[j]); a.RX = f(lay.cRD[j]); a.x_wstride = M * lay.cC[j + 1]; a.x_kcontig = 0; a.ldx = lay.cC[j + 1];
      if (j == 0) {
        a.Y = f(lay.cP[j]); a.RY = nullptr; a.y_wstride = M * lay.cK[j];
      } else {
        a.Y = f(lay.cA[j - 1]); a.RY = f(lay.cRA[j - 1]); a.y_wstride = in_stride; a.y_view = VIEW_PATCH;
        a.cv.H = lay.cH[j]; a.cv.W = lay.cW[j]; a.cv.Cin = lay.cC[j]; a.cv.Cout = lay.cC[j + 1];
      }
      a.ry_bits = 0; a.y_kcontig = 0; a.ldy = lay.cK[j];
      a.zbits = zbits; a.z_stride = z_stride;
      a.M = lay.cC[j + 1]; a.N = lay.cK[j]; a.K = (int)M;
      a.C = g + lay.cwoff[j]; a.RC = hz + lay.cwoff[j]; a.ldc = lay.cK[j]; a.c_wstride = lay.Pp;
      a.gb = g + lay.cboff[j]; a.hzb = hz + lay.cboff[j];
      a.epi = EPI_WGRAD; a.k = k; a.active_mask = active;
      if (lay.cSplit[j] > 1) {
        a.ksplit = lay.cSplit[j]; a.part = f(lay.cPart); a.part_stride = (int64_t)lay.cC[j + 1] * lay.cK[j];
        a.part_b = f(lay.cPartB);
      }
      if ((e = launch_gemm_f32(a, s)) != hipSuccess) return DW_ERR_HIP;
    }
    if (j == 0) break;
    {
      // dA[q][ci] = sum over (tap, co) of D[q - tap][co] * W[co][tap][ci] for every position q of the map below
      GemmArgs a{};
      a.X = f(lay.cD[j]); a.RX = f(lay.cRD[j]); a.x_wstride = M * lay.cC[j + 1]; a.x_kcontig = 1; a.x_view = VIEW_SHIFTED;
      a.Y = theta + lay.cwoff[j]; a.RY = nullptr; a.ry_bits = 1; a.y_wstride = lay.Pp; a.y_kcontig = 0; a.y_view = VIEW_TAPS;
      a.cv.H = lay.cH[j]; a.cv.W = lay.cW[j]; a.cv.Cin = lay.cC[j]; a.cv.Cout = lay.cC[j + 1];
      a.ldx = lay.cC[j + 1]; a.ldy = lay.cC[j];
      a.zbits = zbits; a.z_stride = z_stride; a.z_off = lay.cwoff[j];
      a.M = (int)((int64_t)B * lay.cH[j] * lay.cW[j]); a.N = lay.cC[j]; a.K = 9 * lay.cC[j + 1];
      a.C = f(lay.cD[j - 1]); a.RC = f(lay.cRD[j - 1]); a.ldc = lay.cC[j]; a.c_wstride = in_stride;
      a.mask_src = f(lay.cA[j - 1]); a.ld_mask = lay.cC[j]; a.mask_wstride = in_stride;
      a.epi = EPI_MASK; a.k = k; a.active_mask = active;
      if ((e = launch_gemm_f32(a, s)) != hipSuccess) return DW_ERR_HIP;
    }
  }
  return DW_OK;
}

}  // namespace dw
