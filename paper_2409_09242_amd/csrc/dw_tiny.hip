// One worker step of a small fp32 MLP in a single kernel (gfx950, wave64).
//
// A model whose parameters and activations fit in the LDS of one compute unit spends its step waiting for a chain of
// short kernels (Rademacher bits, a product and its sum of slices per layer and direction, head, update: 9 launches of
// 2 to 7 us each for a 32-64-10 model).  Here one block per worker keeps everything on chip and walks through the
// whole of Section IV-B: z from the counter-based stream, forward and R-forward pass, softmax head, backward and
// R-backward pass (g and the Hessian-vector product Hz, Section II eq.(2) and the Hutchinson display), D = z*Hz with
// its block mean along fan-in, moments, bias correction, parameter update (eq.(4)) and the squared distance of the
// new parameters to the centre for the next communication round (Section V-B).  The products are plain FMA loops out
// of LDS (a few 10^5 flop per worker: the matrix cores would not be fed), summed in index order.
//
// LDS (floats): W_l with rows padded by one (so that the threads of a wave, which own consecutive outputs j, read
// different banks), b_l, the same layout for z as +-1 floats, a_0, then a_l and Ra_l of the hidden layers, two pairs of
// error buffers (d_l, Rd_l and d_{l-1}, Rd_{l-1}), and g, Hz in the canonical layout for the update pass.
#include <cstddef>

#include "dw_internal.h"
#include "dw_device_util.h"
#include "dw_head_math.h"

namespace dw {

namespace {

constexpr int kTinyThreads = 1024;                  // 16 waves on the one compute unit: four per SIMD hide the LDS latency
constexpr int kTinyMaxLdsFloats = 39 * 1024;        // 156 KB of the compute unit's 160 KB

struct TinyArgs {
  const float* x; const int32_t* y;                  // [k][B][d_0], [k][B]
  const uint32_t* zbits_in; int64_t z_stride_in;     // caller's sign bits, or nullptr: drawn here
  uint32_t* zbits; int64_t z_stride;                 // the library's sign-bit buffer (written when drawn here)
  float* theta; float* m; float* v; float* g; float* hz; const float* centre;
  double* partials; int n_blocks;                    // [k][n_blocks] squared-distance partial sums
  float* act[DW_MAX_LAYERS];                         // a_l of the hidden layers in memory, [k][B][d_l] (index l)
  float* loss;                                       // [k] or nullptr
  int64_t P, Pp;
  int L, B, k;
  int dims[DW_MAX_LAYERS + 1];
  int avg_block;
  float lr, beta1, beta2, eps, hpow;
  uint64_t active_mask;
  uint64_t key[DW_MAX_K];                            // keys of the workers' Rademacher streams at this step
  UpdateScalars sc;
};

__device__ __forceinline__ uint64_t tiny_mix64(uint64_t x) {     // SplitMix64 output function
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

__device__ __forceinline__ float tiny_denom(float vhat, float hpow) {       // (sqrt(v_hat))^hpow
  if (hpow == 1.0f) return sqrtf(vhat);
  if (hpow == 0.0f) return 1.0f;
  if (hpow == 2.0f) return vhat;
  return powf(vhat, 0.5f * hpow);
}

__global__ __launch_bounds__(kTinyThreads) void tiny_step_kernel(TinyArgs a) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i = blockIdx.x;                                    // one block per worker
  const bool active = (a.active_mask >> i) & 1ull;
  const int L = a.L, B = a.B;
  const int64_t P = a.P;
  __shared__ double red[kTinyThreads / 64];
  float nsum = 0.f;
  float* th_g = a.theta + (int64_t)i * a.Pp;

  if (active) {
    // per-worker scalars from the kernel-argument block (scalar loads; indexing the by-value argument with a
    // variable would copy it to scratch memory)
    typedef const char __attribute__((address_space(4)))* karg_bytes;
    typedef const float __attribute__((address_space(4)))* karg_floats;
    typedef const uint64_t __attribute__((address_space(4)))* karg_u64;
    const karg_bytes ka = (karg_bytes)__builtin_amdgcn_kernarg_segment_ptr();
    const uint64_t key = ((karg_u64)(ka + offsetof(TinyArgs, key)))[i];
    const karg_floats bc = (karg_floats)(ka + offsetof(TinyArgs, sc));
    const float ib1 = bc[i], ib2 = bc[DW_MAX_K + i];
    static_assert(offsetof(UpdateScalars, inv_bc2) == DW_MAX_K * sizeof(float), "inv_bc2 follows inv_bc1");

    // ---- LDS map --------------------------------------------------------------------------------------------
    int wsize = 0, hidden = 0, dmax = DW_MAX_CLASSES;
    for (int l = 1; l <= L; ++l) {
      wsize += a.dims[l] * (a.dims[l - 1] + 1) + a.dims[l];
      if (l < L) { hidden += a.dims[l]; if (a.dims[l] > dmax) dmax = a.dims[l]; }
    }
    const int nzw = 2 * (int)((P + 63) >> 6);                  // 32-bit words of sign bits
    float* Wp = lds;                                           // padded weights and biases, layer after layer
    float* Zp = Wp + wsize;                                    // z as +-1 in the same layout
    float* A0 = Zp + wsize;                                    // a_0 [B][d_0]
    float* AH = A0 + B * a.dims[0];                            // a_l, Ra_l of the hidden layers, [B][d_l] each
    float* DB = AH + 2 * B * hidden;                           // error buffers: 2 x (d, Rd), [B][dmax] each
    float* GL = DB + 4 * B * dmax;                             // g, canonical layout, padded to a multiple of 4
    const int Pq = (int)((P + 3) & ~3ll);
    float* HL = GL + Pq;                                       // Hz
    uint32_t* ZW = reinterpret_cast<uint32_t*>(HL + Pq);       // sign-bit words
    float* LV = HL + Pq + nzw;                                 // per-sample losses
    for (int e = (int)P + tid; e < Pq; e += kTinyThreads) { GL[e] = 0.f; HL[e] = 0.f; }   // (tail of the last group of four)

    // the update's operands of this thread's first group of four: asked for now, used at the very end
    const int nq_all = Pq >> 2;
    float4 T0 = make_float4(0.f, 0.f, 0.f, 0.f), M0 = T0, V0 = T0, C0 = T0;
    if (tid < nq_all) {
      T0 = reinterpret_cast<const float4*>(th_g)[tid];
      M0 = reinterpret_cast<const float4*>(a.m + (int64_t)i * a.Pp)[tid];
      V0 = reinterpret_cast<const float4*>(a.v + (int64_t)i * a.Pp)[tid];
      C0 = reinterpret_cast<const float4*>(a.centre)[tid];
    }
    // ---- z: drawn from the worker's stream (element j = bit j%64 of word j/64), or the caller's -------------
    if (a.zbits_in) {
      const uint32_t* src = a.zbits_in + (int64_t)i * a.z_stride_in;
      for (int w = tid; w < nzw; w += kTinyThreads) ZW[w] = src[w];
    } else {
      uint32_t* dst = a.zbits + (int64_t)i * a.z_stride;
      for (int w = tid; w < (nzw >> 1); w += kTinyThreads) {
        const uint64_t xw = tiny_mix64(key + 0x9E3779B97F4A7C15ull * (uint64_t)(w + 1));
        ZW[2 * w] = (uint32_t)xw; ZW[2 * w + 1] = (uint32_t)(xw >> 32);
        reinterpret_cast<uint2*>(dst)[w] = make_uint2((uint32_t)xw, (uint32_t)(xw >> 32));
      }
    }
    // input minibatch and parameters (padded layout), in the same pass over memory
    {
      const float* xs = a.x + (int64_t)i * B * a.dims[0];
      for (int e = tid; e < B * a.dims[0]; e += kTinyThreads) A0[e] = xs[e];
      int64_t off = 0; int pos = 0;
      for (int l = 1; l <= L; ++l) {
        const int dout = a.dims[l], din = a.dims[l - 1];
        for (int e = tid; e < dout * din; e += kTinyThreads) {
          const int j = e / din, kk = e - j * din;
          Wp[pos + j * (din + 1) + kk] = th_g[off + e];
        }
        off += (int64_t)dout * din; pos += dout * (din + 1);
        for (int e = tid; e < dout; e += kTinyThreads) Wp[pos + e] = th_g[off + e];
        off += dout; pos += dout;
      }
    }
    __syncthreads();
    // the direction z as +-1 in the same layout
    {
      int64_t off = 0; int pos = 0;
      for (int l = 1; l <= L; ++l) {
        const int dout = a.dims[l], din = a.dims[l - 1];
        for (int e = tid; e < dout * din; e += kTinyThreads) {
          const int j = e / din, kk = e - j * din;
          const int64_t c = off + e;
          Zp[pos + j * (din + 1) + kk] = ((ZW[c >> 5] >> (c & 31)) & 1u) ? 1.f : -1.f;
        }
        off += (int64_t)dout * din; pos += dout * (din + 1);
        for (int e = tid; e < dout; e += kTinyThreads) {
          const int64_t c = off + e;
          Zp[pos + e] = ((ZW[c >> 5] >> (c & 31)) & 1u) ? 1.f : -1.f;
        }
        off += dout; pos += dout;
      }
    }
    __syncthreads();

    // ---- forward and R-forward: s = a W^T + b, Rs = Ra W^T + a V^T + c ---------------------------------------
    float* SL = DB;                          // logits and their derivative land in the first error buffers
    float* RSL = DB + B * dmax;
    {
      int pos = 0, hoff = 0;
      const float* Ain = A0; const float* RAin = nullptr;
      for (int l = 1; l <= L; ++l) {
        const int dout = a.dims[l], din = a.dims[l - 1];
        const float* bl = Wp + pos + dout * (din + 1);
        const float* cl = Zp + pos + dout * (din + 1);
        float* Aout = AH + hoff; float* RAout = Aout + B * dout;
        float* act_g = l < L ? a.act[l] + (int64_t)i * B * dout : nullptr;
        for (int o = tid; o < B * dout; o += kTinyThreads) {
          const int n = o / dout, j = o - n * dout;
          const float* wr = Wp + pos + j * (din + 1);
          const float* zr = Zp + pos + j * (din + 1);
          const float* ar = Ain + n * din;
          float s = 0.f, rs = 0.f;
          if (RAin) {
            const float* rar = RAin + n * din;
#pragma unroll 4
            for (int kk = 0; kk < din; ++kk) {
              const float av = ar[kk], wv = wr[kk];
              s = fmaf(av, wv, s);
              rs = fmaf(rar[kk], wv, rs);
              rs = fmaf(av, zr[kk], rs);
            }
          } else {
#pragma unroll 4
            for (int kk = 0; kk < din; ++kk) {
              const float av = ar[kk];
              s = fmaf(av, wr[kk], s);
              rs = fmaf(av, zr[kk], rs);
            }
          }
          s += bl[j]; rs += cl[j];
          if (l < L) {
            const bool on = s > 0.f;                           // ReLU: slope 0 at exactly 0
            Aout[o] = on ? s : 0.f; RAout[o] = on ? rs : 0.f;
            act_g[o] = on ? s : 0.f;
          } else {
            SL[n * dmax + j] = s; RSL[n * dmax + j] = rs;
          }
        }
        __syncthreads();
        pos += dout * (din + 1) + dout;
        if (l < L) { Ain = Aout; RAin = RAout; hoff += 2 * B * dout; }
      }
    }

    // ---- softmax cross-entropy head: d_L = (p - onehot)/B, Rd_L ---------------------------------------------
    float* D0 = DB + 2 * B * dmax;           // d_L, Rd_L go to the second pair (the first still holds the logits)
    float* RD0 = D0 + B * dmax;
    {
      const int C = a.dims[L];
      const float invB = 1.0f / (float)B;
      const int32_t* ys = a.y + (int64_t)i * B;
      float* lossv = LV;
      for (int n = tid; n < B; n += kTinyThreads) {
        float s[DW_MAX_CLASSES], rs[DW_MAX_CLASSES], d[DW_MAX_CLASSES], rd[DW_MAX_CLASSES];
#pragma unroll
        for (int c = 0; c < DW_MAX_CLASSES; ++c) {
          s[c] = c < C ? SL[n * dmax + c] : 0.f;
          rs[c] = c < C ? RSL[n * dmax + c] : 0.f;
        }
        lossv[n] = head_row(s, rs, ys[n], C, invB, d, rd);
#pragma unroll
        for (int c = 0; c < DW_MAX_CLASSES; ++c)
          if (c < C) { D0[n * dmax + c] = d[c]; RD0[n * dmax + c] = rd[c]; }
      }
      __syncthreads();
      if (tid == 0 && a.loss) {
        float t = 0.f;
        for (int n = 0; n < B; ++n) t += lossv[n];             // index order
        a.loss[i] = t * invB;
      }
      __syncthreads();
    }

    // ---- backward and R-backward ----------------------------------------------------------------------------
    {
      int pos = wsize, hoff = 2 * B * hidden;
      int64_t off = P;
      float* Dl = D0; float* RDl = RD0;                        // errors of layer l
      float* Dn = DB; float* RDn = DB + B * dmax;              // errors of layer l-1 (written here)
      for (int l = L; l >= 1; --l) {
        const int dout = a.dims[l], din = a.dims[l - 1];
        pos -= dout * (din + 1) + dout;
        off -= (int64_t)dout * din + dout;
        const float* Ain; const float* RAin;
        if (l > 1) { hoff -= 2 * B * din; Ain = AH + hoff; RAin = Ain + B * din; } else { Ain = A0; RAin = nullptr; }
        // weight gradient and its R-companion: gW = d^T a, HzW = Rd^T a + d^T Ra (sums over the minibatch)
        for (int e = tid; e < dout * din; e += kTinyThreads) {
          const int j = e / din, kk = e - j * din;
          float gs = 0.f, hs = 0.f;
          if (RAin) {
#pragma unroll 4
            for (int n = 0; n < B; ++n) {
              const float dv = Dl[n * dmax + j], av = Ain[n * din + kk];
              gs = fmaf(dv, av, gs);
              hs = fmaf(RDl[n * dmax + j], av, hs);
              hs = fmaf(dv, RAin[n * din + kk], hs);
            }
          } else {
#pragma unroll 4
            for (int n = 0; n < B; ++n) {
              const float av = Ain[n * din + kk];
              gs = fmaf(Dl[n * dmax + j], av, gs);
              hs = fmaf(RDl[n * dmax + j], av, hs);
            }
          }
          GL[off + e] = gs; HL[off + e] = hs;
        }
        for (int j = tid; j < dout; j += kTinyThreads) {       // bias gradients: column sums
          float gs = 0.f, hs = 0.f;
          for (int n = 0; n < B; ++n) { gs += Dl[n * dmax + j]; hs += RDl[n * dmax + j]; }
          GL[off + (int64_t)dout * din + j] = gs; HL[off + (int64_t)dout * din + j] = hs;
        }
        // data gradient through W_l, masked by the ReLU of layer l-1: d' = (d W) * [a > 0], Rd' = (Rd W + d V) * [a > 0]
        if (l > 1) {
          for (int o = tid; o < B * din; o += kTinyThreads) {
            const int n = o / din, kk = o - n * din;
            float ds = 0.f, rds = 0.f;
#pragma unroll 4
            for (int j = 0; j < dout; ++j) {
              const float dv = Dl[n * dmax + j], wv = Wp[pos + j * (din + 1) + kk];
              ds = fmaf(dv, wv, ds);
              rds = fmaf(RDl[n * dmax + j], wv, rds);
              rds = fmaf(dv, Zp[pos + j * (din + 1) + kk], rds);
            }
            const bool on = Ain[o] > 0.f;
            Dn[n * dmax + kk] = on ? ds : 0.f; RDn[n * dmax + kk] = on ? rds : 0.f;
          }
        }
        __syncthreads();
        float* t0 = Dl; Dl = Dn; Dn = t0; t0 = RDl; RDl = RDn; RDn = t0;
      }
    }

    // ---- D = z*Hz, block mean along fan-in, moments, update (same arithmetic as update_kernel) ----------------
    {
      float* m_g = a.m + (int64_t)i * a.Pp; float* v_g = a.v + (int64_t)i * a.Pp;
      float* g_g = a.g + (int64_t)i * a.Pp; float* hz_g = a.hz + (int64_t)i * a.Pp;
      const int nq = Pq >> 2;
      const float inv_b = 1.0f / (float)a.avg_block;
      const int group_lanes = a.avg_block >> 2;
      for (int q0 = 0; q0 < nq; q0 += kTinyThreads) {          // (uniform trip count: every lane takes the shuffles)
        const int q = q0 + tid;
        const bool valid = q < nq;
        const int64_t e0 = (int64_t)q << 2;
        float4 T = make_float4(0.f, 0.f, 0.f, 0.f), M = T, V = T, Cn = T, G = T, H = T;
        uint32_t zb4 = 0;
        bool avg = false;
        if (valid) {
          if (q0 == 0) {
            T = T0; M = M0; V = V0; Cn = C0;
          } else {
            T = reinterpret_cast<const float4*>(th_g)[q]; M = reinterpret_cast<const float4*>(m_g)[q];
            V = reinterpret_cast<const float4*>(v_g)[q];
            Cn = reinterpret_cast<const float4*>(a.centre)[q];
          }
          G = reinterpret_cast<const float4*>(GL)[q]; H = reinterpret_cast<const float4*>(HL)[q];
          zb4 = ZW[e0 >> 5] >> (e0 & 31);
          // biases are not averaged: is this group of four inside a weight matrix?
          int64_t o2 = 0;
          for (int l = 1; l <= L; ++l) {
            const int64_t wn = (int64_t)a.dims[l] * a.dims[l - 1];
            avg = avg || (e0 >= o2 && e0 < o2 + wn);
            o2 += wn + a.dims[l];
          }
          avg = avg && a.avg_block > 1;
        }
        const float g[4] = {G.x, G.y, G.z, G.w}, hz[4] = {H.x, H.y, H.z, H.w};
        float th[4] = {T.x, T.y, T.z, T.w}, mm[4] = {M.x, M.y, M.z, M.w}, vv[4] = {V.x, V.y, V.z, V.w};
        const float cc[4] = {Cn.x, Cn.y, Cn.z, Cn.w};
        float D[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) D[e] = ((zb4 >> e) & 1u) ? hz[e] : -hz[e];      // Hutchinson: z * Hz
        float Ds[4] = {D[0], D[1], D[2], D[3]};
        if (a.avg_block == 2) {
          const float p0 = 0.5f * (D[0] + D[1]), p1 = 0.5f * (D[2] + D[3]);
          if (avg) { Ds[0] = Ds[1] = p0; Ds[2] = Ds[3] = p1; }
        } else if (a.avg_block >= 4) {
          float s = (D[0] + D[1]) + (D[2] + D[3]);
          for (int o = 1; o < group_lanes; o <<= 1) s += __shfl_xor(s, o);
          s *= inv_b;
          if (avg) { Ds[0] = Ds[1] = Ds[2] = Ds[3] = s; }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          mm[e] = a.beta1 * mm[e] + (1.0f - a.beta1) * g[e];
          vv[e] = a.beta2 * vv[e] + (1.0f - a.beta2) * (Ds[e] * Ds[e]);
          const float mhat = mm[e] * ib1, vhat = vv[e] * ib2;
          th[e] = th[e] - a.lr * (mhat / (tiny_denom(vhat, a.hpow) + a.eps));
          const float d = th[e] - cc[e];
          if (valid && e0 + e < P) nsum += d * d;
        }
        if (valid) {
          // (a last group that reaches past P touches the row's padding, which holds zeros and stays zero: g = Hz = 0)
          reinterpret_cast<float4*>(th_g)[q] = make_float4(th[0], th[1], th[2], th[3]);
          reinterpret_cast<float4*>(m_g)[q] = make_float4(mm[0], mm[1], mm[2], mm[3]);
          reinterpret_cast<float4*>(v_g)[q] = make_float4(vv[0], vv[1], vv[2], vv[3]);
          reinterpret_cast<float4*>(g_g)[q] = G;
          reinterpret_cast<float4*>(hz_g)[q] = H;
        }
      }
    }
  } else {
    // a frozen worker only reports its distance to the centre
    const int nq = (int)((P + 3) >> 2);
    for (int q = tid; q < nq; q += kTinyThreads) {
      const float4 t = reinterpret_cast<const float4*>(th_g)[q], c = reinterpret_cast<const float4*>(a.centre)[q];
      const float d0 = t.x - c.x, d1 = t.y - c.y, d2 = t.z - c.z, d3 = t.w - c.w;
      nsum += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
    }
  }
  double ws = (double)nsum;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) ws += __shfl_xor(ws, o);
  if (lane == 0) red[wave] = ws;
  __syncthreads();
  if (tid == 0) {
    double t = 0.0;
    for (int w = 0; w < kTinyThreads / 64; ++w) t += red[w];
    a.partials[(int64_t)i * a.n_blocks] = t;
    for (int b = 1; b < a.n_blocks; ++b) a.partials[(int64_t)i * a.n_blocks + b] = 0.0;
  }
}

int tiny_lds_floats(const dw_config& c, int64_t P) {
  int64_t wsize = 0, hidden = 0, dmax = DW_MAX_CLASSES;
  for (int l = 1; l <= c.n_layers; ++l) {
    wsize += (int64_t)c.dims[l] * (c.dims[l - 1] + 1) + c.dims[l];
    if (l < c.n_layers) { hidden += c.dims[l]; if (c.dims[l] > dmax) dmax = c.dims[l]; }
  }
  const int64_t B = c.batch, Pq = (P + 3) / 4 * 4;
  const int64_t total = 2 * wsize + B * c.dims[0] + 2 * B * hidden + 4 * B * dmax + 2 * Pq + 2 * ((P + 63) / 64) + B + 64;
  return total > (1 << 30) ? (1 << 30) : (int)total;
}

}  // namespace

// A model takes this path when it is fp32 without a convolutional front end, one Hutchinson probe per step, the
// AdaHessian step, an averaging block inside one wave's reach, and everything listed above fits in LDS.
bool tiny_step_ok(const dw_config& c, const Layout& lay) {
  if (c.n_layers < 1 || c.dtype != DW_F32 || c.n_conv != 0 || c.n_samples > 1 || c.optimizer != DW_OPT_ADAHESSIAN)
    return false;
  if (c.avg_block > 64 || lay.P > 16384 || c.batch > 1024) return false;
  return tiny_lds_floats(c, lay.P) <= kTinyMaxLdsFloats;
}

hipError_t launch_tiny_step(const dw_config& c, char* ws, const Layout& lay, const void* d_x, const int32_t* d_y,
                            const uint32_t* d_zbits, const UpdateArgs& u, const uint64_t* keys_host, float* d_loss,
                            hipStream_t s) {
  KernelScope ks(KC_STEP, s);
  TinyArgs a{};
  a.x = reinterpret_cast<const float*>(d_x); a.y = d_y;
  a.zbits_in = d_zbits; a.z_stride_in = 2 * ((lay.P + 63) / 64);
  a.zbits = reinterpret_cast<uint32_t*>(ws + lay.zbits); a.z_stride = lay.z_stride;
  a.theta = u.theta; a.m = u.m; a.v = u.v; a.centre = u.centre;
  a.g = reinterpret_cast<float*>(ws + lay.g); a.hz = reinterpret_cast<float*>(ws + lay.hz);
  a.partials = u.partials; a.n_blocks = (int)lay.n_upd_blocks;
  for (int l = 1; l < c.n_layers; ++l) a.act[l] = reinterpret_cast<float*>(ws + lay.act[l]);
  a.loss = d_loss;
  a.P = lay.P; a.Pp = lay.Pp; a.L = c.n_layers; a.B = c.batch; a.k = c.k;
  for (int l = 0; l <= c.n_layers; ++l) a.dims[l] = c.dims[l];
  a.avg_block = c.avg_block;
  a.lr = c.lr; a.beta1 = c.beta1; a.beta2 = c.beta2; a.eps = c.eps; a.hpow = c.hpow;
  a.active_mask = u.active_mask;
  for (int i = 0; i < DW_MAX_K; ++i) a.key[i] = i < c.k ? keys_host[i] : 0;
  a.sc = u.sc;
  const int smem = tiny_lds_floats(c, lay.P) * (int)sizeof(float);
  static LdsLimitOnce lds_limit;
  const hipError_t e = lds_limit.raise(reinterpret_cast<const void*>(tiny_step_kernel), kTinyMaxLdsFloats * (int)sizeof(float));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(tiny_step_kernel, dim3((unsigned)c.k), dim3(kTinyThreads), smem, s, a);
  return hipGetLastError();
}

}  // namespace dw
