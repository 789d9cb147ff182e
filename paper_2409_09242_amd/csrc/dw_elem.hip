// Streaming kernels of the optimizer and of the communication round (gfx950, wave64).
//
//   update_kernel   Section IV-B: D = z*Hz (Hutchinson, one sample), block mean of D along fan-in,
//                   Adam-like moments with D in the second moment, bias correction, parameter update
//                   (the preconditioned step of eq.(4)); also the squared distance of the new parameters
//                   to the centre, which the next communication round turns into u (Section V-B).
//   weight_kernel   Section V-B: u = log||theta_i - centre||, history, raw score a (eq.(10)-(11)),
//                   piecewise-linear weights h1(a), h2(a).
//   pull_kernel     Section V-B eq.(12)-(13): elastic pull of every participating worker and of the centre.
//
// All three are bound by HBM bandwidth.  One thread owns the same four consecutive parameters of every
// worker: the centre values stay in registers while the block walks over the k replicas, so the centre is
// read once per launch, and the reduction over workers into the centre needs no atomics.
#include <cstddef>
#include <type_traits>

#include "dw_internal.h"
#include "dw_device_util.h"

namespace dw {

__device__ __forceinline__ float sign_from_bit(uint32_t bits, int b) {
  // bit set -> +1, clear -> -1
  return ((bits >> b) & 1u) ? 1.0f : -1.0f;
}

__device__ __forceinline__ bool in_bias(const BiasRanges& br, int64_t j) {
  bool r = false;
#pragma unroll
  for (int l = 0; l < DW_MAX_LAYERS; ++l)
    if (l < br.n) r = r || (j >= br.begin[l] && j < br.end[l]);
  return r;
}

__device__ __forceinline__ bool in_fused(const FusedRanges& fr, int64_t j) {
  bool r = false;
#pragma unroll
  for (int l = 0; l < DW_MAX_LAYERS; ++l)
    if (l < fr.n) r = r || (j >= fr.begin[l] && j < fr.end[l]);
  return r;
}

__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
  return x;
}

__device__ __forceinline__ float denom_pow(float vhat, float hpow) {
  // (sqrt(v_hat))^hpow
  if (hpow == 1.0f) return sqrtf(vhat);
  if (hpow == 0.0f) return 1.0f;
  if (hpow == 2.0f) return vhat;
  return powf(vhat, 0.5f * hpow);
}

// OPT: the local step (DW_OPT_*).  The baselines' first-order steps (Section II eq.(3); Section VI) move 12 bytes
// (SGD: g and theta read, theta written) or 20 bytes (momentum: also the velocity read and written) per parameter
// and worker where the AdaHessian step moves 32.
template <bool HAS_B16, int OPT>
__global__ __launch_bounds__(kUpdThreads) void update_kernel(UpdateArgs a) {
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int64_t nq = (a.P + 3) >> 2;      // caller-supplied g / Hz rows end at P
  // which chunk of kUpdChunk parameters: the block index, or an entry of the list (read from the kernel-argument
  // block by a scalar load: indexing the by-value argument with a variable would copy it to scratch memory)
  int blk = blockIdx.x;
  if (a.n_list > 0) {
    typedef const char __attribute__((address_space(4)))* karg_bytes;
    typedef const int __attribute__((address_space(4)))* karg_ints;
    const karg_bytes ka = (karg_bytes)__builtin_amdgcn_kernarg_segment_ptr();
    blk = ((karg_ints)(ka + offsetof(UpdateArgs, block_list)))[blockIdx.x];
  }
  const int64_t qbase = (int64_t)blk * (kUpdThreads * kUpdQuads) + tid;
  __shared__ double wave_part[DW_MAX_K][kUpdThreads / 64];

  // a block whose parameters were all updated by a weight-gradient kernel has nothing to do unless some worker
  // is frozen (then it still reports that worker's distance to the centre)
  if (a.fused.n > 0) {
    const int64_t j0 = (int64_t)blk * kUpdChunk, j1 = j0 + kUpdChunk;
    bool inside = false;
    for (int l = 0; l < a.fused.n; ++l) inside = inside || (j0 >= a.fused.begin[l] && j1 <= a.fused.end[l]);
    const uint64_t all = a.k >= 64 ? ~0ull : ((1ull << a.k) - 1ull);
    if (inside && (a.active_mask & all) == all) {
      if (tid < a.k) a.partials[(int64_t)tid * a.n_blocks + blk] = 0.0;
      return;
    }
  }

  float4 cen[kUpdQuads];
  bool valid[kUpdQuads], avg[kUpdQuads], fz[kUpdQuads];
  uint32_t zshift[kUpdQuads];
#pragma unroll
  for (int u = 0; u < kUpdQuads; ++u) {
    const int64_t q = qbase + (int64_t)u * kUpdThreads;
    fz[u] = a.fused.n > 0 && in_fused(a.fused, q << 2);
    valid[u] = q < nq;
    cen[u] = valid[u] ? reinterpret_cast<const float4*>(a.centre)[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    avg[u] = a.avg_block > 1 && !in_bias(a.bias, q << 2);
    zshift[u] = (uint32_t)((q << 2) & 31);
  }
  const float inv_b = 1.0f / (float)a.avg_block;
  const int group_lanes = a.avg_block >> 2;           // lanes that share one averaging block (when b > 4)

  // a launch of few chunks spreads the workers over the grid's second dimension: the chain of k dependent memory
  // round trips per block would otherwise set the kernel's duration
  const int i0 = gridDim.y > 1 ? (int)blockIdx.y : 0, i1 = gridDim.y > 1 ? i0 + 1 : a.k;
  for (int i = i0; i < i1; ++i) {
    const bool active = (a.active_mask >> i) & 1ull;
    float nsum = 0.f;
    float4* th4 = reinterpret_cast<float4*>(a.theta + (int64_t)i * a.Pp);
    if (active) {
      float4* m4 = reinterpret_cast<float4*>(a.m + (int64_t)i * a.Pp);
      float4* v4 = reinterpret_cast<float4*>(a.v + (int64_t)i * a.Pp);
      const float4* g4 = reinterpret_cast<const float4*>(a.g + (int64_t)i * a.g_stride);
      const float4* h4 = reinterpret_cast<const float4*>(a.hz + (int64_t)i * a.g_stride);
      const uint32_t* zb = a.zbits + (int64_t)i * a.z_stride;
      const float ib1 = a.sc.inv_bc1[i], ib2 = a.sc.inv_bc2[i];
      float4 G[kUpdQuads], H[kUpdQuads], T[kUpdQuads], M[kUpdQuads], V[kUpdQuads];
      uint32_t Z[kUpdQuads];
#pragma unroll
      for (int u = 0; u < kUpdQuads; ++u) {
        const int64_t q = qbase + (int64_t)u * kUpdThreads;
        G[u] = H[u] = T[u] = M[u] = V[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        Z[u] = 0;
        if (valid[u] && !fz[u]) {
          G[u] = nt_load4(g4 + q); T[u] = nt_load4(th4 + q);
          if (OPT != DW_OPT_SGD) M[u] = nt_load4(m4 + q);
          if (OPT == DW_OPT_ADAHESSIAN) {
            H[u] = nt_load4(h4 + q); V[u] = nt_load4(v4 + q);
            Z[u] = zb[q >> 3] >> zshift[u];
          }
        }
      }
      if (OPT != DW_OPT_ADAHESSIAN) {
        // first-order step of a baseline: theta -= lr * g, or the same through the velocity b = momentum * b + g
#pragma unroll
        for (int u = 0; u < kUpdQuads; ++u) {
          const int64_t q = qbase + (int64_t)u * kUpdThreads;
          float g[4] = {G[u].x, G[u].y, G[u].z, G[u].w};
          float th[4] = {T[u].x, T[u].y, T[u].z, T[u].w};
          float bb[4] = {M[u].x, M[u].y, M[u].z, M[u].w};
          const float cc[4] = {cen[u].x, cen[u].y, cen[u].z, cen[u].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (OPT == DW_OPT_MOMENTUM) { bb[e] = a.momentum * bb[e] + g[e]; th[e] = th[e] - a.lr * bb[e]; }
            else th[e] = th[e] - a.lr * g[e];
            const float d = th[e] - cc[e];
            nsum += d * d;
          }
          if (valid[u]) {
            nt_store4(th4 + q, make_float4(th[0], th[1], th[2], th[3]));
            if (OPT == DW_OPT_MOMENTUM) nt_store4(m4 + q, make_float4(bb[0], bb[1], bb[2], bb[3]));
            if (HAS_B16) {
              ushort4 w;
              w.x = f32_to_bf16_rne(th[0]); w.y = f32_to_bf16_rne(th[1]);
              w.z = f32_to_bf16_rne(th[2]); w.w = f32_to_bf16_rne(th[3]);
              reinterpret_cast<ushort4*>(a.wb16 + (int64_t)i * a.Pp)[q] = w;
            }
          }
        }
      }
#pragma unroll
      for (int u = 0; OPT == DW_OPT_ADAHESSIAN && u < kUpdQuads; ++u) {
        const int64_t q = qbase + (int64_t)u * kUpdThreads;
        float g[4] = {G[u].x, G[u].y, G[u].z, G[u].w};
        float hz[4] = {H[u].x, H[u].y, H[u].z, H[u].w};
        float th[4] = {T[u].x, T[u].y, T[u].z, T[u].w};
        float mm[4] = {M[u].x, M[u].y, M[u].z, M[u].w};
        float vv[4] = {V[u].x, V[u].y, V[u].z, V[u].w};
        // quads updated elsewhere run on zeros and add nothing to the distance
        const float cc[4] = {fz[u] ? 0.f : cen[u].x, fz[u] ? 0.f : cen[u].y, fz[u] ? 0.f : cen[u].z, fz[u] ? 0.f : cen[u].w};
        float D[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)                                              // Hutchinson: z * Hz, or its mean
          D[e] = a.d_scale > 0.f ? hz[e] * a.d_scale : sign_from_bit(Z[u], e) * hz[e];
        // spatial average over avg_block consecutive parameters (all lanes take part in the shuffles)
        float Ds[4] = {D[0], D[1], D[2], D[3]};
        if (a.avg_block == 2) {
          const float p0 = 0.5f * (D[0] + D[1]), p1 = 0.5f * (D[2] + D[3]);
          if (avg[u]) { Ds[0] = Ds[1] = p0; Ds[2] = Ds[3] = p1; }
        } else if (a.avg_block >= 4) {
          float s = (D[0] + D[1]) + (D[2] + D[3]);
          for (int off = 1; off < group_lanes; off <<= 1) s += __shfl_xor(s, off);
          s *= inv_b;
          if (avg[u]) { Ds[0] = Ds[1] = Ds[2] = Ds[3] = s; }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          mm[e] = a.beta1 * mm[e] + (1.0f - a.beta1) * g[e];
          vv[e] = a.beta2 * vv[e] + (1.0f - a.beta2) * (Ds[e] * Ds[e]);
          const float mhat = mm[e] * ib1;
          const float vhat = vv[e] * ib2;
          th[e] = th[e] - a.lr * (mhat / (denom_pow(vhat, a.hpow) + a.eps));
          const float d = th[e] - cc[e];
          nsum += d * d;
        }
        if (valid[u] && !fz[u]) {
          nt_store4(th4 + q, make_float4(th[0], th[1], th[2], th[3]));
          nt_store4(m4 + q, make_float4(mm[0], mm[1], mm[2], mm[3]));
          nt_store4(v4 + q, make_float4(vv[0], vv[1], vv[2], vv[3]));
          if (HAS_B16) {
            ushort4 w;
            w.x = f32_to_bf16_rne(th[0]); w.y = f32_to_bf16_rne(th[1]);
            w.z = f32_to_bf16_rne(th[2]); w.w = f32_to_bf16_rne(th[3]);
            reinterpret_cast<ushort4*>(a.wb16 + (int64_t)i * a.Pp)[q] = w;
          }
        }
      }
    } else {
#pragma unroll
      for (int u = 0; u < kUpdQuads; ++u) {
        const int64_t q = qbase + (int64_t)u * kUpdThreads;
        if (valid[u]) {
          const float4 t = th4[q];
          const float d0 = t.x - cen[u].x, d1 = t.y - cen[u].y, d2 = t.z - cen[u].z, d3 = t.w - cen[u].w;
          nsum += (d0 * d0 + d1 * d1) + (d2 * d2 + d3 * d3);
        }
      }
    }
    const double ws = wave_sum((double)nsum);
    if (lane == 0) wave_part[i][wave] = ws;
  }
  __syncthreads();
  if (tid >= i0 && tid < i1) {
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kUpdThreads / 64; ++w) s += wave_part[tid][w];
    a.partials[(int64_t)tid * a.n_blocks + blk] = s;
  }
}

hipError_t launch_update(const UpdateArgs& args, int n_blocks, hipStream_t s) {
  KernelScope ks(KC_UPDATE, s);
  UpdateArgs a = args;
  a.n_blocks = n_blocks; a.n_list = 0;
  int grid = n_blocks, grid_y = 1;
  // When weight-gradient kernels have updated most ranges and no worker is frozen, only the chunks that touch
  // other parameters (biases, small layers) have work: launch those, after clearing everybody's partial sums.
  const uint64_t all = a.k >= 64 ? ~0ull : ((1ull << a.k) - 1ull);
  if (a.fused.n > 0 && (a.active_mask & all) == all) {
    int n = 0;
    bool fits = true;
    for (int b = 0; b < n_blocks && fits; ++b) {
      const int64_t j0 = (int64_t)b * kUpdChunk, j1 = j0 + kUpdChunk;
      bool inside = false;
      for (int l = 0; l < a.fused.n; ++l) {
        if (j0 >= a.fused.begin[l] && j1 <= a.fused.end[l]) {
          inside = true;
          // skip ahead to the last chunk that is still inside this range
          const int64_t last = a.fused.end[l] / kUpdChunk - 1;
          if (last > b) b = (int)last;
          break;
        }
      }
      if (inside) continue;
      if (n == 64) fits = false; else a.block_list[n++] = b;
    }
    if (fits && n > 0) {
      hipError_t e = launch_fill_zero(a.partials, (size_t)(((int64_t)a.k * n_blocks * sizeof(double) + 15) / 16 * 16), s);   // the array is carved in 256-byte units
      if (e != hipSuccess) return e;
      a.n_list = n; grid = n; grid_y = a.k;
    }
  }
  // few chunks (small models): one worker per block row as well; with many chunks a block walks through the workers
  // and reads its piece of the centre once
  if (a.n_list == 0 && n_blocks < 1024 && a.k > 1) grid_y = a.k;
  const dim3 g3(grid, grid_y), b3(kUpdThreads);
  auto launch = [&](auto b16, auto opt) {
    hipLaunchKernelGGL((update_kernel<decltype(b16)::value, decltype(opt)::value>), g3, b3, 0, s, a);
  };
  auto by_opt = [&](auto b16) {
    if (a.optimizer == DW_OPT_SGD) launch(b16, std::integral_constant<int, DW_OPT_SGD>{});
    else if (a.optimizer == DW_OPT_MOMENTUM) launch(b16, std::integral_constant<int, DW_OPT_MOMENTUM>{});
    else launch(b16, std::integral_constant<int, DW_OPT_ADAHESSIAN>{});
  };
  if (a.wb16) by_opt(std::true_type{}); else by_opt(std::false_type{});
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// Dynamic-weight scalars: one block per worker.
// ---------------------------------------------------------------------------------------------------
// Dynamic-weight scalars of worker i from its squared distance S (Section V-B): u = log||theta_i - centre||, the raw
// score a over the history ring (eq.(10)-(11)), the piecewise-linear weights h1(a), h2(a).  `write`: record u in the
// ring and the scores in memory (one caller per worker and round); the ring slot of this round is not read here, so
// other blocks may evaluate the same worker without writing while one block records.
// man1, man2: the caller's weights of this worker (DW_MANUAL).
__device__ __forceinline__ void weight_scalars(const WeightArgs& a, int i, double S, float man1, float man2, bool write,
                                               float* omh1, float* h2o) {
  // u = log ||theta_i - centre||_2 (natural log; squared norm floored so identical vectors stay finite)
  const double u = 0.5 * log(S > 1e-30 ? S : 1e-30);
  const int ring = a.p + 1;
  double* R = a.u_ring + (int64_t)i * (DW_MAX_P + 1);
  // raw score: c_0 weighs the newest difference u_t - u_{t-1}, c_1 the one before, ...; differences the
  // history cannot supply yet contribute nothing
  double sc = 0.0;
  for (int j = 0; j < a.p; ++j) {
    if (j + 1 >= a.n_valid) break;
    const int hi = (a.slot - j + 2 * ring) % ring;
    const int lo = (a.slot - j - 1 + 2 * ring) % ring;
    sc += (double)a.c[j] * ((j == 0 ? u : R[hi]) - R[lo]);
  }
  double h1, h2;
  const double alpha = a.alpha, kappa = a.kappa;
  if (a.mode == DW_FIXED) {
    h1 = alpha; h2 = alpha;
  } else if (a.mode == DW_MANUAL) {
    h1 = man1; h2 = man2;
  } else if (sc < kappa) {
    h1 = 1.0; h2 = 0.0;
  } else if (sc <= 0.0) {
    h1 = 1.0 + (1.0 - alpha) / kappa * (sc - kappa);
    h2 = -alpha / kappa * sc + alpha;
  } else {
    h1 = alpha; h2 = alpha;
  }
  *omh1 = (float)(1.0 - h1);
  *h2o = (float)h2;
  if (write) {
    R[a.slot] = u;
    double* out = a.score + (int64_t)i * 4;
    out[0] = u; out[1] = sc; out[2] = h1; out[3] = h2;
    a.omh1[i] = (float)(1.0 - h1);
    a.h2[i] = (float)h2;
  }
}

__global__ __launch_bounds__(256) void weight_kernel(WeightArgs a) {
  const int i = blockIdx.x;
  const int tid = threadIdx.x;
  __shared__ double red[256 / 64];
  double s = 0.0;
  for (int b = tid; b < a.n_blocks; b += 256) s += a.partials[(int64_t)i * a.n_blocks + b];
  for (int b = tid; b < a.n_blocks_f; b += 256) s += a.partials_f[(int64_t)i * a.n_blocks_f + b];
  s = wave_sum(s);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  if (tid != 0) return;
  double S = 0.0;
  for (int w = 0; w < 256 / 64; ++w) S += red[w];
  float o, w;
  weight_scalars(a, i, S, a.man_h1[i], a.man_h2[i], true, &o, &w);      // (i is uniform: scalar loads)
}

hipError_t launch_weights(const WeightArgs& a, hipStream_t s) {
  KernelScope ks(KC_WEIGHTS, s);
  hipLaunchKernelGGL(weight_kernel, dim3(a.k), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// Elastic pull.  theta_i <- centre + (1-h1_i)(theta_i - centre)  (the same value as eq.(12), written so
// that h1 = 1 returns the centre exactly);  centre <- centre + sum_i h2_i (theta_i - centre)  (eq.(13)).
// Sequential rounds apply eq.(13) after every worker instead: the thread that owns a parameter keeps the
// centre in a register and walks the workers in index order, so the bytes moved are the same.
// ---------------------------------------------------------------------------------------------------
// FUSED_W: a model with few partial sums computes the weights inside the pull (every block for itself, in the same
// order, so all blocks pull with the same values; block 0 records them): one launch per round instead of two.
template <bool HAS_B16, bool FUSED_W>
__global__ __launch_bounds__(kUpdThreads) void pull_kernel(PullArgs a, WeightArgs wa) {
  __shared__ float s_omh1[DW_MAX_K], s_h2[DW_MAX_K];
  if (FUSED_W) {
    const int i = threadIdx.x;
    if (i < wa.k) {
      double S = 0.0;
      for (int b = 0; b < wa.n_blocks; ++b) S += wa.partials[(int64_t)i * wa.n_blocks + b];
      for (int b = 0; b < wa.n_blocks_f; ++b) S += wa.partials_f[(int64_t)i * wa.n_blocks_f + b];
      // the caller's weights sit in the kernel-argument block behind the first argument; they are read from there by
      // address (indexing the by-value argument with the thread index would copy it to scratch memory)
      typedef const char __attribute__((address_space(4)))* karg_bytes;
      typedef const float __attribute__((address_space(4)))* karg_floats;
      constexpr size_t wa_at = (sizeof(PullArgs) + alignof(WeightArgs) - 1) / alignof(WeightArgs) * alignof(WeightArgs);
      const karg_bytes ka = (karg_bytes)__builtin_amdgcn_kernarg_segment_ptr();
      const float man1 = ((karg_floats)(ka + wa_at + offsetof(WeightArgs, man_h1)))[i];
      const float man2 = ((karg_floats)(ka + wa_at + offsetof(WeightArgs, man_h2)))[i];
      weight_scalars(wa, i, S, man1, man2, blockIdx.x == 0, &s_omh1[i], &s_h2[i]);
    }
    __syncthreads();
  }
  const int64_t nq = a.Pp >> 2;
  const int64_t qbase = (int64_t)blockIdx.x * (kUpdThreads * kUpdQuads) + threadIdx.x;
  float4 cen[kUpdQuads], acc[kUpdQuads];
  bool valid[kUpdQuads];
#pragma unroll
  for (int u = 0; u < kUpdQuads; ++u) {
    const int64_t q = qbase + (int64_t)u * kUpdThreads;
    valid[u] = q < nq;
    cen[u] = valid[u] ? reinterpret_cast<const float4*>(a.centre)[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    acc[u] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  for (int i = 0; i < a.k; ++i) {
    if (!((a.part_mask >> i) & 1ull)) continue;
    const float o = FUSED_W ? s_omh1[i] : a.omh1[i], w = FUSED_W ? s_h2[i] : a.h2[i];
    float4* th4 = reinterpret_cast<float4*>(a.theta + (int64_t)i * a.Pp);
    float4 T[kUpdQuads];
#pragma unroll
    for (int u = 0; u < kUpdQuads; ++u) {
      const int64_t q = qbase + (int64_t)u * kUpdThreads;
      T[u] = valid[u] ? nt_load4(th4 + q) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < kUpdQuads; ++u) {
      const int64_t q = qbase + (int64_t)u * kUpdThreads;
      const float d0 = T[u].x - cen[u].x, d1 = T[u].y - cen[u].y, d2 = T[u].z - cen[u].z, d3 = T[u].w - cen[u].w;
      float4 r;
      r.x = fmaf(o, d0, cen[u].x); r.y = fmaf(o, d1, cen[u].y);
      r.z = fmaf(o, d2, cen[u].z); r.w = fmaf(o, d3, cen[u].w);
      if (a.sequential) {     // eq.(13) takes effect at once: the next worker of the round sees the moved centre
        cen[u].x = fmaf(w, d0, cen[u].x); cen[u].y = fmaf(w, d1, cen[u].y);
        cen[u].z = fmaf(w, d2, cen[u].z); cen[u].w = fmaf(w, d3, cen[u].w);
      } else {
        acc[u].x = fmaf(w, d0, acc[u].x); acc[u].y = fmaf(w, d1, acc[u].y);
        acc[u].z = fmaf(w, d2, acc[u].z); acc[u].w = fmaf(w, d3, acc[u].w);
      }
      if (valid[u]) {
        nt_store4(th4 + q, r);
        if (HAS_B16) {
          ushort4 b;
          b.x = f32_to_bf16_rne(r.x); b.y = f32_to_bf16_rne(r.y);
          b.z = f32_to_bf16_rne(r.z); b.w = f32_to_bf16_rne(r.w);
          reinterpret_cast<ushort4*>(a.wb16 + (int64_t)i * a.Pp)[q] = b;
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kUpdQuads; ++u) {
    const int64_t q = qbase + (int64_t)u * kUpdThreads;
    if (valid[u]) {
      float4 c = cen[u];
      c.x += acc[u].x; c.y += acc[u].y; c.z += acc[u].z; c.w += acc[u].w;
      reinterpret_cast<float4*>(a.centre)[q] = c;
    }
  }
}

hipError_t launch_pull(const PullArgs& a, hipStream_t s) {
  KernelScope ks(KC_PULL, s);
  const int64_t nq = a.Pp >> 2;
  const int n_blocks = (int)((nq + kUpdThreads * kUpdQuads - 1) / (kUpdThreads * kUpdQuads));
  WeightArgs none{};
  if (a.wb16)
    hipLaunchKernelGGL((pull_kernel<true, false>), dim3(n_blocks), dim3(kUpdThreads), 0, s, a, none);
  else
    hipLaunchKernelGGL((pull_kernel<false, false>), dim3(n_blocks), dim3(kUpdThreads), 0, s, a, none);
  return hipGetLastError();
}

// the round of a model with few partial sums per worker in one launch: weights and pull together
bool sync_fusable(const WeightArgs& w, const PullArgs& p) {
  const int64_t nq = p.Pp >> 2;
  const int64_t n_blocks = (nq + kUpdThreads * kUpdQuads - 1) / (kUpdThreads * kUpdQuads);
  return w.n_blocks + w.n_blocks_f <= 16 && n_blocks <= 64;
}

hipError_t launch_weights_and_pull(const WeightArgs& w, const PullArgs& a, hipStream_t s) {
  KernelScope ks(KC_PULL, s);
  const int64_t nq = a.Pp >> 2;
  const int n_blocks = (int)((nq + kUpdThreads * kUpdQuads - 1) / (kUpdThreads * kUpdQuads));
  if (a.wb16)
    hipLaunchKernelGGL((pull_kernel<true, true>), dim3(n_blocks), dim3(kUpdThreads), 0, s, a, w);
  else
    hipLaunchKernelGGL((pull_kernel<false, true>), dim3(n_blocks), dim3(kUpdThreads), 0, s, a, w);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// Rademacher bits: a stateless counter-based stream on the SplitMix64 output function (Steele, Lea &
// Flood 2014).  64-bit word w of a worker is mix(key + GAMMA*(w+1)); element j of z is +1 when bit
// (j mod 64) of word j/64 is set.  The paper only asks for a Rademacher vector (Section IV-B).
// ---------------------------------------------------------------------------------------------------
struct RadKeys { uint64_t key[DW_MAX_K]; };

__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

__global__ __launch_bounds__(256) void rademacher_kernel(uint32_t* zbits, int64_t z_stride, int64_t n_words64,
                                                         RadKeys keys, uint64_t active_mask) {
  const int i = blockIdx.y;
  if (!((active_mask >> i) & 1ull)) return;
  const int64_t w = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (w >= n_words64) return;
  const uint64_t x = mix64(keys.key[i] + 0x9E3779B97F4A7C15ull * (uint64_t)(w + 1));
  uint2 o; o.x = (uint32_t)x; o.y = (uint32_t)(x >> 32);
  reinterpret_cast<uint2*>(zbits + (int64_t)i * z_stride)[w] = o;
}

hipError_t launch_rademacher(uint32_t* zbits, int64_t z_stride, int64_t n_words64, const uint64_t* keys_host,
                             int k, uint64_t active_mask, hipStream_t s) {
  KernelScope ks(KC_RADEMACHER, s);
  RadKeys keys;
  for (int i = 0; i < DW_MAX_K; ++i) keys.key[i] = i < k ? keys_host[i] : 0;
  dim3 grid((unsigned)((n_words64 + 255) / 256), (unsigned)k);
  hipLaunchKernelGGL(rademacher_kernel, grid, dim3(256), 0, s, zbits, z_stride, n_words64, keys, active_mask);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// Transposed copy of one layer's part of z.  The data gradient through W_l [R = d_l][C = d_{l-1}] contracts over
// the R index, so its large-tile kernel wants the sign bits of a column of V_l (fixed c, consecutive r) side by
// side: bit (r, c) of z sits at woff + r*C + c, its copy at woff + c*R + r of zt.  A block moves a 512 x 512 bit
// super-tile: 64-byte row pieces in, 64 transposes of 64 x 64 bits in LDS (tile (a, b) and tile (b, a) swap places),
// 64-byte row pieces out.  A 64 x 64 tile is one 64-bit word per lane; it is transposed by six exchange steps with
// the lane 32, 16, .. 1 away (swap the off-diagonal blocks of every 2j x 2j block).
// Requires R % 128 == 0, C % 128 == 0, woff % 128 == 0.
// ---------------------------------------------------------------------------------------------------
constexpr int kTrEdge = 512;                       // bits
constexpr int kTrRow = kTrEdge / 8 + 8;            // LDS bytes per row (8 bytes of padding)

template <int J>
__device__ __forceinline__ uint64_t transpose64_step(uint64_t w, int lane) {
  // bits whose position has bit J clear
  constexpr uint64_t lo = J == 32 ? 0x00000000FFFFFFFFull : J == 16 ? 0x0000FFFF0000FFFFull : J == 8 ? 0x00FF00FF00FF00FFull
                          : J == 4 ? 0x0F0F0F0F0F0F0F0Full : J == 2 ? 0x3333333333333333ull : 0x5555555555555555ull;
  const uint64_t p = __shfl_xor(w, J);
  return (lane & J) ? ((w & ~lo) | ((p >> J) & lo)) : ((w & lo) | ((p << J) & ~lo));
}
__device__ __forceinline__ uint64_t transpose64(uint64_t w, int lane) {
  w = transpose64_step<32>(w, lane); w = transpose64_step<16>(w, lane); w = transpose64_step<8>(w, lane);
  w = transpose64_step<4>(w, lane); w = transpose64_step<2>(w, lane); w = transpose64_step<1>(w, lane);
  return w;
}

__global__ __launch_bounds__(256) void transpose_bits_kernel(const uint32_t* z, int64_t z_stride, uint32_t* zt, int64_t zt_stride, int64_t woff,
                                                             int R, int C, uint64_t active_mask) {
  __shared__ __attribute__((aligned(16))) char tile[kTrEdge * kTrRow];
  const int worker = blockIdx.z;
  if (!((active_mask >> worker) & 1ull)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r0 = blockIdx.y * kTrEdge, c0 = blockIdx.x * kTrEdge;
  const char* src = reinterpret_cast<const char*>(z + (int64_t)worker * z_stride) + (woff >> 3);
  char* dst = reinterpret_cast<char*>(zt + (int64_t)worker * zt_stride) + (woff >> 3);
  for (int u = tid; u < kTrEdge * 4; u += 256) {
    const int row = u >> 2, q = u & 3;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r0 + row < R && c0 + q * 128 < C)
      v = *reinterpret_cast<const uint4*>(src + (((int64_t)(r0 + row) * C + c0) >> 3) + q * 16);
    uint2* t = reinterpret_cast<uint2*>(tile + row * kTrRow + q * 16);
    t[0] = make_uint2(v.x, v.y); t[1] = make_uint2(v.z, v.w);
  }
  __syncthreads();
  // 8 x 8 tiles: units are the 8 diagonal tiles and the 28 pairs (a, b), (b, a) with a < b
  for (int u = wave; u < 36; u += 4) {
    int a = 0, b = u;                                // u-th pair in the order (0,0..7), (1,1..7), ...
    while (b >= 8 - a) { b -= 8 - a; a += 1; }
    b += a;
    uint64_t* pab = reinterpret_cast<uint64_t*>(tile + (a * 64 + lane) * kTrRow + b * 8);
    uint64_t* pba = reinterpret_cast<uint64_t*>(tile + (b * 64 + lane) * kTrRow + a * 8);
    const uint64_t wab = transpose64(*pab, lane);
    const uint64_t wba = transpose64(*pba, lane);    // the same word when a == b
    *pba = wab;
    if (a != b) *pab = wba;
  }
  __syncthreads();
  for (int u = tid; u < kTrEdge * 4; u += 256) {
    const int row = u >> 2, q = u & 3;
    if (c0 + row < C && r0 + q * 128 < R) {
      const uint2* t = reinterpret_cast<const uint2*>(tile + row * kTrRow + q * 16);
      const uint2 x = t[0], y = t[1];
      *reinterpret_cast<uint4*>(dst + (((int64_t)(c0 + row) * R + r0) >> 3) + q * 16) = make_uint4(x.x, x.y, y.x, y.y);
    }
  }
}

hipError_t launch_transpose_bits(const uint32_t* z, int64_t z_stride, uint32_t* zt, int64_t zt_stride, int64_t woff, int R, int C, int k,
                                 uint64_t active_mask, hipStream_t s) {
  KernelScope ks(KC_RADEMACHER, s);
  const dim3 grid((unsigned)((C + kTrEdge - 1) / kTrEdge), (unsigned)((R + kTrEdge - 1) / kTrEdge), (unsigned)k);
  hipLaunchKernelGGL(transpose_bits_kernel, grid, dim3(256), 0, s, z, z_stride, zt, zt_stride, woff, R, C, active_mask);
  return hipGetLastError();
}

// Running sum of z_j * Hz_j over the probes of one step (Section IV-B with n > 1), one float4 per thread.
// blockIdx.z picks one of the parameter ranges in `keep` (begin and end multiples of 4); what lies between them
// belongs to weight-gradient kernels that keep the sum themselves.
__global__ __launch_bounds__(256) void probe_sum_kernel(float* dacc, const float* hz, const uint32_t* zbits, int64_t Pp,
                                                        int64_t z_stride, uint64_t active_mask, int first,
                                                        FusedRanges keep) {
  const int i = blockIdx.y;
  if (!((active_mask >> i) & 1ull)) return;
  int64_t q0 = 0, q1 = 0;
#pragma unroll
  for (int r = 0; r < DW_MAX_LAYERS; ++r)                    // (static indices: the argument stays in registers)
    if (r == (int)blockIdx.z) { q0 = keep.begin[r] >> 2; q1 = keep.end[r] >> 2; }
  for (int64_t q = q0 + (int64_t)blockIdx.x * 256 + threadIdx.x; q < q1; q += (int64_t)gridDim.x * 256) {
    const float4 h = reinterpret_cast<const float4*>(hz + (int64_t)i * Pp)[q];
    const uint32_t z = zbits[(int64_t)i * z_stride + (q >> 3)] >> ((q << 2) & 31);
    float4 d = first ? make_float4(0.f, 0.f, 0.f, 0.f) : reinterpret_cast<const float4*>(dacc + (int64_t)i * Pp)[q];
    d.x += sign_from_bit(z, 0) * h.x; d.y += sign_from_bit(z, 1) * h.y;
    d.z += sign_from_bit(z, 2) * h.z; d.w += sign_from_bit(z, 3) * h.w;
    reinterpret_cast<float4*>(dacc + (int64_t)i * Pp)[q] = d;
  }
}

// skip: ranges (ascending, disjoint, bounds multiples of 4) that the sum leaves out
hipError_t launch_probe_sum(float* dacc, const float* hz, const uint32_t* zbits, int64_t Pp, int64_t z_stride, int k,
                            uint64_t active_mask, int first, const FusedRanges& skip, hipStream_t s) {
  KernelScope ks(KC_UPDATE, s);
  FusedRanges keep{};
  int64_t pos = 0, longest = 0;
  for (int r = 0; r <= skip.n; ++r) {
    const int64_t end = r < skip.n ? skip.begin[r] : Pp;
    if (end > pos) {
      // at most DW_MAX_LAYERS - 1 layers are fused (the output layer never is): the pieces between them fit
      if (keep.n == DW_MAX_LAYERS) return hipErrorInvalidValue;
      keep.begin[keep.n] = pos; keep.end[keep.n] = end;
      longest = end - pos > longest ? end - pos : longest;
      keep.n += 1;
    }
    if (r < skip.n) pos = skip.end[r];
  }
  if (keep.n == 0) return hipSuccess;
  int64_t nb = ((longest >> 2) + 255) / 256;
  if (nb > 16384) nb = 16384;
  hipLaunchKernelGGL(probe_sum_kernel, dim3((unsigned)nb, (unsigned)k, (unsigned)keep.n), dim3(256), 0, s, dacc, hz, zbits,
                     Pp, z_stride, active_mask, first, keep);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------------
// Small utilities: replicate the centre into all workers, zero fill, refresh the bf16 weight copy.
// ---------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void broadcast_kernel(float* theta, const float* centre, uint16_t* wb16,
                                                        int64_t Pp, int k) {
  const int64_t nq = Pp >> 2;
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < nq; q += (int64_t)gridDim.x * 256) {
    const float4 c = reinterpret_cast<const float4*>(centre)[q];
    ushort4 b;
    b.x = f32_to_bf16_rne(c.x); b.y = f32_to_bf16_rne(c.y); b.z = f32_to_bf16_rne(c.z); b.w = f32_to_bf16_rne(c.w);
    for (int i = 0; i < k; ++i) {
      reinterpret_cast<float4*>(theta + (int64_t)i * Pp)[q] = c;
      if (wb16) reinterpret_cast<ushort4*>(wb16 + (int64_t)i * Pp)[q] = b;
    }
  }
}

hipError_t launch_broadcast(float* theta, const float* centre, uint16_t* wb16, int64_t Pp, int k, hipStream_t s) {
  const int64_t nq = Pp >> 2;
  int64_t nb = (nq + 255) / 256;
  if (nb > 65536) nb = 65536;
  hipLaunchKernelGGL(broadcast_kernel, dim3((unsigned)nb), dim3(256), 0, s, theta, centre, wb16, Pp, k);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint4* p, int64_t n16) {
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < n16; q += (int64_t)gridDim.x * 256)
    p[q] = make_uint4(0, 0, 0, 0);
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {   // bytes must be a multiple of 16
  const int64_t n16 = (int64_t)(bytes / 16);
  if (n16 == 0) return hipSuccess;
  int64_t nb = (n16 + 255) / 256;
  if (nb > 65536) nb = 65536;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)nb), dim3(256), 0, s, reinterpret_cast<uint4*>(p), n16);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void refresh_bf16_kernel(const float* theta, uint16_t* wb16, int64_t nq) {
  for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < nq; q += (int64_t)gridDim.x * 256) {
    const float4 c = reinterpret_cast<const float4*>(theta)[q];
    ushort4 b;
    b.x = f32_to_bf16_rne(c.x); b.y = f32_to_bf16_rne(c.y); b.z = f32_to_bf16_rne(c.z); b.w = f32_to_bf16_rne(c.w);
    reinterpret_cast<ushort4*>(wb16)[q] = b;
  }
}

hipError_t launch_refresh_bf16(const float* theta, uint16_t* wb16, int64_t n, hipStream_t s) {
  const int64_t nq = n >> 2;
  int64_t nb = (nq + 255) / 256;
  if (nb > 65536) nb = 65536;
  if (nb == 0) return hipSuccess;
  hipLaunchKernelGGL(refresh_bf16_kernel, dim3((unsigned)nb), dim3(256), 0, s, theta, wb16, nq);
  return hipGetLastError();
}

// Column sums of a bf16 matrix [B][n] per worker.  Block: 32 units of 8 columns x 8 row groups; a thread adds the rows
// r = group, group + 8, ... of its 8 columns, the groups are then added in order through LDS.
__global__ __launch_bounds__(256) void col_sums_bf16_kernel(const uint16_t* src, int B, int n, float* out, int64_t out_wstride,
                                                            uint64_t active_mask) {
  const int worker = blockIdx.y;
  if (!((active_mask >> worker) & 1ull)) return;
  const int unit = threadIdx.x & 31, group = threadIdx.x >> 5;
  const int col = (blockIdx.x * 32 + unit) * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (col < n) {
    const uint16_t* p = src + (int64_t)worker * B * n + col;
#pragma unroll 4
    for (int r = group; r < B; r += 8) {
      const uint4 u = *reinterpret_cast<const uint4*>(p + (int64_t)r * n);
      const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        acc[2 * q] += __uint_as_float(w[q] << 16);
        acc[2 * q + 1] += __uint_as_float(w[q] & 0xFFFF0000u);
      }
    }
  }
  __shared__ float part[8][32][9];
#pragma unroll
  for (int q = 0; q < 8; ++q) part[group][unit][q] = acc[q];
  __syncthreads();
  const int c = threadIdx.x;                                  // one thread per column of the block's 256
  if (blockIdx.x * 256 + c < n) {
    float t = 0.f;
#pragma unroll
    for (int gq = 0; gq < 8; ++gq) t += part[gq][c >> 3][c & 7];
    out[(int64_t)worker * out_wstride + blockIdx.x * 256 + c] = t;
  }
}

hipError_t launch_col_sums_bf16(const uint16_t* src, int B, int n, float* out, int64_t out_wstride, int k,
                                uint64_t active_mask, hipStream_t s) {
  hipLaunchKernelGGL(col_sums_bf16_kernel, dim3((unsigned)((n + 255) / 256), (unsigned)k), dim3(256), 0, s, src, B, n, out,
                     out_wstride, active_mask);
  return hipGetLastError();
}

}  // namespace dw
