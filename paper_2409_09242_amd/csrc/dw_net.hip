// Forward / backward pass of the MLP classifier and of its directional derivative along z.
//
// Per worker and minibatch (Section II eq.(2), Section III-B eq.(6)): a_0 = x, s_l = a_{l-1} W_l^T + b_l,
// a_l = ReLU(s_l), p = softmax(s_L), loss = -mean log p[y]; backward d_L = (p - onehot)/B,
// gW_l = d_l^T a_{l-1}, gb_l = sum_n d_l, d_{l-1} = (d_l W_l) * [s_{l-1} > 0].
// The Hessian-vector product of the Hutchinson estimate (Section IV-B) is the derivative of that gradient
// along z = (V_l, c_l): Ra_0 = 0, Rs_l = Ra_{l-1} W_l^T + a_{l-1} V_l^T + c_l, Ra_l = [s_l > 0] Rs_l,
// Rd_L = p * (Rs_L - <p, Rs_L>)/B, HzW_l = Rd_l^T a_{l-1} + d_l^T Ra_{l-1}, Hzb_l = sum_n Rd_l,
// Rd_{l-1} = (Rd_l W_l + d_l V_l) * [s_{l-1} > 0].
// Every matrix product above runs in the dual GEMM kernels; this file holds the softmax head and the
// order of the launches.
#include "dw_internal.h"
#include "dw_device_util.h"
#include "dw_head_math.h"

namespace dw {

// one block per worker; thread n handles sample n (looping when B > blockDim)
__global__ __launch_bounds__(256) void head_kernel(HeadArgs a) {
  const int i = blockIdx.x;
  if (!((a.active_mask >> i) & 1ull)) return;
  const float* S = a.s + (int64_t)i * a.B * a.ld;
  const float* RS = a.Rs + (int64_t)i * a.B * a.ld;
  float* D = a.delta + (int64_t)i * a.B * a.ld;
  float* RD = a.Rdelta + (int64_t)i * a.B * a.ld;
  const int32_t* Y = a.y + (int64_t)i * a.B;
  const float invB = 1.0f / (float)a.B;
  float loss = 0.f;
  for (int n = threadIdx.x; n < a.B; n += blockDim.x) {
    float s[DW_MAX_CLASSES], rs[DW_MAX_CLASSES], d[DW_MAX_CLASSES], rd[DW_MAX_CLASSES];
#pragma unroll
    for (int c = 0; c < DW_MAX_CLASSES; ++c) {
      s[c] = c < a.C ? S[(int64_t)n * a.ld + c] : 0.f;
      rs[c] = c < a.C ? RS[(int64_t)n * a.ld + c] : 0.f;
    }
    loss += head_row(s, rs, Y[n], a.C, invB, d, rd);
#pragma unroll
    for (int c = 0; c < DW_MAX_CLASSES; ++c) {
      if (c < a.ld) {
        D[(int64_t)n * a.ld + c] = d[c];
        RD[(int64_t)n * a.ld + c] = rd[c];
        if (a.delta_b16) {
          a.delta_b16[((int64_t)i * a.B + n) * a.ld + c] = f32_to_bf16_rne(d[c]);
          a.Rdelta_b16[((int64_t)i * a.B + n) * a.ld + c] = f32_to_bf16_rne(rd[c]);
        }
      }
    }
  }
  __shared__ float red[256];
  red[threadIdx.x] = loss;
  __syncthreads();
  for (int st = 128; st >= 1; st >>= 1) {
    if ((int)threadIdx.x < st) red[threadIdx.x] += red[threadIdx.x + st];
    __syncthreads();
  }
  if (threadIdx.x == 0 && a.loss) a.loss[i] = red[0] * invB;
}

hipError_t launch_head(const HeadArgs& a, hipStream_t s) {
  KernelScope ks(KC_HEAD, s);
  hipLaunchKernelGGL(head_kernel, dim3(a.k), dim3(256), 0, s, a);
  return hipGetLastError();
}

int run_network(const dw_config& cfg, char* ws, const Layout& lay, const void* d_x, const int32_t* d_y,
                const uint32_t* zbits, int64_t z_stride, uint64_t active, float* d_loss, const UpdateArgs* fuse,
                bool fuse_dist, hipStream_t s, const void* in_ract, void* d_in, void* rd_in, bool r_only,
                int pair_phase, const SideStream* side) {
  const bool b16 = cfg.dtype == DW_BF16;
  const int L = cfg.n_layers, k = cfg.k, B = cfg.batch;
  const int HL = DW_MAX_CLASSES;                     // row stride of the output-layer buffers
  float* theta = reinterpret_cast<float*>(ws + lay.theta);
  float* g = reinterpret_cast<float*>(ws + lay.g);
  float* hz = reinterpret_cast<float*>(ws + lay.hz);
  auto act = [&](int l) -> const void* { return l == 0 ? d_x : (const void*)(ws + lay.act[l]); };
  // R-quantities of the hidden layers: the earlier of two probes taken together keeps its own (see Layout::pair)
  const bool keep = pair_phase == 1;
  auto ract_buf = [&](int l) -> void* { return ws + (keep ? lay.ract_p[l] : lay.ract[l]); };
  auto rdelta_buf = [&](int l) -> void* { return ws + (keep ? lay.rdelta_p[l] : lay.rdelta[l]); };
  auto ract = [&](int l) -> const void* { return l == 0 ? in_ract : (const void*)ract_buf(l); };
  auto act_stride = [&](int l) -> int64_t { return (int64_t)B * cfg.dims[l]; };
  // weights as the GEMMs read them: fp32 master copy, or its bf16 rounding kept by the update and the pull
  auto weights = [&](int l) -> const void* {
    return b16 ? (const void*)(reinterpret_cast<uint16_t*>(ws + lay.wb16) + lay.woff[l - 1])
               : (const void*)(theta + lay.woff[l - 1]);
  };
  auto gemm_on = [&](const GemmArgs& a, hipStream_t st) { return b16 ? launch_gemm_bf16(a, st) : launch_gemm_f32(a, st); };
  auto gemm = [&](const GemmArgs& a) { return gemm_on(a, s); };
  hipError_t e;

  // layers whose data gradient reads the sign bits of V_l column by column get a transposed copy of those bits
  // (when the caller's z allows 16-byte accesses; otherwise those layers take the general kernel)
  uint32_t* zt = nullptr;
  const bool z_aligned = z_stride % 4 == 0 && (reinterpret_cast<uintptr_t>(zbits) & 15u) == 0;
  for (int l = 2; l <= L && b16 && z_aligned; ++l) {
    if (!lay.zt_layer[l - 1]) continue;
    zt = reinterpret_cast<uint32_t*>(ws + lay.zbits_t);
    if ((e = launch_transpose_bits(zbits, z_stride, zt, lay.z_stride, lay.woff[l - 1], cfg.dims[l], cfg.dims[l - 1], k,
                                   active, s)) != hipSuccess)
      return DW_ERR_HIP;
  }

  HeadArgs hd{};
  hd.s = reinterpret_cast<const float*>(ws + lay.sL); hd.Rs = reinterpret_cast<const float*>(ws + lay.rsL);
  hd.delta = reinterpret_cast<float*>(ws + lay.dL); hd.Rdelta = reinterpret_cast<float*>(ws + lay.rdL);
  hd.delta_b16 = b16 ? reinterpret_cast<uint16_t*>(ws + lay.dL16) : nullptr;
  hd.Rdelta_b16 = b16 ? reinterpret_cast<uint16_t*>(ws + lay.rdL16) : nullptr;
  hd.y = d_y; hd.loss = d_loss; hd.B = B; hd.C = cfg.dims[L]; hd.ld = HL; hd.k = k; hd.active_mask = active;
  bool head_done = false;

  // forward with R-forward
  for (int l = 1; l <= L; ++l) {
    GemmArgs a{};
    a.X = act(l - 1); a.RX = ract(l - 1); a.x_wstride = act_stride(l - 1); a.x_kcontig = 1; a.ldx = cfg.dims[l - 1];
    a.Y = weights(l); a.RY = nullptr; a.ry_bits = 1; a.y_wstride = lay.Pp; a.y_kcontig = 1;
    a.ldy = cfg.dims[l - 1];
    a.zbits = zbits; a.z_stride = z_stride; a.z_off = lay.woff[l - 1]; a.zb_off = lay.boff[l - 1];
    a.M = B; a.N = cfg.dims[l]; a.K = cfg.dims[l - 1];
    a.bias = theta + lay.boff[l - 1]; a.bias_wstride = lay.Pp;
    if (l < L) {
      a.C = ws + lay.act[l]; a.RC = ract_buf(l); a.ldc = cfg.dims[l]; a.c_wstride = act_stride(l);
      a.epi = EPI_RELU; a.r_only = r_only ? 1 : 0;
    } else {
      a.C = ws + lay.sL; a.RC = ws + lay.rsL; a.ldc = HL; a.c_wstride = (int64_t)B * HL;
      a.epi = EPI_LINEAR;
    }
    a.k = k; a.active_mask = active;
    if (!b16 && l == L && out_head_f32_ok(a)) {
      // fp32: the output layer's product and the softmax head in one kernel (the logits buffer serves as its
      // scratch for the per-block losses)
      if ((e = launch_out_head_f32(a, hd, reinterpret_cast<float*>(ws + lay.sL), s)) != hipSuccess) return DW_ERR_HIP;
      head_done = true;
      break;
    }
    if (!b16 && lay.fwdSplit[l - 1] > 1) {             // long contraction, few output tiles
      a.ksplit = lay.fwdSplit[l - 1]; a.part = reinterpret_cast<float*>(ws + lay.cPart);
      a.part_stride = (int64_t)B * a.ldc; a.part_b = nullptr;
    }
    if ((e = gemm(a)) != hipSuccess) return DW_ERR_HIP;
  }

  // softmax cross-entropy head
  if (!head_done) {
    if ((e = launch_head(hd, s)) != hipSuccess) return DW_ERR_HIP;
  }

  // backward with R-backward.  d_l, Rd_l of layer l (its own buffer per layer, so both phases can read them):
  auto delta_of = [&](int l, const void*& dl, const void*& rdl, int& ldd, int64_t& dstride) {
    if (l == L) {
      dl = ws + (b16 ? lay.dL16 : lay.dL); rdl = ws + (b16 ? lay.rdL16 : lay.rdL); ldd = HL; dstride = (int64_t)B * HL;
    } else {
      dl = ws + lay.delta[l]; rdl = rdelta_buf(l); ldd = cfg.dims[l]; dstride = act_stride(l);
    }
  };
  auto weight_gradient = [&](int l, hipStream_t st) -> hipError_t {   // and its R-companion: contraction over the minibatch
    const void* dl; const void* rdl; int ldd; int64_t dstride;
    delta_of(l, dl, rdl, ldd, dstride);
    GemmArgs a{};
    a.X = dl; a.RX = rdl; a.x_wstride = dstride; a.x_kcontig = 0; a.ldx = ldd;
    a.Y = act(l - 1); a.RY = ract(l - 1); a.ry_bits = 0; a.y_wstride = act_stride(l - 1); a.y_kcontig = 0;
    a.ldy = cfg.dims[l - 1];
    a.zbits = zbits; a.z_stride = z_stride;
    a.M = cfg.dims[l]; a.N = cfg.dims[l - 1]; a.K = B;
    a.C = g + lay.woff[l - 1]; a.RC = hz + lay.woff[l - 1]; a.ldc = cfg.dims[l - 1]; a.c_wstride = lay.Pp;
    a.gb = g + lay.boff[l - 1]; a.hzb = hz + lay.boff[l - 1];
    a.epi = EPI_WGRAD; a.k = k; a.active_mask = active;
    if (fuse != nullptr && lay.fuse_base[l - 1] >= 0 && keep) {
      // left to the later probe's launch; the bias part of this probe's Hz is the column sum of Rd_l
      KernelScope ks(KC_GEMM_WGRAD, st);
      return launch_col_sums_bf16(reinterpret_cast<const uint16_t*>(rdl), B, cfg.dims[l], hz + lay.boff[l - 1], lay.Pp, k,
                                  active, st);
    }
    if (fuse != nullptr && lay.fuse_base[l - 1] >= 0) {
      // the kernel applies this step's update to W_l instead of storing gW_l and HzW_l
      const int64_t wo = lay.woff[l - 1];
      a.z_off = wo;
      a.fu.on = 1;
      a.fu.dist = fuse_dist ? 1 : 0;
      a.fu.theta = fuse->theta + wo; a.fu.m = fuse->m + wo; a.fu.v = fuse->v + wo;
      a.fu.centre = fuse->centre + wo; a.fu.wb16 = fuse->wb16 ? fuse->wb16 + wo : nullptr;
      a.fu.partials = reinterpret_cast<double*>(ws + lay.partials_f);
      a.fu.part_stride = lay.n_fuse_slots; a.fu.part_base = lay.fuse_base[l - 1];
      a.fu.avg_block = fuse->avg_block;
      a.fu.lr = fuse->lr; a.fu.beta1 = fuse->beta1; a.fu.beta2 = fuse->beta2; a.fu.eps = fuse->eps; a.fu.hpow = fuse->hpow;
      a.fu.sc = fuse->sc;
      a.fu.probe_mode = fuse->probe_mode; a.fu.first = fuse->probe_first;
      a.fu.dacc = fuse->dacc ? fuse->dacc + wo : nullptr; a.fu.d_scale = fuse->d_scale;
      if (pair_phase == 2) {                          // (a fused layer is a hidden layer: its Rd_l has a kept copy)
        a.RXp = ws + lay.rdelta_p[l]; a.RYp = l == 1 ? nullptr : (const void*)(ws + lay.ract_p[l - 1]);
        a.zbits_p = reinterpret_cast<const uint32_t*>(ws + lay.zbits_p);
      }
    }
    return gemm_on(a, st);
  };
  // A small model without fused layers: the weight gradient of layer l only needs d_l, so those of the layers above
  // the first go to the side stream as soon as d_l is there and run beside the data gradients further down.
  const bool overlap = side != nullptr && lay.overlap_wgrad && fuse == nullptr && d_in == nullptr && L >= 2;
  auto fork_wgrad = [&](int l) -> hipError_t {        // d_l, Rd_l were just enqueued on s
    if ((e = hipEventRecord(side->fork[l], s)) != hipSuccess) return e;
    if ((e = hipStreamWaitEvent(side->s, side->fork[l], 0)) != hipSuccess) return e;
    return weight_gradient(l, side->s);
  };
  if (overlap && fork_wgrad(L) != hipSuccess) return DW_ERR_HIP;
  // The data gradients, output layer first.  A fused weight gradient overwrites W_l, which the data gradient
  // through W_l reads, so all data gradients are launched before the weight gradients.
  // (down to the first layer only when the caller wants the gradient with respect to the input)
  for (int l = L; l >= (d_in ? 1 : 2); --l) {
    const void* dl; const void* rdl; int ldd; int64_t dstride;
    delta_of(l, dl, rdl, ldd, dstride);
    GemmArgs a{};                                     // through W_l, masked by the ReLU of layer l-1
    a.X = dl; a.RX = rdl; a.x_wstride = dstride; a.x_kcontig = 1; a.ldx = ldd;
    a.Y = weights(l); a.RY = nullptr; a.ry_bits = 1; a.y_wstride = lay.Pp; a.y_kcontig = 0;
    a.ldy = cfg.dims[l - 1];
    a.zbits = zbits; a.z_stride = z_stride; a.z_off = lay.woff[l - 1];
    a.zbits_t = lay.zt_layer[l - 1] ? zt : nullptr; a.zt_stride = lay.z_stride;
    a.M = B; a.N = cfg.dims[l - 1]; a.K = cfg.dims[l];
    a.C = l == 1 ? d_in : (void*)(ws + lay.delta[l - 1]); a.RC = l == 1 ? rd_in : rdelta_buf(l - 1);
    a.ldc = cfg.dims[l - 1];
    a.c_wstride = act_stride(l - 1);
    a.mask_src = act(l - 1); a.ld_mask = cfg.dims[l - 1]; a.mask_wstride = act_stride(l - 1);
    a.epi = EPI_MASK; a.k = k; a.active_mask = active; a.r_only = (r_only && l > 1) ? 1 : 0;
    if (!b16 && l > 1 && lay.dgSplit[l - 1] > 1) {      // long contraction, few output tiles
      a.ksplit = lay.dgSplit[l - 1]; a.part = reinterpret_cast<float*>(ws + lay.cPart);
      a.part_stride = (int64_t)B * a.ldc; a.part_b = nullptr;
    }
    if ((e = gemm(a)) != hipSuccess) return DW_ERR_HIP;
    if (overlap && l - 1 >= 2 && fork_wgrad(l - 1) != hipSuccess) return DW_ERR_HIP;
  }
  // weight gradients (with the side stream: only the first layer's is left; then the caller's stream waits for the others)
  for (int l = overlap ? 1 : L; l >= 1; --l)
    if ((e = weight_gradient(l, s)) != hipSuccess) return DW_ERR_HIP;
  if (overlap) {
    if ((e = hipEventRecord(side->join, side->s)) != hipSuccess) return DW_ERR_HIP;
    if ((e = hipStreamWaitEvent(s, side->join, 0)) != hipSuccess) return DW_ERR_HIP;
  }
  return DW_OK;
}

}  // namespace dw
