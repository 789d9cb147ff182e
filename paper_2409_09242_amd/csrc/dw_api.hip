// Host side of libdw: configuration checks, workspace carving, per-call bookkeeping and the order in
// which the kernels of one worker step / one communication round are enqueued.  Nothing here computes
// any part of the method on the host except the scalars 1 - beta^t (Section IV-B bias correction) and
// the keys of the Rademacher stream.
#include <climits>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "dw_internal.h"

using namespace dw;

namespace {

thread_local int g_last_hip = 0;

inline int hip_fail(hipError_t e) {
  g_last_hip = (int)e;
  return DW_ERR_HIP;
}
#define DW_HIP(expr)                                   \
  do {                                                 \
    hipError_t e__ = (expr);                           \
    if (e__ != hipSuccess) return hip_fail(e__);       \
  } while (0)

}  // namespace

int dw::note_hip_error(hipError_t e) { return hip_fail(e); }

namespace {

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
inline bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }


int validate(const dw_config* c, Layout* lay) {
  if (!c) return DW_ERR_NULL;
  if (c->k < 1 || c->k > DW_MAX_K) return DW_ERR_CONFIG;
  if (c->dtype != DW_F32 && c->dtype != DW_BF16) return DW_ERR_CONFIG;
  if (c->fuse_update != 0 && c->fuse_update != 1) return DW_ERR_CONFIG;
  if (c->n_samples < 0 || c->n_samples > DW_MAX_SAMPLES) return DW_ERR_CONFIG;
  if (c->optimizer != DW_OPT_ADAHESSIAN && c->optimizer != DW_OPT_SGD && c->optimizer != DW_OPT_MOMENTUM)
    return DW_ERR_CONFIG;
  if (c->optimizer != DW_OPT_ADAHESSIAN && (c->n_samples > 1 || c->fuse_update != 0)) return DW_ERR_CONFIG;
  if (c->optimizer == DW_OPT_MOMENTUM && !(c->momentum >= 0.f && c->momentum < 1.f)) return DW_ERR_HYPER;
  if (c->n_layers < 0 || c->n_layers > DW_MAX_LAYERS) return DW_ERR_CONFIG;
  const int L = c->n_layers;
  const int align = c->dtype == DW_BF16 ? 8 : 4;
  int64_t P = 0;
  if (L == 0) {
    if (c->n_conv != 0) return DW_ERR_CONFIG;
    if (c->n_params < 4 || c->n_params % 4 != 0) return DW_ERR_CONFIG;
    P = c->n_params;
  } else {
    if (c->batch < 1 || c->batch > (1 << 20)) return DW_ERR_CONFIG;
    for (int l = 0; l <= L; ++l)
      if (c->dims[l] < 1 || c->dims[l] > (1 << 20)) return DW_ERR_CONFIG;
    for (int l = 0; l < L; ++l)
      if (c->dims[l] % align != 0) return DW_ERR_CONFIG;
    if (c->dims[L] > DW_MAX_CLASSES) return DW_ERR_CONFIG;
    const int nc = c->n_conv;
    if (nc < 0 || nc > DW_MAX_CONV) return DW_ERR_CONFIG;
    lay->n_conv = nc;
    if (nc > 0) {
      // convolutional front end: fp32, no fusion; maps shrink by 2 per convolution, the last is pooled 2x2
      if (c->dtype != DW_F32 || c->fuse_update != 0) return DW_ERR_CONFIG;
      if (c->conv_avg != 0 && c->conv_avg != 1) return DW_ERR_CONFIG;
      if (c->img_h < 3 || c->img_w < 3 || c->img_c < 1 || c->img_h > 4096 || c->img_w > 4096 || c->img_c > 1024)
        return DW_ERR_CONFIG;
      lay->cH[0] = c->img_h; lay->cW[0] = c->img_w; lay->cC[0] = c->img_c;
      for (int j = 0; j < nc; ++j) {
        const int co = c->conv_c[j];
        if (co < 4 || co % 4 != 0 || co > 1024) return DW_ERR_CONFIG;
        lay->cH[j + 1] = lay->cH[j] - 2; lay->cW[j + 1] = lay->cW[j] - 2; lay->cC[j + 1] = co;
        if (lay->cH[j + 1] < 1 || lay->cW[j + 1] < 1) return DW_ERR_CONFIG;
        if ((int64_t)c->batch * lay->cH[j + 1] * lay->cW[j + 1] > (int64_t)1 << 30) return DW_ERR_CONFIG;
        lay->cK[j] = (int)round_up(9 * lay->cC[j], 4);
        lay->cwoff[j] = P; P += (int64_t)co * lay->cK[j];
        lay->cboff[j] = P; P += co;
      }
      if (lay->cH[nc] % 2 != 0 || lay->cW[nc] % 2 != 0) return DW_ERR_CONFIG;
      if ((int64_t)c->dims[0] != (int64_t)(lay->cH[nc] / 2) * (lay->cW[nc] / 2) * lay->cC[nc]) return DW_ERR_CONFIG;
    }
    for (int l = 1; l <= L; ++l) {
      lay->woff[l - 1] = P;
      P += (int64_t)c->dims[l] * c->dims[l - 1];
      lay->boff[l - 1] = P;
      P += c->dims[l];
    }
    if (c->n_params != 0 && c->n_params != P) return DW_ERR_CONFIG;
  }
  // hyper-parameters
  if (!(c->lr > 0.f) || !(c->beta1 >= 0.f && c->beta1 < 1.f) || !(c->beta2 >= 0.f && c->beta2 < 1.f) ||
      !(c->eps > 0.f) || !(c->hpow >= 0.f && c->hpow <= 2.f))
    return DW_ERR_HYPER;
  if (!is_pow2(c->avg_block) || c->avg_block > 256) return DW_ERR_HYPER;
  if (c->n_layers > 0 && c->n_conv > 0 && c->avg_block != 1) return DW_ERR_HYPER;   // linear layers are not averaged there
  if (L == 0) {
    if (P % c->avg_block != 0) return DW_ERR_HYPER;
  } else {
    for (int l = 0; l < L; ++l)
      if (c->dims[l] % c->avg_block != 0) return DW_ERR_HYPER;
  }
  if (!(c->alpha > 0.f && c->alpha <= 1.f) || !(c->kappa < 0.f)) return DW_ERR_HYPER;
  if (c->p < 1 || c->p > DW_MAX_P) return DW_ERR_HYPER;
  double csum = 0.0;
  for (int j = 0; j < c->p; ++j) {
    if (!(c->c[j] >= 0.f)) return DW_ERR_HYPER;
    csum += c->c[j];
  }
  if (std::fabs(csum - 1.0) > 1e-5) return DW_ERR_HYPER;

  // workspace
  const int k = c->k;
  lay->P = P;
  lay->Pp = round_up(P, 64);
  lay->z_stride = round_up(2 * ((P + 63) / 64), 64);
  lay->n_upd_blocks = (lay->Pp + kUpdChunk - 1) / kUpdChunk;
  size_t pos = 0;
  auto take = [&](size_t bytes) { size_t at = pos; pos += (size_t)round_up((int64_t)bytes, 256); return at; };
  const size_t vec = (size_t)k * lay->Pp * sizeof(float);
  lay->theta = take(vec); lay->m = take(vec); lay->v = take(vec);
  lay->centre = take((size_t)lay->Pp * sizeof(float));
  if (L > 0) { lay->g = take(vec); lay->hz = take(vec); }
  if (L > 0 && c->n_samples > 1) lay->dacc = take(vec);
  if (c->dtype == DW_BF16) lay->wb16 = take((size_t)k * lay->Pp * 2);
  lay->zbits = take((size_t)k * lay->z_stride * 4);
  if (c->dtype == DW_BF16) {
    bool any = false;
    for (int l = 2; l <= L; ++l) {
      lay->zt_layer[l - 1] = gemm_bf16_dgrad_dma_shape_ok(c->batch, c->dims[l], c->dims[l - 1], k, lay->woff[l - 1]);
      any = any || lay->zt_layer[l - 1];
    }
    if (any) lay->zbits_t = take((size_t)k * lay->z_stride * 4);
  }
  if (L > 0) {
    const size_t es = c->dtype == DW_BF16 ? 2 : 4;
    const int64_t B = c->batch;
    int dmax = 4;
    for (int l = 1; l < L; ++l) {
      lay->act[l] = take((size_t)k * B * c->dims[l] * es);
      lay->ract[l] = take((size_t)k * B * c->dims[l] * es);
      if (c->dims[l] > dmax) dmax = c->dims[l];
    }
    for (int l = 1; l < L; ++l) {
      lay->delta[l] = take((size_t)k * B * c->dims[l] * es);
      lay->rdelta[l] = take((size_t)k * B * c->dims[l] * es);
    }
    const size_t head = (size_t)k * B * DW_MAX_CLASSES * sizeof(float);
    lay->sL = take(head); lay->rsL = take(head); lay->dL = take(head); lay->rdL = take(head);
    if (c->dtype == DW_BF16) { lay->dL16 = take(head / 2); lay->rdL16 = take(head / 2); }
  }
  size_t part = 0, part_b = 0;                       // scratch of products whose contraction is cut into slices
  if (L > 0 && lay->n_conv > 0) {
    const int64_t B = c->batch;
    for (int j = 0; j < lay->n_conv; ++j) {
      const size_t M = (size_t)B * lay->cH[j + 1] * lay->cW[j + 1];
      if (j == 0) lay->cP[j] = take((size_t)k * M * lay->cK[j] * 4);   // (the later convolutions read the map itself)
      const size_t out = (size_t)k * M * lay->cC[j + 1] * 4;
      lay->cA[j] = take(out); lay->cRA[j] = take(out); lay->cD[j] = take(out); lay->cRD[j] = take(out);
    }
    // weight gradients of the convolutions contract over all output positions of the minibatch and have few output
    // tiles: cut the contraction so that about 1024 blocks exist, slices of at least 512 positions
    for (int j = 0; j < lay->n_conv; ++j) {
      const int64_t M = B * lay->cH[j + 1] * lay->cW[j + 1];
      const int64_t blocks = (int64_t)((lay->cC[j + 1] + 63) / 64) * ((lay->cK[j] + 63) / 64) * k;
      int64_t split = 1024 / blocks;
      if (split > M / 512) split = M / 512;
      if (split > 64) split = 64;
      lay->cSplit[j] = (int)(split < 1 ? 1 : split);
      if (lay->cSplit[j] > 1) {
        const size_t need = (size_t)lay->cSplit[j] * k * 2 * lay->cC[j + 1] * lay->cK[j] * 4;
        const size_t need_b = (size_t)lay->cSplit[j] * k * 2 * lay->cC[j + 1] * 4;
        part = need > part ? need : part; part_b = need_b > part_b ? need_b : part_b;
      }
    }
    const size_t flat = (size_t)k * B * c->dims[0];
    lay->pool = take(flat * 4); lay->rpool = take(flat * 4); lay->dpool = take(flat * 4); lay->rdpool = take(flat * 4);
    lay->pidx = take(flat);
  }
  if (L > 0 && c->dtype == DW_F32) {
    // fp32 forward products with a long contraction and a handful of output tiles (the output layer; the first linear
    // layer behind a convolutional front end): same cut, slices of at least 64 (measured: 256 -> 64 takes 12 % off
    // the step of the 784-512-512-10 configuration, nothing off the others)
    const int64_t B = c->batch;
    for (int l = 1; l <= L; ++l) {
      const int64_t n = c->dims[l], kk = c->dims[l - 1];
      const int64_t tiles = n <= 32 ? (B + 127) / 128 : B <= 32 ? (n + 127) / 128 : ((B + 63) / 64) * ((n + 63) / 64);
      int64_t split = tiles * k < 256 ? 1024 / (tiles * k) : 1;
      if (split > kk / 64) split = kk / 64;
      if (split > 64) split = 64;
      lay->fwdSplit[l - 1] = (int)(split < 1 ? 1 : split);
      if (lay->fwdSplit[l - 1] > 1) {
        const size_t need = (size_t)lay->fwdSplit[l - 1] * k * 2 * B * (l == L ? DW_MAX_CLASSES : n) * 4;
        part = need > part ? need : part;
      }
    }
    // and the data gradients through W_l (B x d_{l-1} outputs, contraction d_l) of the same kind
    for (int l = 2; l <= L; ++l) {
      const int64_t n = c->dims[l - 1], kk = c->dims[l];
      const int64_t tiles = n <= 32 ? (B + 127) / 128 : B <= 32 ? (n + 127) / 128 : ((B + 63) / 64) * ((n + 63) / 64);
      int64_t split = tiles * k < 256 ? 1024 / (tiles * k) : 1;
      if (split > kk / 64) split = kk / 64;
      if (split > 64) split = 64;
      lay->dgSplit[l - 1] = (int)(split < 1 ? 1 : split);
      if (lay->dgSplit[l - 1] > 1) {
        const size_t need = (size_t)lay->dgSplit[l - 1] * k * 2 * B * n * 4;
        part = need > part ? need : part;
      }
    }
  }
  if (part > 0) { lay->cPart = take(part); lay->cPartB = take(part_b > 0 ? part_b : 256); }
  lay->partials = take((size_t)k * lay->n_upd_blocks * sizeof(double));
  // layers whose weight-gradient kernel applies the update itself: one partial-sum slot per output tile
  lay->n_fuse_slots = 0;
  for (int l = 1; l <= L; ++l) {
    lay->fuse_base[l - 1] = -1;
    const bool b16 = c->dtype == DW_BF16;
    if (!c->fuse_update) continue;
    if (b16 ? gemm_bf16_wgrad_fusable(c->dims[l], c->dims[l - 1], k, c->avg_block, c->hpow, lay->woff[l - 1])
            : gemm_f32_wgrad_fusable(c->dims[l], c->dims[l - 1], k, c->avg_block, c->hpow, lay->woff[l - 1])) {
      lay->fuse_base[l - 1] = lay->n_fuse_slots;
      lay->n_fuse_slots += b16 ? gemm_bf16_wgrad_tiles(c->dims[l], c->dims[l - 1], c->n_samples)
                               : gemm_f32_wgrad_tiles(c->dims[l], c->dims[l - 1]);
    }
  }
  if (lay->n_fuse_slots > 0) lay->partials_f = take((size_t)k * lay->n_fuse_slots * sizeof(double));
  if (lay->n_fuse_slots > 0 && c->dtype == DW_BF16 && c->n_samples == 2) {
    lay->pair = true;
    lay->zbits_p = take((size_t)k * lay->z_stride * 4);
    for (int l = 1; l < L; ++l) {
      lay->ract_p[l] = take((size_t)k * c->batch * c->dims[l] * 2);
      lay->rdelta_p[l] = take((size_t)k * c->batch * c->dims[l] * 2);
    }
  }
  // small models without a convolutional front end or fused layers: weight gradients beside the data gradients
  if (L >= 2 && lay->n_conv == 0 && lay->n_fuse_slots == 0) {
    int64_t blocks = 0;                                   // 64 x 64 output tiles of all weight gradients
    for (int l = 1; l <= L; ++l) blocks += (int64_t)((c->dims[l] + 63) / 64) * ((c->dims[l - 1] + 63) / 64) * k;
    lay->overlap_wgrad = blocks < 4096 && !tiny_step_ok(*c, *lay);
  }
  lay->u_ring = take((size_t)k * (DW_MAX_P + 1) * sizeof(double));
  lay->score = take((size_t)k * 4 * sizeof(double));
  lay->omh1 = take((size_t)k * sizeof(float));
  lay->h2 = take((size_t)k * sizeof(float));
  lay->loss = take((size_t)k * sizeof(float));
  lay->total = pos;
  return DW_OK;
}

uint64_t mix64_host(uint64_t x) {
  x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
  x ^= x >> 27; x *= 0x94D049BB133111EBull;
  x ^= x >> 31;
  return x;
}

uint64_t mask_from(const uint8_t* h, int k) {
  uint64_t mk = 0;
  for (int i = 0; i < k; ++i)
    if (!h || h[i]) mk |= 1ull << i;
  return mk;
}

}  // namespace

struct dw_handle {
  dw_config cfg;
  Layout lay;
  char* ws;
  int64_t t[DW_MAX_K];      // local steps per worker
  int64_t calls;            // dw_worker_step / dw_update_only calls so far
  int64_t rounds;           // communication rounds so far
  bool norms_valid;         // the squared distances in `partials` match the current theta and centre
  int last_tau;             // communication period of the latest dw_elastic_sync call (1 before the first)
  Profiler* prof;           // non-null while per-kernel timing is enabled
  SideStream* side;         // non-null when lay.overlap_wgrad

  template <class T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

namespace {

// `fused_step`: the weight-gradient kernels of this step update the layers marked in the layout themselves
void fill_update_args(dw_handle* h, UpdateArgs& a, const float* g, const float* hz, int64_t g_stride,
                      const uint32_t* zbits, int64_t z_stride, uint64_t active, bool fused_step = false) {
  const dw_config& c = h->cfg;
  const Layout& L = h->lay;
  a.theta = h->at<float>(L.theta); a.m = h->at<float>(L.m); a.v = h->at<float>(L.v);
  a.g = g; a.hz = hz; a.centre = h->at<float>(L.centre);
  a.zbits = zbits;
  a.wb16 = c.dtype == DW_BF16 ? h->at<uint16_t>(L.wb16) : nullptr;
  a.partials = h->at<double>(L.partials);
  a.P = L.P; a.Pp = L.Pp; a.g_stride = g_stride; a.z_stride = z_stride;
  a.k = c.k; a.avg_block = c.avg_block;
  a.lr = c.lr; a.beta1 = c.beta1; a.beta2 = c.beta2; a.eps = c.eps; a.hpow = c.hpow;
  a.optimizer = c.optimizer; a.momentum = c.momentum;
  a.d_scale = 0.f;
  a.probe_mode = 0; a.probe_first = 0; a.dacc = nullptr;
  a.active_mask = active;
  a.bias.n = c.n_layers;
  for (int l = 0; l < c.n_layers; ++l) {
    a.bias.begin[l] = L.boff[l];
    a.bias.end[l] = L.boff[l] + c.dims[l + 1];
  }
  a.fused.n = 0;
  if (fused_step) {
    for (int l = 0; l < c.n_layers; ++l) {
      if (L.fuse_base[l] < 0) continue;
      a.fused.begin[a.fused.n] = L.woff[l];
      a.fused.end[a.fused.n] = L.woff[l] + (int64_t)c.dims[l + 1] * c.dims[l];
      a.fused.n += 1;
    }
  }
  for (int i = 0; i < DW_MAX_K; ++i) {
    a.sc.inv_bc1[i] = 1.f; a.sc.inv_bc2[i] = 1.f;
    if (i < c.k && ((active >> i) & 1ull)) {
      const double t = (double)h->t[i];      // already incremented for this step
      a.sc.inv_bc1[i] = (float)(1.0 / (1.0 - std::pow((double)c.beta1, t)));
      a.sc.inv_bc2[i] = (float)(1.0 / (1.0 - std::pow((double)c.beta2, t)));
    }
  }
}

inline int probes(const dw_handle* h) { return h->cfg.n_samples > 1 ? h->cfg.n_samples : 1; }

// draw probe `sample` of the active workers' next step (step counts before the increment): stream position
// t_i * n_samples + sample, which for one probe per step is t_i
int draw_z(dw_handle* h, uint64_t active, hipStream_t s, int sample = 0, uint32_t* dst = nullptr) {
  uint64_t keys[DW_MAX_K];
  const uint64_t G = 0x9E3779B97F4A7C15ull;
  for (int i = 0; i < h->cfg.k; ++i) {
    const uint64_t k1 = mix64_host(h->cfg.seed + G * (uint64_t)(i + 1));
    keys[i] = mix64_host(k1 + G * (uint64_t)(h->t[i] * probes(h) + sample + 1));
  }
  DW_HIP(launch_rademacher(dst ? dst : h->at<uint32_t>(h->lay.zbits), h->lay.z_stride, (h->lay.P + 63) / 64, keys,
                           h->cfg.k, active, s));
  return DW_OK;
}

// the partial sums of fused weight-gradient kernels describe the step that wrote them: clear them before any
// other kernel measures the distances (or before the next fused step writes the active workers' slots)
int clear_fused_partials(dw_handle* h, hipStream_t s) {
  if (h->lay.n_fuse_slots > 0)
    DW_HIP(launch_fill_zero(h->at<char>(h->lay.partials_f),
                            (size_t)round_up((int64_t)h->cfg.k * h->lay.n_fuse_slots * (int64_t)sizeof(double), 256), s));
  return DW_OK;
}

int run_update(dw_handle* h, const float* g, const float* hz, int64_t g_stride, const uint32_t* d_zbits,
               uint64_t active, hipStream_t s) {
  const uint32_t* zb = d_zbits ? d_zbits : h->at<uint32_t>(h->lay.zbits);
  const int64_t zs = d_zbits ? 2 * ((h->lay.P + 63) / 64) : h->lay.z_stride;
  for (int i = 0; i < h->cfg.k; ++i)
    if ((active >> i) & 1ull) h->t[i] += 1;
  UpdateArgs a;
  fill_update_args(h, a, g, hz, g_stride, zb, zs, active);
  { const int st = clear_fused_partials(h, s); if (st != DW_OK) return st; }
  DW_HIP(launch_update(a, (int)h->lay.n_upd_blocks, s));
  h->norms_valid = true;
  h->calls += 1;
  return DW_OK;
}

// network and update of one step; with fused layers the step counts and the update's scalars are needed by the
// weight-gradient kernels, so they are fixed before the network runs
int run_step(dw_handle* h, const void* d_x, const int32_t* d_y, const uint32_t* d_zbits, uint64_t active,
             float* loss, hipStream_t s) {
  const uint32_t* zb = d_zbits ? d_zbits : h->at<uint32_t>(h->lay.zbits);
  const int64_t zs = d_zbits ? 2 * ((h->lay.P + 63) / 64) : h->lay.z_stride;
  if (probes(h) > 1) {
    // n probes of the same minibatch: the network runs once per probe (loss and g come out the same each time),
    // z_j*Hz_j is summed, and the update takes D = sum / n.  Fused layers keep their part of the sum in the
    // weight-gradient kernel and apply the update in the last probe's; the rest goes through the sum kernel.
    // Two probes with fused bf16 layers (lay.pair): the earlier probe's pass leaves the fused weight gradients out
    // and keeps its z, Ra_l, Rd_l; the later probe's kernels multiply for both and need no sum in memory.
    const int n = probes(h);
    const bool fused = h->lay.n_fuse_slots > 0;
    const bool pair = h->lay.pair && !d_zbits;
    uint32_t* zb_p = pair ? h->at<uint32_t>(h->lay.zbits_p) : nullptr;
    float* dacc = h->at<float>(h->lay.dacc);
    int st = clear_fused_partials(h, s);
    if (st != DW_OK) return st;
    UpdateArgs a;
    for (int j = 0; j < n; ++j) {
      const bool last = j == n - 1;
      const uint32_t* zj = pair && !last ? zb_p : zb;      // this probe's sign bits
      st = draw_z(h, active, s, j, pair && !last ? zb_p : nullptr);
      if (st != DW_OK) return st;
      if (last)
        for (int i = 0; i < h->cfg.k; ++i)
          if ((active >> i) & 1ull) h->t[i] += 1;
      if (last || j == 0) fill_update_args(h, a, h->at<float>(h->lay.g), dacc, h->lay.Pp, zb, zs, active, fused);
      a.d_scale = 1.0f / (float)n;
      a.probe_mode = pair ? 3 : last ? 2 : 1; a.probe_first = j == 0 ? 1 : 0; a.dacc = dacc;
      // probes after the first find the activations and the plain data gradients of this minibatch in the workspace
      if (h->lay.n_conv > 0) {
        // the window mean is linear: taken per probe on z_j*Hz_j, it gives the window mean of their mean
        st = run_network_cnn(h->cfg, h->ws, h->lay, d_x, d_y, zb, zs, active, loss, s);
        if (st == DW_OK && h->cfg.conv_avg)
          DW_HIP(launch_conv_window_mean(h->at<float>(h->lay.hz), zb, h->lay.Pp, zs, h->lay, h->cfg.k, active, s));
      } else {
        st = run_network(h->cfg, h->ws, h->lay, d_x, d_y, zj, zs, active, loss, fused ? &a : nullptr, true, s, nullptr,
                         nullptr, nullptr, j > 0, pair ? j + 1 : 0, h->side);
      }
      if (st != DW_OK) return st;
      DW_HIP(launch_probe_sum(dacc, h->at<float>(h->lay.hz), zj, h->lay.Pp, zs, h->cfg.k, active, j == 0 ? 1 : 0,
                              a.fused, s));
    }
    DW_HIP(launch_update(a, (int)h->lay.n_upd_blocks, s));
    h->norms_valid = true;
    h->calls += 1;
    return DW_OK;
  }
  if (tiny_step_ok(h->cfg, h->lay)) {
    // a model that fits in one compute unit's LDS: z, network, update and distances in one kernel, a block per worker
    uint64_t keys[DW_MAX_K];
    const uint64_t G = 0x9E3779B97F4A7C15ull;
    for (int i = 0; i < h->cfg.k; ++i) {
      const uint64_t k1 = mix64_host(h->cfg.seed + G * (uint64_t)(i + 1));
      keys[i] = mix64_host(k1 + G * (uint64_t)(h->t[i] + 1));          // stream position t_i: before the increment
    }
    for (int i = 0; i < h->cfg.k; ++i)
      if ((active >> i) & 1ull) h->t[i] += 1;
    UpdateArgs a;
    fill_update_args(h, a, h->at<float>(h->lay.g), h->at<float>(h->lay.hz), h->lay.Pp, zb, zs, active, false);
    DW_HIP(launch_tiny_step(h->cfg, h->ws, h->lay, d_x, d_y, d_zbits, a, keys, loss, s));
    h->norms_valid = true;
    h->calls += 1;
    return DW_OK;
  }
  for (int i = 0; i < h->cfg.k; ++i)
    if ((active >> i) & 1ull) h->t[i] += 1;
  const bool fused = h->lay.n_fuse_slots > 0;
  UpdateArgs a;
  fill_update_args(h, a, h->at<float>(h->lay.g), h->at<float>(h->lay.hz), h->lay.Pp, zb, zs, active, fused);
  int st = clear_fused_partials(h, s);
  if (st != DW_OK) return st;
  const UpdateArgs* fu = fused ? &a : nullptr;
  // The distances to the centre are only used by a communication round.  Fused layers pay for them with a read
  // of the centre per worker, so they skip it on steps after which, going by the period of the latest
  // dw_elastic_sync call, no round is due; should a round come anyway, it measures the distances itself.
  const bool dist = !fused || h->last_tau <= 1 || (h->calls + 1) % h->last_tau == 0;
  if (h->lay.n_conv > 0) {
    st = run_network_cnn(h->cfg, h->ws, h->lay, d_x, d_y, zb, zs, active, loss, s);
    if (st != DW_OK) return st;
    if (h->cfg.conv_avg)
      DW_HIP(launch_conv_window_mean(h->at<float>(h->lay.hz), zb, h->lay.Pp, zs, h->lay, h->cfg.k, active, s));
  } else {
    st = run_network(h->cfg, h->ws, h->lay, d_x, d_y, zb, zs, active, loss, fu, dist, s, nullptr, nullptr, nullptr, false, 0,
                     h->side);
    if (st != DW_OK) return st;
  }
  DW_HIP(launch_update(a, (int)h->lay.n_upd_blocks, s));
  h->norms_valid = dist;
  h->calls += 1;
  return DW_OK;
}

}  // namespace


extern "C" {

const char* dw_strerror(int status) {
  switch (status) {
    case DW_OK: return "ok";
    case DW_ERR_NULL: return "required pointer is NULL";
    case DW_ERR_CONFIG: return "invalid configuration (dims, k, batch, dtype or alignment)";
    case DW_ERR_HYPER: return "invalid hyper-parameter (lr, beta, eps, hpow, avg_block, alpha, kappa, p or c)";
    case DW_ERR_WORKSPACE: return "workspace too small or misaligned";
    case DW_ERR_ARG: return "invalid call argument";
    case DW_ERR_HIP: return "HIP runtime error";
    case DW_ERR_MODE: return "call not valid for this handle";
    case DW_ERR_TOO_LARGE: return "size beyond the fixed capacity of a call that allocates nothing";
    default: return status > 0 ? "ok (positive result)" : "unknown status";
  }
}

int dw_last_hip_error(void) { return g_last_hip; }

int dw_param_count(const dw_config* cfg, int64_t* n_params) {
  if (!cfg || !n_params) return DW_ERR_NULL;
  Layout lay;
  const int st = validate(cfg, &lay);
  if (st != DW_OK) return st;
  *n_params = lay.P;
  return DW_OK;
}

// stream (default priority, not synchronising with the legacy default stream) and events of a SideStream
static hipError_t make_side_stream(SideStream** out, int n_layers) {
  SideStream* sd = new (std::nothrow) SideStream();
  if (!sd) return hipErrorOutOfMemory;
  sd->s = nullptr; sd->join = nullptr;
  for (int l = 0; l <= DW_MAX_LAYERS; ++l) sd->fork[l] = nullptr;
  hipError_t e = hipStreamCreateWithFlags(&sd->s, hipStreamNonBlocking);
  for (int l = 2; l <= n_layers && e == hipSuccess; ++l) e = hipEventCreateWithFlags(&sd->fork[l], hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&sd->join, hipEventDisableTiming);
  *out = sd;                                             // (freed by the caller, also after a failure)
  return e;
}

static void free_side_stream(SideStream* sd) {
  if (!sd) return;
  for (int l = 0; l <= DW_MAX_LAYERS; ++l)
    if (sd->fork[l]) (void)hipEventDestroy(sd->fork[l]);
  if (sd->join) (void)hipEventDestroy(sd->join);
  if (sd->s) { (void)hipStreamSynchronize(sd->s); (void)hipStreamDestroy(sd->s); }
  delete sd;
}

size_t dw_workspace_bytes(const dw_config* cfg) {
  Layout lay;
  if (validate(cfg, &lay) != DW_OK) return 0;
  return lay.total;
}

int dw_init(dw_handle** out, const dw_config* cfg, void* d_workspace, size_t workspace_bytes,
            const float* theta0, int theta0_on_device, void* stream) {
  if (!out || !cfg || !d_workspace || !theta0) return DW_ERR_NULL;
  Layout lay;
  const int st = validate(cfg, &lay);
  if (st != DW_OK) return st;
  if (workspace_bytes < lay.total || (reinterpret_cast<uintptr_t>(d_workspace) & 255u)) return DW_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  dw_handle* h = new (std::nothrow) dw_handle();
  if (!h) return DW_ERR_ARG;
  h->cfg = *cfg;
  h->lay = lay;
  h->ws = reinterpret_cast<char*>(d_workspace);
  std::memset(h->t, 0, sizeof(h->t));
  h->calls = 0; h->rounds = 0; h->norms_valid = false; h->prof = nullptr; h->last_tau = 1; h->side = nullptr;
  int rc = DW_OK;
  do {
    if (lay.overlap_wgrad) {
      const hipError_t es = make_side_stream(&h->side, cfg->n_layers);
      if (es != hipSuccess) { rc = hip_fail(es); break; }
    }
    hipError_t e = launch_fill_zero(h->ws, lay.total, s);            // moments, padding, history: all zero
    if (e != hipSuccess) { rc = hip_fail(e); break; }
    e = hipMemcpyAsync(h->at<float>(lay.centre), theta0, (size_t)lay.P * sizeof(float),
                       theta0_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, s);
    if (e != hipSuccess) { rc = hip_fail(e); break; }
    e = launch_broadcast(h->at<float>(lay.theta), h->at<float>(lay.centre),
                         cfg->dtype == DW_BF16 ? h->at<uint16_t>(lay.wb16) : nullptr, lay.Pp, cfg->k, s);
    if (e != hipSuccess) { rc = hip_fail(e); break; }
    if (!theta0_on_device) {
      e = hipStreamSynchronize(s);                                    // the host buffer may go away
      if (e != hipSuccess) { rc = hip_fail(e); break; }
    }
  } while (0);
  if (rc != DW_OK) { free_side_stream(h->side); delete h; return rc; }
  *out = h;
  return DW_OK;
}

static void free_profiler(dw_handle* h) {
  if (!h->prof) return;
  for (int i = 0; i < h->prof->created; ++i) {
    (void)hipEventDestroy(h->prof->start[i]);
    (void)hipEventDestroy(h->prof->stop[i]);
  }
  delete h->prof;
  h->prof = nullptr;
}

// makes the handle's profiler current for the launches of one API call
struct ProfilerGuard {
  explicit ProfilerGuard(dw_handle* h) { tl_profiler = h->prof; }
  ~ProfilerGuard() { tl_profiler = nullptr; }
};

int dw_profile(dw_handle* h, int enable) {
  if (!h) return DW_ERR_NULL;
  if (enable && !h->prof) {
    h->prof = new (std::nothrow) Profiler();
    if (!h->prof) return DW_ERR_ARG;
  } else if (!enable) {
    free_profiler(h);
  }
  return DW_OK;
}

int dw_profile_read(dw_handle* h, int64_t* n_launches, double* total_ms, int64_t* n_dropped, void* stream) {
  if (!h || !n_launches || !total_ms) return DW_ERR_NULL;
  if (!h->prof) return DW_ERR_MODE;
  DW_HIP(hipStreamSynchronize((hipStream_t)stream));
  for (int c = 0; c < KC_COUNT; ++c) { n_launches[c] = 0; total_ms[c] = 0.0; }
  Profiler* p = h->prof;
  for (int i = 0; i < p->used; ++i) {
    float ms = 0.f;
    DW_HIP(hipEventElapsedTime(&ms, p->start[i], p->stop[i]));
    n_launches[p->cls[i]] += 1;
    total_ms[p->cls[i]] += (double)ms;
  }
  if (n_dropped) *n_dropped = p->dropped;
  p->used = 0; p->dropped = 0;
  return DW_OK;
}

int dw_destroy(dw_handle* h) {
  if (!h) return DW_ERR_NULL;
  free_profiler(h);
  free_side_stream(h->side);
  delete h;
  return DW_OK;
}

int dw_worker_step(dw_handle* h, const void* d_x, const int32_t* d_y, const uint32_t* d_zbits,
                   const uint8_t* h_active, float* d_loss, void* stream) {
  if (!h || !d_x || !d_y) return DW_ERR_NULL;
  if (h->cfg.n_layers == 0) return DW_ERR_MODE;
  ProfilerGuard pg(h);
  if ((reinterpret_cast<uintptr_t>(d_x) & 15u) || (reinterpret_cast<uintptr_t>(d_zbits) & 7u)) return DW_ERR_ARG;
  hipStream_t s = (hipStream_t)stream;
  const uint64_t active = mask_from(h_active, h->cfg.k);
  if (active == 0) { h->calls += 1; return DW_OK; }
  if (probes(h) > 1 && d_zbits) return DW_ERR_ARG;       // several probes per step come from the library's stream
  // (a baseline's first-order step draws no z: the direction the network's R-parts then run along is whatever the
  // sign-bit buffer holds, and their result is not used)
  if (!d_zbits && probes(h) == 1 && h->cfg.optimizer == DW_OPT_ADAHESSIAN && !tiny_step_ok(h->cfg, h->lay)) {
    const int st = draw_z(h, active, s);
    if (st != DW_OK) return st;
  }
  return run_step(h, d_x, d_y, d_zbits, active, d_loss, s);    // (no loss wanted: nothing adds it up)
}

int dw_update_only(dw_handle* h, const float* d_g, const float* d_hz, const uint32_t* d_zbits,
                   const uint8_t* h_active, void* stream) {
  if (!h || !d_g) return DW_ERR_NULL;
  const bool first_order = h->cfg.optimizer != DW_OPT_ADAHESSIAN;
  if (!d_hz && !first_order) return DW_ERR_NULL;
  if (!d_hz) d_hz = d_g;                              // never read by a first-order step
  if (h->lay.P % 4 != 0) return DW_ERR_MODE;          // worker i sits at offset i*P: needs 16-byte rows
  if (h->lay.n_conv > 0 && h->cfg.conv_avg) return DW_ERR_MODE;   // the window mean needs a writable Hz
  ProfilerGuard pg(h);
  if ((reinterpret_cast<uintptr_t>(d_g) & 15u) || (reinterpret_cast<uintptr_t>(d_hz) & 15u) ||
      (reinterpret_cast<uintptr_t>(d_zbits) & 7u))
    return DW_ERR_ARG;
  hipStream_t s = (hipStream_t)stream;
  const uint64_t active = mask_from(h_active, h->cfg.k);
  if (active == 0) { h->calls += 1; return DW_OK; }
  if (!d_zbits && !first_order) {
    const int st = draw_z(h, active, s);
    if (st != DW_OK) return st;
  }
  return run_update(h, d_g, d_hz, h->lay.P, d_zbits, active, s);
}

int dw_elastic_sync(dw_handle* h, int mode, const float* h_h1, const float* h_h2,
                    const uint8_t* h_participate, int tau, void* stream) {
  if (!h) return DW_ERR_NULL;
  const int sequential = (mode & DW_SEQUENTIAL) ? 1 : 0;
  mode &= ~DW_SEQUENTIAL;
  if (mode != DW_FIXED && mode != DW_MANUAL && mode != DW_DYNAMIC) return DW_ERR_ARG;
  if (mode == DW_MANUAL && (!h_h1 || !h_h2)) return DW_ERR_NULL;
  if (tau < 1) return DW_ERR_ARG;
  h->last_tau = tau;
  if (h->calls % tau != 0) return 0;
  ProfilerGuard pg(h);
  hipStream_t s = (hipStream_t)stream;
  const dw_config& c = h->cfg;
  const Layout& L = h->lay;
  if (!h->norms_valid) {
    // distances only: no worker is marked active, so the update kernel just measures theta_i - centre
    UpdateArgs a;
    fill_update_args(h, a, nullptr, nullptr, 0, h->at<uint32_t>(L.zbits), L.z_stride, 0ull);
    { const int st = clear_fused_partials(h, s); if (st != DW_OK) return st; }
    DW_HIP(launch_update(a, (int)L.n_upd_blocks, s));
  }
  WeightArgs w;
  w.partials = h->at<double>(L.partials);
  w.n_blocks = (int)L.n_upd_blocks;
  w.partials_f = L.n_fuse_slots > 0 ? h->at<double>(L.partials_f) : nullptr;
  w.n_blocks_f = L.n_fuse_slots;
  w.u_ring = h->at<double>(L.u_ring);
  w.score = h->at<double>(L.score);
  w.omh1 = h->at<float>(L.omh1);
  w.h2 = h->at<float>(L.h2);
  w.k = c.k; w.p = c.p; w.mode = mode;
  const int ring = c.p + 1;
  w.slot = (int)(h->rounds % ring);
  w.n_valid = (int)(h->rounds + 1 < ring ? h->rounds + 1 : ring);
  w.alpha = c.alpha; w.kappa = c.kappa;
  for (int j = 0; j < DW_MAX_P; ++j) w.c[j] = j < c.p ? c.c[j] : 0.f;
  for (int i = 0; i < DW_MAX_K; ++i) {
    w.man_h1[i] = (mode == DW_MANUAL && i < c.k) ? h_h1[i] : 0.f;
    w.man_h2[i] = (mode == DW_MANUAL && i < c.k) ? h_h2[i] : 0.f;
  }
  PullArgs p;
  p.theta = h->at<float>(L.theta); p.centre = h->at<float>(L.centre);
  p.wb16 = c.dtype == DW_BF16 ? h->at<uint16_t>(L.wb16) : nullptr;
  p.omh1 = w.omh1; p.h2 = w.h2;
  p.Pp = L.Pp; p.k = c.k;
  p.part_mask = mask_from(h_participate, c.k);
  p.sequential = sequential;
  if (sync_fusable(w, p)) {
    DW_HIP(launch_weights_and_pull(w, p, s));
  } else {
    DW_HIP(launch_weights(w, s));
    DW_HIP(launch_pull(p, s));
  }
  h->rounds += 1;
  h->norms_valid = false;
  return 1;
}

size_t dw_partition_scratch_bytes(int64_t n) {
  if (n < 1 || n > DW_MAX_POINTS) return 0;
  return partition_scratch_bytes(n);
}

int64_t dw_overlap_partition(int64_t n, int64_t o, int k, uint64_t seed, int32_t* d_index, void* d_scratch,
                             size_t scratch_bytes, void* stream) {
  if (n < 1 || n > DW_MAX_POINTS || o < 0 || o > n || k < 1 || k > DW_MAX_K) return DW_ERR_ARG;
  const int64_t sz = (n - o) / k;
  if (!d_scratch || (!d_index && o + sz > 0)) return DW_ERR_NULL;
  if (scratch_bytes < partition_scratch_bytes(n) || (reinterpret_cast<uintptr_t>(d_scratch) & 255u))
    return DW_ERR_WORKSPACE;
  DW_HIP(launch_partition(n, o, k, seed, d_index, d_scratch, (hipStream_t)stream));
  return sz;
}

int dw_draw_batch(dw_handle* h, const void* d_data, const int32_t* d_labels, int64_t n, const int32_t* d_index,
                  int64_t m, uint64_t seed, const uint8_t* h_active, void* d_x, int32_t* d_y, void* stream) {
  if (!h || !d_data || !d_labels || !d_index || !d_x || !d_y) return DW_ERR_NULL;
  if (h->cfg.n_layers == 0) return DW_ERR_MODE;
  if (n < 1 || n > DW_MAX_POINTS || m < 1 || m > n) return DW_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(d_data) & 15u) || (reinterpret_cast<uintptr_t>(d_x) & 15u)) return DW_ERR_ARG;
  ProfilerGuard pg(h);
  const uint64_t active = mask_from(h_active, h->cfg.k);
  if (active == 0) return DW_OK;
  const uint64_t G = 0x9E3779B97F4A7C15ull;
  uint64_t keys[DW_MAX_K];
  for (int j = 0; j < h->cfg.k; ++j)
    keys[j] = mix64_host(mix64_host(seed + G * (uint64_t)(j + 1)) + G * (uint64_t)(h->t[j] + 1));
  // one sample: d_0 values, or a whole image in front of a convolutional model
  const int64_t row_elems = h->lay.n_conv > 0 ? (int64_t)h->cfg.img_h * h->cfg.img_w * h->cfg.img_c : h->cfg.dims[0];
  const int64_t row_bytes64 = row_elems * (h->cfg.dtype == DW_BF16 ? 2 : 4);
  if (row_bytes64 % 16 != 0 || row_bytes64 > (1 << 30)) return DW_ERR_MODE;     // rows are moved as 16-byte pieces
  const int row_bytes = (int)row_bytes64;
  DW_HIP(launch_gather(d_data, d_labels, d_index, n, m, row_bytes, h->cfg.batch, h->cfg.k, keys, active, d_x, d_y,
                       (hipStream_t)stream));
  return DW_OK;
}

static int state_ptr(dw_handle* h, int what, int worker, int64_t offset, int64_t count, char** ptr, size_t* bytes) {
  const Layout& L = h->lay;
  const int k = h->cfg.k;
  if (offset < 0 || count < 0) return DW_ERR_ARG;
  if (what != DW_S_CENTRE && (worker < 0 || worker >= k)) return DW_ERR_ARG;
  size_t base = 0, es = 4;
  int64_t n = L.P, stride = L.Pp;
  if (what > DW_S_ACT && what < DW_S_ACT + h->cfg.n_layers) {
    const int l = what - DW_S_ACT;
    es = h->cfg.dtype == DW_BF16 ? 2 : 4;
    n = (int64_t)h->cfg.batch * h->cfg.dims[l];
    if (offset + count > n) return DW_ERR_ARG;
    *ptr = h->ws + L.act[l] + ((size_t)worker * n + offset) * es;
    *bytes = (size_t)count * es;
    return DW_OK;
  }
  switch (what) {
    case DW_S_THETA: base = L.theta; break;
    case DW_S_M: base = L.m; break;
    case DW_S_V: base = L.v; break;
    case DW_S_G: if (h->cfg.n_layers == 0) return DW_ERR_MODE; base = L.g; break;
    case DW_S_HZ: if (h->cfg.n_layers == 0) return DW_ERR_MODE; base = L.hz; break;
    case DW_S_CENTRE: base = L.centre; worker = 0; break;
    case DW_S_ZBITS: base = L.zbits; n = 2 * ((L.P + 63) / 64); stride = L.z_stride; break;
    case DW_S_ZBITS_T: if (L.zbits_t == 0) return DW_ERR_MODE; base = L.zbits_t; n = 2 * ((L.P + 63) / 64); stride = L.z_stride; break;
    case DW_S_SCORE: base = L.score; es = 8; n = 4; stride = 4; break;
    default: return DW_ERR_ARG;
  }
  if (offset + count > n) return DW_ERR_ARG;
  *ptr = h->ws + base + ((size_t)worker * stride + offset) * es;
  *bytes = (size_t)count * es;
  return DW_OK;
}

int dw_get_state(dw_handle* h, int what, int worker, int64_t offset, int64_t count, void* h_buf, void* stream) {
  if (!h || !h_buf) return DW_ERR_NULL;
  hipStream_t s = (hipStream_t)stream;
  if (what == DW_S_STEPS) {
    if (worker < 0 || worker >= h->cfg.k || offset != 0 || count != 1) return DW_ERR_ARG;
    *reinterpret_cast<int64_t*>(h_buf) = h->t[worker];
    return DW_OK;
  }
  if (what == DW_S_COUNTERS) {
    if (offset != 0 || count != 3) return DW_ERR_ARG;
    int64_t* out = reinterpret_cast<int64_t*>(h_buf);
    out[0] = h->calls; out[1] = h->rounds; out[2] = h->last_tau;
    return DW_OK;
  }
  if (what == DW_S_U_HIST) {
    if (worker < 0 || worker >= h->cfg.k || offset != 0 || count != 2 + DW_MAX_P) return DW_ERR_ARG;
    double ring[DW_MAX_P + 1];
    DW_HIP(hipMemcpyAsync(ring, h->at<double>(h->lay.u_ring) + (size_t)worker * (DW_MAX_P + 1), sizeof(ring),
                          hipMemcpyDeviceToHost, s));
    DW_HIP(hipStreamSynchronize(s));
    double* out = reinterpret_cast<double*>(h_buf);
    const int R = h->cfg.p + 1;
    const int n = (int)(h->rounds < R ? h->rounds : R);
    out[0] = (double)n;
    for (int j = 0; j < DW_MAX_P + 1; ++j) out[1 + j] = 0.0;
    for (int j = 0; j < n; ++j) {                      // oldest first
      const int64_t round = h->rounds - n + j;
      out[1 + j] = ring[round % R];
    }
    return DW_OK;
  }
  char* p; size_t bytes;
  const int st = state_ptr(h, what, worker, offset, count, &p, &bytes);
  if (st != DW_OK) return st;
  if (bytes == 0) return DW_OK;
  DW_HIP(hipMemcpyAsync(h_buf, p, bytes, hipMemcpyDeviceToHost, s));
  DW_HIP(hipStreamSynchronize(s));
  return DW_OK;
}

int dw_set_state(dw_handle* h, int what, int worker, int64_t offset, int64_t count, const void* h_buf, void* stream) {
  if (!h || !h_buf) return DW_ERR_NULL;
  hipStream_t s = (hipStream_t)stream;
  if (what == DW_S_STEPS) {
    if (worker < 0 || worker >= h->cfg.k || offset != 0 || count != 1) return DW_ERR_ARG;
    const int64_t t = *reinterpret_cast<const int64_t*>(h_buf);
    if (t < 0) return DW_ERR_ARG;
    h->t[worker] = t;
    return DW_OK;
  }
  if (what == DW_S_COUNTERS) {
    if (offset != 0 || count != 3) return DW_ERR_ARG;
    const int64_t* in = reinterpret_cast<const int64_t*>(h_buf);
    if (in[0] < 0 || in[1] < 0 || in[2] < 1 || in[2] > INT32_MAX) return DW_ERR_ARG;
    h->calls = in[0]; h->rounds = in[1]; h->last_tau = (int)in[2];
    h->norms_valid = false;                               // whatever was measured belongs to another point of the run
    return DW_OK;
  }
  if (what == DW_S_U_HIST) {
    // the n most recent u of one worker, oldest first: value j is that of round rounds - n + j and goes to the ring
    // slot the weight kernel reads it from
    if (worker < 0 || worker >= h->cfg.k || offset != 0 || count != 2 + DW_MAX_P) return DW_ERR_ARG;
    const double* in = reinterpret_cast<const double*>(h_buf);
    const int R = h->cfg.p + 1;
    const int64_t want = h->rounds < R ? h->rounds : R;
    if (!(in[0] == (double)want)) return DW_ERR_ARG;
    double ring[DW_MAX_P + 1];
    for (int j = 0; j < DW_MAX_P + 1; ++j) ring[j] = 0.0;
    for (int j = 0; j < (int)want; ++j) {
      if (!std::isfinite(in[1 + j])) return DW_ERR_ARG;
      ring[(h->rounds - want + j) % R] = in[1 + j];
    }
    DW_HIP(hipMemcpyAsync(h->at<double>(h->lay.u_ring) + (size_t)worker * (DW_MAX_P + 1), ring, sizeof(ring),
                          hipMemcpyHostToDevice, s));
    DW_HIP(hipStreamSynchronize(s));                      // `ring` lives on this frame
    return DW_OK;
  }
  if (what != DW_S_THETA && what != DW_S_M && what != DW_S_V && what != DW_S_CENTRE) return DW_ERR_ARG;
  char* p; size_t bytes;
  const int st = state_ptr(h, what, worker, offset, count, &p, &bytes);
  if (st != DW_OK) return st;
  if (bytes == 0) return DW_OK;
  DW_HIP(hipMemcpyAsync(p, h_buf, bytes, hipMemcpyHostToDevice, s));
  if (what == DW_S_THETA && h->cfg.dtype == DW_BF16) {
    float* th = h->at<float>(h->lay.theta) + (size_t)worker * h->lay.Pp;
    uint16_t* wb = h->at<uint16_t>(h->lay.wb16) + (size_t)worker * h->lay.Pp;
    DW_HIP(launch_refresh_bf16(th, wb, h->lay.Pp, s));
  }
  DW_HIP(hipStreamSynchronize(s));
  if (what == DW_S_THETA || what == DW_S_CENTRE) h->norms_valid = false;
  return DW_OK;
}

}  // extern "C"
