/*
 * dw.h -- C ABI of the dynamic-weighted elastic AdaHessian hot path for AMD MI355X (gfx950).
 *
 * The library simulates one master ("centre") and k worker replicas of a ReLU MLP classifier on a
 * single GPU, as in the paper's single-device experiments (Xu & Carr, "A Dynamic Weighting Strategy
 * to Mitigate Worker Node Failure in Distributed Deep Learning", Section VI).  Its three hot calls
 * follow the paper's problem statement:
 *
 *   dw_init          master model + k workers, each starting as a copy of it   (Section II, assumptions)
 *   dw_worker_step   one local AdaHessian step per worker on its own minibatch  (Section II eq.(2),(4);
 *                    Section IV-B: Hutchinson estimate z*(Hz), spatial averaging, Adam-like moments)
 *   dw_elastic_sync  one communication round every tau steps: log-distance u, raw score a,
 *                    weights h1(a), h2(a), elastic pull of worker and master    (Section V-B eq.(10)-(13);
 *                    Section IV-A eq.(8)-(9) for the fixed-rate case; tau: Section VI footnote)
 *
 * Conventions
 *   - Every function returns DW_OK (0) or a negative dw_status; dw_elastic_sync returns 1 when a round
 *     was enqueued and 0 when the step count is not a multiple of tau.  On error nothing is enqueued.
 *   - Pointers named d_* are device pointers, h_* are host pointers.  The caller owns all memory,
 *     including the workspace handed to dw_init, and the stream.  The library allocates no device
 *     memory and never synchronises the stream, except dw_get_state/dw_set_state/dw_init (see there).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls on one handle must be
 *     issued from one host thread at a time and on one stream.
 *   - Canonical parameter layout (index space of theta, m, v, g, Hz and of the Rademacher vector z):
 *     for l = 1..L the weight W_l row-major [d_l][d_{l-1}] followed by the bias b_l[d_l], no padding
 *     (with a convolutional front end its kernels and biases come first, see dw_config.n_conv).
 *   - Rademacher bits: element j of z is +1 when bit (j mod 32) of 32-bit word floor(j/32) is set, else -1.
 */
#ifndef DW_H_
#define DW_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DW_MAX_LAYERS 8      /* linear layers L                                  */
#define DW_MAX_K 64          /* worker replicas k                                */
#define DW_MAX_P 8           /* length p of the raw-score history weights c_j    */
#define DW_MAX_CLASSES 16    /* width d_L of the output layer                    */
#define DW_MAX_SAMPLES 8     /* Rademacher probes per step                       */
#define DW_MAX_CONV 2        /* 3x3 convolutions in front of the linear layers   */

typedef enum {
  DW_OK = 0,
  DW_ERR_NULL = -1,          /* a required pointer is NULL                                   */
  DW_ERR_CONFIG = -2,        /* dims / k / batch / dtype out of range or misaligned          */
  DW_ERR_HYPER = -3,         /* lr, beta, eps, alpha, kappa, p, c_j or avg_block invalid      */
  DW_ERR_WORKSPACE = -4,     /* workspace too small or not 256-byte aligned                  */
  DW_ERR_ARG = -5,           /* bad call argument (mode, worker index, range, alignment)     */
  DW_ERR_HIP = -6,           /* a HIP runtime call failed (see dw_last_hip_error)            */
  DW_ERR_MODE = -7,          /* call not valid for this handle (MLP call on a flat problem ...) */
  DW_ERR_TOO_LARGE = -8      /* size beyond the fixed capacity of a call that allocates nothing */
} dw_status;

/* arithmetic type of the network part (optimizer state is always fp32) */
#define DW_F32 0             /* fp32 weights, activations, MFMA accumulation                            */
#define DW_BF16 1            /* bf16 weights/activations (round-to-nearest-even), fp32 accumulation     */

/* the local step a worker takes (dw_config.optimizer) */
#define DW_OPT_ADAHESSIAN 0  /* Section IV-B, the method's own step                                             */
#define DW_OPT_SGD 1         /* theta -= lr * g  (Section II eq.(3)): worker step of the EASGD baseline, Section VI */
#define DW_OPT_MOMENTUM 2    /* b = momentum * b + g; theta -= lr * b: EASGD with momentum (Section VI; Section VII
                                uses momentum 0.5, lr 0.01).  The velocity b is the state read through DW_S_M.   */

/* how dw_elastic_sync chooses the per-worker weights (h1_i, h2_i) */
#define DW_FIXED 0           /* h1 = h2 = alpha: plain elastic averaging (Section IV-A)                 */
#define DW_MANUAL 1          /* caller-supplied: weights set with foreknowledge of the failures (Section VI) */
#define DW_DYNAMIC 2         /* h1(a), h2(a) from the raw score (Section V-B)                           */
/* may be OR-ed into the mode: the participating workers exchange with the master one after the other, in index
 * order, each exchange being eq.(12)-(13) with the centre as the previous one left it (asynchronous procedure,
 * Section II; full communication round, Section VI).  Without it all differences use the centre of the round's
 * start.  The weights are those of the round either way (u_i is measured against the centre at its start). */
#define DW_SEQUENTIAL 16

/* selectors for dw_get_state / dw_set_state */
#define DW_S_THETA 0         /* float[P]   worker parameters                                            */
#define DW_S_M 1             /* float[P]   first moment                                                 */
#define DW_S_V 2             /* float[P]   second moment                                                */
#define DW_S_G 3             /* float[P]   last gradient                                                */
#define DW_S_HZ 4            /* float[P]   last Hessian-vector product                                  */
#define DW_S_CENTRE 5        /* float[P]   master parameters (worker index ignored)                     */
#define DW_S_ZBITS 6         /* uint32[ceil(P/32)] bits of the last z drawn by the library              */
#define DW_S_SCORE 7         /* double[4]  {u, a, h1, h2} of the last round (get only)                  */
#define DW_S_U_HIST 8        /* double[1+DW_MAX_P+1]: count n, then the n most recent u, oldest first   */
#define DW_S_STEPS 9         /* int64[1]   local steps t_i taken by the worker                          */
#define DW_S_ZBITS_T 10      /* uint32[ceil(P/32)] the last z with the W-parts of some layers transposed: for the layers
                                whose data gradient runs on the large-tile bf16 kernel, bit (r, c) of V_l [d_l][d_{l-1}]
                                sits at woff_l + c*d_l + r; other positions are unspecified; get only; DW_ERR_MODE when
                                the handle keeps no such copy                                                */
#define DW_S_COUNTERS 11     /* int64[3]   {calls of dw_worker_step/dw_update_only so far, communication rounds so far,
                                period tau of the latest dw_elastic_sync call}; belongs to the handle, worker ignored */
#define DW_S_ACT 16          /* DW_S_ACT + l, l = 1..L-1: hidden activations a_l of the last step, [B][d_l]
                                floats (DW_F32) or bfloat16 bit patterns as uint16 (DW_BF16); get only      */

typedef struct dw_handle dw_handle;

typedef struct {
  int32_t n_layers;                 /* L >= 1 linear layers; 0 = flat parameter vector (update/sync only)   */
  int32_t dims[DW_MAX_LAYERS + 1];  /* d_0..d_L; d_0..d_{L-1} multiples of 4 (8 for DW_BF16), d_L <= DW_MAX_CLASSES */
  int64_t n_params;                 /* flat problem: P (multiple of 4); MLP: 0 or the P implied by dims     */
  int32_t k;                        /* workers, 1..DW_MAX_K                                                 */
  int32_t batch;                    /* minibatch size B per worker (m of eq.(2)); ignored when n_layers = 0 */
  int32_t dtype;                    /* DW_F32 | DW_BF16                                                     */
  float lr, beta1, beta2, eps;      /* eta and beta of Section VII; eps added to the denominator            */
  float hpow;                       /* Hessian power: denominator (sqrt(v_hat))^hpow + eps                  */
  int32_t avg_block;                /* spatial-averaging block b along fan-in: power of two <= 256 dividing
                                       d_0..d_{L-1} (flat problem: dividing P); 1 = no averaging             */
  float alpha;                      /* fixed moving rate, 0 < alpha <= 1 (Section IV-A)                     */
  float kappa;                      /* the negative constant of the piecewise maps h1, h2 (Section V-B)      */
  int32_t p;                        /* number of history differences, 1..DW_MAX_P                           */
  float c[DW_MAX_P];                /* c_0 (most recent) .. c_{p-1}; must sum to 1 within 1e-5 (eq.(10)-(11)) */
  uint64_t seed;                    /* seed of the library's Rademacher stream                              */
  int32_t n_samples;                /* Rademacher probes per dw_worker_step (the n of Section IV-B's Hutchinson
                                       estimate; the experiments use 1).  0 or 1: one probe.  Up to DW_MAX_SAMPLES:
                                       D is the mean of z_j*(Hz_j); probe j of a worker's step t comes from
                                       position t*n + j of its stream; the network runs once per probe and
                                       dw_worker_step takes no caller-supplied z.  With fuse_update = 1 the
                                       weight-gradient kernels keep the running sum of z_j*(Hz_j) of their
                                       layers and the last probe's applies the update; with two probes in
                                       DW_BF16 one launch per layer multiplies for both probes instead.         */
  int32_t fuse_update;              /* 0: g and Hz of the last dw_worker_step stay readable (DW_S_G, DW_S_HZ).
                                       1: the library may apply the update of a weight matrix inside the kernel
                                          that produces its gradient; the W-parts of g and Hz of such layers are
                                          then never written (reading them returns stale values).  Same
                                          arithmetic either way.                                              */
  /* Convolutional front end (Section VI trains a small CNN): n_conv 3x3 convolutions, stride 1, no padding, each
   * followed by ReLU, one 2x2 max-pool after the last, then the flattened map (row, column, channel) feeds the
   * linear layers, so dims[0] must equal (H_out/2)*(W_out/2)*conv_c[n_conv-1].  Needs DW_F32, avg_block = 1,
   * fuse_update = 0.  The minibatch x is then [k][B][img_h][img_w][img_c] floats (channels last).
   * Parameters of convolution j come first in the canonical layout: W_j [C_j][K_j] with K_j = 9*C_{j-1} rounded up
   * to a multiple of 4, entry (dy*3 + dx)*C_{j-1} + ci of a row being tap (dy, dx) on input channel ci, the last
   * K_j - 9*C_{j-1} entries of a row padding (they must be 0 in theta_0 and then stay 0); then b_j [C_j]. */
  int32_t n_conv;                   /* 0 (none) .. DW_MAX_CONV                                              */
  int32_t img_h, img_w, img_c;      /* input image                                                          */
  int32_t conv_c[DW_MAX_CONV];      /* output channels C_j, multiples of 4                                  */
  int32_t conv_avg;                 /* 1: D = z*Hz of a convolution kernel is replaced by its mean over the
                                       3x3 window of each (output, input) channel pair (Section IV-B); biases
                                       and linear layers are not averaged                                    */
  /* Baseline worker steps (Section VI compares against elastic averaging SGD with and without momentum).  With
   * DW_OPT_SGD or DW_OPT_MOMENTUM the step uses the minibatch gradient alone: no z is drawn, avg_block, hpow, the
   * betas and eps are not used, n_samples must be 0 or 1 and fuse_update 0, and dw_update_only ignores d_hz (it
   * may be NULL).  The communication round is the same call (DW_FIXED gives elastic averaging SGD). */
  int32_t optimizer;                /* DW_OPT_ADAHESSIAN (0, default) | DW_OPT_SGD | DW_OPT_MOMENTUM          */
  float momentum;                   /* delta of DW_OPT_MOMENTUM, 0 <= momentum < 1                           */
} dw_config;

/* Human-readable text for a status code (never NULL). */
const char* dw_strerror(int status);
/* hipError_t (as int) of the last HIP failure seen by this thread's calls, 0 if none. */
int dw_last_hip_error(void);

/* Validate a configuration and return the parameter count P per replica through *n_params. */
int dw_param_count(const dw_config* cfg, int64_t* n_params);

/* Device bytes dw_init needs for this configuration; 0 if the configuration is invalid. */
size_t dw_workspace_bytes(const dw_config* cfg);

/*
 * Create a handle over a caller-allocated workspace (256-byte aligned device memory of at least
 * dw_workspace_bytes(cfg) bytes, which must outlive the handle).  The centre is set to theta0 and all
 * k workers to copies of it (Section II: each worker starts with a copy of the master's model);
 * moments, step counts and the u history start empty.  theta0 holds P floats in canonical layout and may
 * live on the host (theta0_on_device = 0; copied synchronously) or on the device.
 */
int dw_init(dw_handle** out, const dw_config* cfg, void* d_workspace, size_t workspace_bytes,
            const float* theta0, int theta0_on_device, void* stream);

/* Free the host-side handle (device memory stays with the caller). */
int dw_destroy(dw_handle* h);

/*
 * One local AdaHessian step for every active worker (Section IV-B; update rule eq.(4)):
 *   forward and backward pass on the worker's minibatch -> mean loss and gradient g   (eq.(2), eq.(6))
 *   Rademacher z, Hessian-vector product Hz of the same minibatch loss, D = z*Hz       (Hutchinson, n = 1)
 *   block mean of D over avg_block neighbours along fan-in (biases excluded)
 *   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) D^2;  theta -= lr * (m/(1-b1^t)) / ((sqrt(v/(1-b2^t)))^hpow + eps)
 * and the squared distance of the new theta to the centre, kept for the next dw_elastic_sync.
 *
 *   d_x       [k][B][d_0] inputs: float (DW_F32) or bfloat16 (DW_BF16), 16-byte aligned
 *   d_y       [k][B] int32 class labels in [0, d_L)
 *   d_zbits   [k][zwords] uint32 sign bits of z per worker, zwords = 2*ceil(P/64); NULL = drawn by the
 *             library from its counter-based stream at (seed, worker, t_i)
 *   h_active  [k] bytes, 0 = the worker is frozen this step (no update, t_i unchanged); NULL = all active
 *   d_loss    [k] floats receiving the mean minibatch loss per worker (untouched for frozen ones); may be NULL
 */
int dw_worker_step(dw_handle* h, const void* d_x, const int32_t* d_y, const uint32_t* d_zbits,
                   const uint8_t* h_active, float* d_loss, void* stream);

/*
 * The optimizer part of dw_worker_step alone (Section IV-B: Hutchinson diagonal D = z*(Hz), its spatial average,
 * Adam-like moments with D in the second moment, bias correction; the preconditioned step of eq.(4)), on
 * caller-supplied gradients and Hessian-vector products d_g, d_hz ([k][P] floats each, 16-byte aligned; worker i
 * at offset i*P).  Other arguments as above.  Valid for flat problems and for MLP problems.
 */
int dw_update_only(dw_handle* h, const float* d_g, const float* d_hz, const uint32_t* d_zbits,
                   const uint8_t* h_active, void* stream);

/*
 * One communication round (Section V-B), taken only when the number of dw_worker_step/dw_update_only calls
 * so far is a multiple of tau (tau >= 1).  Every worker records u_i = log||theta_i - centre|| (centre as at
 * the start of the round) in its history and its raw score a_i (eq.(10)-(11)); then for each participating
 * worker  theta_i -= h1_i (theta_i - centre)  (eq.(12))  and the centre moves by the sum over participating
 * workers of  h2_i (theta_i - centre)  (eq.(13)), all differences taken against the centre before the round.
 *
 *   mode            DW_FIXED | DW_MANUAL | DW_DYNAMIC, optionally + DW_SEQUENTIAL
 *   h_h1, h_h2      [k] floats, required for DW_MANUAL, ignored otherwise
 *   h_participate   [k] bytes, 0 = this worker's communication is suppressed in this round (it still
 *                   records u); NULL = all participate
 * Returns 1 if a round was enqueued, 0 if skipped, negative on error.
 */
int dw_elastic_sync(dw_handle* h, int mode, const float* h_h1, const float* h_h2,
                    const uint8_t* h_participate, int tau, void* stream);

/*
 * Copy `count` elements starting at element `offset` of a state array to / from host memory.  Both calls
 * synchronise the stream before returning.  dw_set_state accepts DW_S_THETA, DW_S_M, DW_S_V, DW_S_CENTRE,
 * DW_S_STEPS, DW_S_COUNTERS and DW_S_U_HIST (for DW_BF16 the bf16 weight copy is refreshed after THETA is set).
 *
 * Checkpoint of a run: theta, m, v and the step count of every worker, the centre, the counters and every worker's
 * history of u (the state the raw score of eq.(10)-(11) is computed from).  Restore them into a handle created with
 * the same configuration, DW_S_COUNTERS before DW_S_U_HIST: the history of a worker must then hold
 * n = min(rounds, p + 1) values, as it does after `rounds` communication rounds (else DW_ERR_ARG).  A restored handle
 * continues bit for bit like the original when the checkpoint was taken right after a communication round; taken
 * between a step and its round it continues with distances summed in another order (same values to rounding).
 * Setting a history by hand is also the way to put a chosen raw score, and so a chosen branch of h1 and h2
 * (Section V-B), in front of the next round.
 */
int dw_get_state(dw_handle* h, int what, int worker, int64_t offset, int64_t count, void* h_buf, void* stream);
int dw_set_state(dw_handle* h, int what, int worker, int64_t offset, int64_t count, const void* h_buf, void* stream);

/*
 * Data overlap (Section V-A).  The n data points are shuffled by one seeded permutation (the order of the keys
 * mix(mix(seed) + GAMMA*(i+1)), SplitMix64's output function and increment, equal keys by index); its first o
 * entries are the subset O shared by all workers, the next k blocks of s = floor((n-o)/k) entries the private
 * subsets S_1..S_k; the last (n-o) mod k entries belong to no worker.
 *
 *   n, o, k     1 <= n <= DW_MAX_POINTS, 0 <= o <= n, 1 <= k <= DW_MAX_K
 *   d_index     device, [k][o + s] int32: row j receives D_j = O u S_j as point indices, O first, both parts in
 *               permutation order (nothing is written when o + s == 0)
 *   d_scratch   device, dw_partition_scratch_bytes(n) bytes, 256-byte aligned; contents undefined afterwards
 * Returns s (>= 0), or a negative dw_status.  Work is enqueued on `stream`; nothing is synchronised.
 */
#define DW_MAX_POINTS (1 << 21)
size_t dw_partition_scratch_bytes(int64_t n);
int64_t dw_overlap_partition(int64_t n, int64_t o, int k, uint64_t seed, int32_t* d_index, void* d_scratch,
                             size_t scratch_bytes, void* stream);

/*
 * dw_overlap_partition for callers that cannot allocate device memory or hand in a scratch buffer: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same result,
 * but the scratch is a fixed array inside the library's device image (12 bytes per point, DW_STATIC_MAX_POINTS points:
 * 1.5 MiB held by every GPU the library runs on until the process ends).  The call allocates and frees nothing.
 *   n           1 <= n <= DW_STATIC_MAX_POINTS; a larger n returns DW_ERR_TOO_LARGE and nothing is enqueued
 * Every call on one GPU uses that GPU's one array (the kernels reset the part they use): calls that overlap in time
 * on the same GPU, on any streams, race with each other; calls on one stream are ordered and safe.
 */
#define DW_STATIC_MAX_POINTS (1 << 17)
int64_t dw_overlap_partition_static(int64_t n, int64_t o, int k, uint64_t seed, int32_t* d_index, void* stream);

/*
 * The minibatch of every active worker (Section II eq.(3): each worker's gradient is that of a minibatch sampled
 * from its own data), drawn on the device from a resident data set: draw b of worker j at its local step t_j is
 * row d_index[j][floor(u * m / 2^64)] with u = mix(key(seed, j, t_j) + GAMMA*(b+1)), key as for the Rademacher
 * stream; independent uniform draws with replacement.  Call it before the dw_worker_step that consumes the batch
 * (same h_active), with a seed different from the configuration's.
 *
 *   h           an MLP or CNN handle: supplies k, the batch size B, the sample size d_0 (dims[0], or img_h*img_w*img_c
 *               with a convolutional front end; d_0 values must fill a multiple of 16 bytes, else DW_ERR_MODE), the
 *               element type and the t_j
 *   d_data      device, [n][d_0] in the handle's dtype (fp32 or bf16), 16-byte aligned
 *   d_labels    device, [n] int32
 *   d_index     device, [k][m] int32 as written by dw_overlap_partition (m = o + s >= 1)
 *   d_x, d_y    device outputs [k][B][d_0] (16-byte aligned) and [k][B]; rows of frozen workers are left alone.
 *               An entry of d_index outside [0, n) gives a row of zeros with label -1.
 */
int dw_draw_batch(dw_handle* h, const void* d_data, const int32_t* d_labels, int64_t n, const int32_t* d_index,
                  int64_t m, uint64_t seed, const uint8_t* h_active, void* d_x, int32_t* d_y, void* stream);

/*
 * Per-kernel timing for benchmarks (not part of the method).  While enabled, every kernel the handle launches
 * is bracketed by two HIP events on the caller's stream.  dw_profile_read synchronises the stream and returns,
 * per kernel class, the number of launches and their summed duration in milliseconds since the last read
 * (arrays of DW_N_KERNEL_CLASSES entries), then clears the record.  At most 8192 launches are kept between
 * reads; *n_dropped receives how many were not recorded (may be NULL).
 */
#define DW_N_KERNEL_CLASSES 10
#define DW_K_RADEMACHER 0    /* Rademacher bit generator                         */
#define DW_K_GEMM_FWD 1      /* forward + R-forward GEMMs                        */
#define DW_K_HEAD 2          /* softmax cross-entropy head                       */
#define DW_K_GEMM_WGRAD 3    /* weight-gradient + Hz GEMMs                       */
#define DW_K_GEMM_DGRAD 4    /* data-gradient + R-data-gradient GEMMs            */
#define DW_K_UPDATE 5        /* fused AdaHessian update (+ distance partials)    */
#define DW_K_WEIGHTS 6       /* dynamic-weight scalars                           */
#define DW_K_PULL 7          /* elastic pull + centre reduction                  */
#define DW_K_GATHER 8        /* minibatch rows drawn from a resident data set    */
#define DW_K_STEP 9          /* whole worker step of a small model in one kernel */
int dw_profile(dw_handle* h, int enable);
int dw_profile_read(dw_handle* h, int64_t* n_launches, double* total_ms, int64_t* n_dropped, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DW_H_ */
