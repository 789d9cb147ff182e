"""Plain CPU oracle for the dynamic-weighted elastic AdaHessian hot path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct statement of what the
GPU library computes.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may
import it; the product path never does, and it shares no code with the HIP kernels.

Everything is float64 numpy, one step of the method per function, in the paper's order and
notation (paper = Xu & Carr, "A Dynamic Weighting Strategy to Mitigate Worker Node Failure in
Distributed Deep Learning"):

  * minibatch mean loss and gradient                     -- Section II eq.(2), Section III-B eq.(6)
  * Hutchinson estimate z * (Hz), z Rademacher           -- Section IV-B, un-numbered display
  * spatial averaging, Adam-like moments, update         -- Section IV-B last paragraph, eq.(4)
  * SGD and momentum steps of the baselines              -- Section II eq.(3), Section VI, Section VII
  * log-distance u, weighted raw score a                 -- Section V-B, eq.(10)-(11)
  * piecewise-linear weights h1, h2                      -- Section V-B, un-numbered displays
  * elastic pull of worker and master                    -- Section V-B eq.(12)-(13)

The Hessian-vector product is computed as the directional derivative of the back-propagated
gradient (Pearlmutter's R-operator); `tests/` pins it to finite differences, to a brute-force
Hessian, and to the closed form for softmax regression.  No function here is "parity unpinned"
except whole multi-step trajectories, for which the paper prints no numbers.

Readings of points the paper leaves open are listed next to the code that takes them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64

# ---------------------------------------------------------------------------------------------
# Parameter layout (canonical, also the index space of z): for each linear layer l = 1..L the
# weight W_l stored row-major as [d_l][d_{l-1}], followed by the bias b_l[d_l]; no padding.
# ---------------------------------------------------------------------------------------------


def layer_offsets(dims: Sequence[int]) -> Tuple[List[Tuple[int, int]], int]:
    """Return [(offset of W_l, offset of b_l)] for l = 1..L and the total count P."""
    offs = []
    pos = 0
    for l in range(1, len(dims)):
        w_off = pos
        pos += dims[l] * dims[l - 1]
        b_off = pos
        pos += dims[l]
        offs.append((w_off, b_off))
    return offs, pos


def unpack(theta: np.ndarray, dims: Sequence[int]):
    """Views (W_l, b_l) into a flat parameter vector."""
    offs, total = layer_offsets(dims)
    assert theta.shape == (total,)
    out = []
    for l, (w_off, b_off) in enumerate(offs, start=1):
        W = theta[w_off:b_off].reshape(dims[l], dims[l - 1])
        b = theta[b_off:b_off + dims[l]]
        out.append((W, b))
    return out


# ---------------------------------------------------------------------------------------------
# Rademacher draws.  The paper only says "z is a Rademacher vector" (Section IV-B); the generator
# is a reading: a stateless counter-based stream built on the SplitMix64 output function
# (Steele, Lea & Flood, "Fast splittable pseudorandom number generators", OOPSLA 2014, in the
# constants of Vigna's public-domain splitmix64).  Word w of worker i at its local step t is
#     mix(key(seed, i, t) + GAMMA * (w + 1)),   key = mix(mix(seed + GAMMA*(i+1)) + GAMMA*(t+1)),
# i.e. the SplitMix64 sequence started from state key.  Element j of z is +1 when bit (j mod 64)
# of word floor(j/64) is set, else -1.
# ---------------------------------------------------------------------------------------------

_GAMMA = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK = (1 << 64) - 1


def _mix64(x: int) -> int:
    x &= _MASK
    x ^= x >> 30
    x = (x * _M1) & _MASK
    x ^= x >> 27
    x = (x * _M2) & _MASK
    x ^= x >> 31
    return x


def splitmix_stream(state: int, n_words: int) -> np.ndarray:
    """n_words outputs of SplitMix64 started from `state` (state is advanced before each output)."""
    out = np.empty(n_words, dtype=np.uint64)
    for w in range(n_words):
        out[w] = _mix64(state + _GAMMA * (w + 1))
    return out


def rademacher_key(seed: int, worker: int, step: int) -> int:
    k1 = _mix64(seed + _GAMMA * (worker + 1))
    return _mix64(k1 + _GAMMA * (step + 1))


def rademacher_words(seed: int, worker: int, step: int, n_params: int) -> np.ndarray:
    """ceil(n_params/64) uint64 words holding the sign bits of z for (seed, worker, step)."""
    n_words = (n_params + 63) // 64
    key = rademacher_key(seed, worker, step)
    # vectorised form of splitmix_stream(key, n_words)
    w = np.arange(1, n_words + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        x = np.uint64(key) + np.uint64(_GAMMA) * w
        x ^= x >> np.uint64(30)
        x *= np.uint64(_M1)
        x ^= x >> np.uint64(27)
        x *= np.uint64(_M2)
        x ^= x >> np.uint64(31)
    return x


def words_to_signs(words: np.ndarray, n_params: int) -> np.ndarray:
    """Expand uint64 words to a float64 vector of +1 / -1 (bit set -> +1)."""
    j = np.arange(n_params, dtype=np.uint64)
    bits = (words[(j >> np.uint64(6)).astype(np.int64)] >> (j & np.uint64(63))) & np.uint64(1)
    return np.where(bits == 1, 1.0, -1.0).astype(F64)


def words_to_u32(words: np.ndarray) -> np.ndarray:
    """The same bits as little-endian 32-bit halves (low half first), as the C ABI carries them."""
    lo = (words & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    hi = (words >> np.uint64(32)).astype(np.uint32)
    return np.stack([lo, hi], axis=1).reshape(-1)


# ---------------------------------------------------------------------------------------------
# Optional storage rounding for the mixed-precision configuration (bf16 weights/activations,
# fp32 state): values are rounded to bfloat16 (round-to-nearest-even) where the mixed-precision
# pipeline stores them; every sum stays in float64 here.
# ---------------------------------------------------------------------------------------------


def round_bf16(a: np.ndarray) -> np.ndarray:
    f = np.asarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).astype(F64).reshape(np.shape(a))


def _identity(a):
    return a


# ---------------------------------------------------------------------------------------------
# Model: ReLU MLP classifier with softmax cross-entropy, mean over the minibatch
# (Section II eq.(2); Section III-B eq.(6)).
# ---------------------------------------------------------------------------------------------


@dataclass
class StepTrace:
    """Intermediates of one worker step, kept for tests."""
    loss: float = 0.0
    g: Optional[np.ndarray] = None
    hz: Optional[np.ndarray] = None
    z: Optional[np.ndarray] = None
    pre_acts: List[np.ndarray] = field(default_factory=list)   # s_l, l = 1..L
    min_abs_preact: float = math.inf                           # distance of the closest hidden unit to a ReLU kink
    ties: List[np.ndarray] = field(default_factory=list)       # per hidden layer: bool [B,d_l], |s_l| within the tie band


def forward(theta, x, dims, q: Callable = _identity):
    """Return (list of a_l for l=0..L-1, list of s_l for l=1..L).  q rounds stored activations."""
    layers = unpack(theta, dims)
    L = len(layers)
    a = [q(np.asarray(x, dtype=F64))]
    s = []
    for l in range(1, L + 1):
        W, b = layers[l - 1]
        s_l = a[l - 1] @ q(W).T + b
        s.append(s_l)
        if l < L:
            a.append(q(np.maximum(s_l, 0.0)))
    return a, s


def softmax_rows(s):
    e = np.exp(s - s.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def loss_only(theta, x, y, dims) -> float:
    """Mean softmax cross-entropy of the minibatch (Section III-B eq.(6))."""
    _, s = forward(theta, x, dims)
    sL = s[-1]
    m = sL.max(axis=1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(sL - m).sum(axis=1))
    return float(np.mean(lse - sL[np.arange(len(y)), y]))


def grad_and_hvp(theta, x, y, dims, z=None, q: Callable = _identity, trace: Optional[StepTrace] = None,
                 tie_band: float = 0.0, tie_choice: Optional[Sequence[np.ndarray]] = None):
    """Mean minibatch gradient g (Section II eq.(2)) and, when z is given, the Hessian-vector
    product Hz of the same minibatch loss (the H z of the Hutchinson display, Section IV-B).

    Hz is the derivative of g along the direction z: every quantity X of the forward and
    backward pass gets a companion RX = d/dr X(theta + r z) at r = 0, propagated by the product
    and chain rules.  ReLU contributes its 0/1 slope (slope 0 at exactly 0, curvature 0).

    Ties at the ReLU kink: the gradient of a ReLU network jumps where a pre-activation crosses 0, so
    for a hidden unit with |s| < tie_band * rms(s_l) an implementation in lower precision may
    legitimately land on either side.  Such units are reported in trace.ties, and for them only
    (never for any other unit) the 0/1 slope may be dictated through tie_choice (one bool [B,d_l]
    array per hidden layer).  With tie_band = 0 there are no ties and the slope is [s > 0].
    """
    theta = np.asarray(theta, dtype=F64)
    x = np.asarray(x, dtype=F64)
    B = x.shape[0]
    layers = unpack(theta, dims)
    L = len(layers)
    offs, P = layer_offsets(dims)
    want_h = z is not None
    if want_h:
        zl = unpack(np.asarray(z, dtype=F64), dims)          # (V_l, c_l): z reshaped like theta

    a, s = forward(theta, x, dims, q)
    Wq = [q(W) for (W, _) in layers]
    slope = []                                                 # ReLU slope of hidden layer l = 1..L-1
    ties = []
    for l in range(1, L):
        s_l = s[l - 1]
        on = s_l > 0.0
        tie = np.abs(s_l) < tie_band * math.sqrt(float(np.mean(s_l * s_l))) if tie_band > 0.0 else np.zeros_like(on)
        if tie_choice is not None:
            on = np.where(tie, np.asarray(tie_choice[l - 1], dtype=bool), on)
        slope.append(on)
        ties.append(tie)
    if trace is not None:
        trace.pre_acts = s
        hidden = [np.abs(v).min() for v in s[:-1]]
        trace.min_abs_preact = float(min(hidden)) if hidden else math.inf
        trace.ties = ties

    # R-forward: Ra_0 = 0 (the input does not depend on theta)
    if want_h:
        Ra = [np.zeros_like(a[0])]
        Rs = []
        for l in range(1, L + 1):
            V, c = zl[l - 1]
            Rs_l = Ra[l - 1] @ Wq[l - 1].T + a[l - 1] @ V.T + c
            Rs.append(Rs_l)
            if l < L:
                Ra.append(q(slope[l - 1] * Rs_l))

    # loss and output error
    p = softmax_rows(s[-1])
    onehot = np.zeros_like(p)
    onehot[np.arange(B), y] = 1.0
    loss = float(-np.mean(np.log(p[np.arange(B), y])))
    delta = (p - onehot) / B                                   # d(mean loss)/d s_L
    if want_h:
        RsL = Rs[-1]
        Rp = p * (RsL - (p * RsL).sum(axis=1, keepdims=True))  # derivative of softmax along Rs_L
        Rdelta = Rp / B

    g = np.zeros(P, dtype=F64)
    hz = np.zeros(P, dtype=F64) if want_h else None
    for l in range(L, 0, -1):
        w_off, b_off = offs[l - 1]
        d_out, d_in = dims[l], dims[l - 1]
        dq = q(delta)                                          # back-propagated errors are stored rounded
        g[w_off:b_off] = (dq.T @ a[l - 1]).reshape(-1)
        g[b_off:b_off + d_out] = dq.sum(axis=0)
        if want_h:
            Rdq = q(Rdelta)
            hz[w_off:b_off] = (Rdq.T @ a[l - 1] + dq.T @ Ra[l - 1]).reshape(-1)
            hz[b_off:b_off + d_out] = Rdq.sum(axis=0)
        if l > 1:
            mask = slope[l - 2]
            if want_h:
                V, _ = zl[l - 1]
                Rdelta = (Rdq @ Wq[l - 1] + dq @ V) * mask
            delta = (dq @ Wq[l - 1]) * mask
    if trace is not None:
        trace.loss, trace.g, trace.hz = loss, g, hz
        trace.z = None if z is None else np.asarray(z, dtype=F64)
    return loss, g, hz


# ---------------------------------------------------------------------------------------------
# AdaHessian step (Section IV-B): D = z * Hz (one Hutchinson sample, n = 1 as in Section VII),
# spatial average of D, Adam-like moments with the averaged D in the second moment, update
# theta <- theta - eta * D_t g_t in the sense of eq.(4).
#
# Readings: blocks of `avg_block` consecutive entries along the fan-in axis of each W_l are
# replaced by their (signed) mean; biases are left alone.  Moments are bias-corrected with the
# worker's own step count t >= 1; the denominator is (sqrt(v_hat))**hpow + eps.
# ---------------------------------------------------------------------------------------------


def spatial_average(D: np.ndarray, dims: Optional[Sequence[int]], avg_block: int) -> np.ndarray:
    if avg_block == 1:
        return D.copy()
    out = D.copy()
    if dims is None:                      # flat vector: blocks of consecutive entries
        assert D.size % avg_block == 0
        blk = D.reshape(-1, avg_block).mean(axis=1, keepdims=True)
        return np.broadcast_to(blk, (D.size // avg_block, avg_block)).reshape(-1).copy()
    offs, _ = layer_offsets(dims)
    for l, (w_off, b_off) in enumerate(offs, start=1):
        d_in = dims[l - 1]
        assert d_in % avg_block == 0
        blk = D[w_off:b_off].reshape(-1, avg_block).mean(axis=1, keepdims=True)
        out[w_off:b_off] = np.broadcast_to(blk, (blk.shape[0], avg_block)).reshape(-1)
    return out


def hutchinson_diagonal(zs, hzs) -> np.ndarray:
    """Hutchinson estimate of diag(H) from n probes (Section IV-B): (1/n) sum_j z_j * (H z_j).
    zs, hzs: [n, P] (or [P] for a single probe)."""
    zs = np.atleast_2d(np.asarray(zs, dtype=F64))
    hzs = np.atleast_2d(np.asarray(hzs, dtype=F64))
    return (zs * hzs).sum(axis=0) / zs.shape[0]


def adahessian_update(theta, m, v, g, hz, z, t, *, lr, beta1, beta2, eps, hpow, dims=None, avg_block=1, average=None):
    """One AdaHessian update of (theta, m, v); returns new arrays.  t is the 1-based step count.
    hz, z: one probe ([P]) or n probes ([n, P]) of the same minibatch.
    average: the spatial averaging of another model family (a function of D); default: the MLP's blocks."""
    D = hutchinson_diagonal(z, hz)                         # Hutchinson diagonal estimate (n = 1 in the experiments)
    Ds = average(D) if average is not None else spatial_average(D, dims, avg_block)
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * Ds * Ds
    m_hat = m_new / (1.0 - beta1 ** t)
    v_hat = v_new / (1.0 - beta2 ** t)
    denom = np.power(v_hat, 0.5 * hpow) + eps              # (sqrt(v_hat))**hpow + eps
    theta_new = theta - lr * m_hat / denom
    return theta_new, m_new, v_new


# ---------------------------------------------------------------------------------------------
# First-order worker steps of the baselines the paper compares with (Section VI: EASGD, and EASGD
# with momentum; Section VII: eta = 0.01, momentum delta = 0.5).  They share the elastic pull.
#
# Reading: the paper does not write the momentum step out; it is taken as the classical heavy-ball
# form of the framework it used (velocity b <- delta*b + g, theta <- theta - eta*b, no dampening,
# no Nesterov look-ahead).
# ---------------------------------------------------------------------------------------------


def sgd_update(theta, g, *, lr):
    """Plain stochastic gradient step (Section II eq.(3)): theta <- theta - eta * g."""
    return theta - lr * g


def momentum_update(theta, buf, g, *, lr, momentum):
    """SGD with momentum: b <- delta*b + g, theta <- theta - eta*b.  Returns (theta, b)."""
    buf_new = momentum * buf + g
    return theta - lr * buf_new, buf_new


OPT_ADAHESSIAN, OPT_SGD, OPT_MOMENTUM = 0, 1, 2


# ---------------------------------------------------------------------------------------------
# Dynamic weighting (Section V-B).
# ---------------------------------------------------------------------------------------------

NORM_FLOOR = 1e-30   # reading: u = log||.|| is taken as 0.5*log(max(sum of squares, NORM_FLOOR)), natural log


def log_distance(theta_i, centre) -> float:
    """u = log || theta^i - theta~^m ||_2 (Section V-B, first display)."""
    d = np.asarray(theta_i, dtype=F64) - np.asarray(centre, dtype=F64)
    return 0.5 * math.log(max(float(np.dot(d, d)), NORM_FLOOR))


def raw_score(u_hist: Sequence[float], c: Sequence[float]) -> float:
    """Weighted raw score a_t (Section V-B eq.(10)-(11)).

    u_hist lists u oldest first, newest last (at most p+1 values are used); c[0] weighs the most
    recent difference u_t - u_{t-1}, c[1] the one before it, and so on.  Reading: differences for
    which the history is still too short contribute nothing.
    """
    a = 0.0
    n = len(u_hist)
    for j in range(len(c)):
        hi = n - 1 - j
        lo = hi - 1
        if lo < 0:
            break
        a += c[j] * (u_hist[hi] - u_hist[lo])
    return a


def h1(a: float, alpha: float, kappa: float) -> float:
    """Pull of the master on the worker (Section V-B, first piecewise display; kappa is its k<0)."""
    if a < kappa:
        return 1.0
    if a <= 0.0:
        return 1.0 + (1.0 - alpha) / kappa * (a - kappa)
    return alpha


def h2(a: float, alpha: float, kappa: float) -> float:
    """Pull of the worker on the master (Section V-B, second piecewise display)."""
    if a < kappa:
        return 0.0
    if a <= 0.0:
        return -alpha / kappa * a + alpha
    return alpha


def elastic_sync(thetas: np.ndarray, centre: np.ndarray, h1s, h2s, participate=None):
    """Elastic pull (Section V-B eq.(12)-(13)) for all workers of one communication round.

    Reading for several workers in one round: every difference theta^i - theta^m uses the centre
    as it stood at the start of the round; the centre then moves by the sum of the participating
    workers' h2-weighted differences.  A worker that does not participate keeps its parameters and
    does not move the centre.  Returns (new thetas [k,P], new centre [P]).
    """
    k = thetas.shape[0]
    new_t = thetas.astype(F64).copy()
    new_c = np.asarray(centre, dtype=F64).copy()
    for i in range(k):
        if participate is not None and not participate[i]:
            continue
        d = thetas[i] - centre
        new_t[i] = thetas[i] - h1s[i] * d            # eq.(12)
        new_c += h2s[i] * d                          # eq.(13), accumulated over the round
    return new_t, new_c


def elastic_sync_sequential(thetas: np.ndarray, centre: np.ndarray, h1s, h2s, participate=None):
    """The same round taken as a sequence of single exchanges (Section II: only asynchronous procedures are
    considered; Section VI: a full communication round on one device).

    Reading: the participating workers talk to the master one after the other, in index order; each exchange
    is eq.(12)-(13) exactly as written for one worker, with the centre as the previous exchange left it.
    The weights h1_i, h2_i are those of the round (the raw scores use the master estimate at the start of
    the round).  Returns (new thetas [k,P], new centre [P]).
    """
    k = thetas.shape[0]
    new_t = thetas.astype(F64).copy()
    c = np.asarray(centre, dtype=F64).copy()
    for i in range(k):
        if participate is not None and not participate[i]:
            continue
        d = new_t[i] - c
        new_t[i] = new_t[i] - h1s[i] * d             # eq.(12)
        c = c + h2s[i] * d                           # eq.(13), seen by the next worker of the round
    return new_t, c


MODE_FIXED, MODE_MANUAL, MODE_DYNAMIC = 0, 1, 2


# ---------------------------------------------------------------------------------------------
# The whole path for k simulated workers and one master, mirroring the library's three calls.
# ---------------------------------------------------------------------------------------------


@dataclass
class OracleConfig:
    dims: Optional[Sequence[int]]     # None: flat parameter vector of length n_params (update-only path)
    k: int
    lr: float = 0.01
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-4
    hpow: float = 1.0
    avg_block: int = 1
    alpha: float = 0.1
    kappa: float = -0.1
    c: Sequence[float] = (0.4, 0.3, 0.2, 0.1)
    seed: int = 0
    bf16: bool = False
    n_params: int = 0
    n_samples: int = 1                # Rademacher probes per step (Section IV-B's n)
    optimizer: int = OPT_ADAHESSIAN   # worker step: AdaHessian, or a baseline's SGD / SGD with momentum (Section VI)
    momentum: float = 0.5             # delta of Section VII (OPT_MOMENTUM only; the velocity lives in self.m)


class OracleTrainer:
    """State of master + k workers (each starting as a copy of the master, Section II assumptions)."""

    def __init__(self, cfg: OracleConfig, theta0: np.ndarray):
        self.cfg = cfg
        if cfg.dims is not None:
            _, self.P = layer_offsets(cfg.dims)
        else:
            self.P = cfg.n_params
        assert theta0.shape == (self.P,)
        self.centre = np.asarray(theta0, dtype=F64).copy()
        self.theta = np.tile(self.centre, (cfg.k, 1))
        self.m = np.zeros((cfg.k, self.P), dtype=F64)
        self.v = np.zeros((cfg.k, self.P), dtype=F64)
        self.t = np.zeros(cfg.k, dtype=np.int64)                 # local steps taken per worker
        self.global_step = 0                                      # calls of worker_step
        self.u_hist: List[List[float]] = [[] for _ in range(cfg.k)]
        self.last_a = np.zeros(cfg.k)
        self.last_h1 = np.zeros(cfg.k)
        self.last_h2 = np.zeros(cfg.k)
        self.last_u = np.zeros(cfg.k)
        self.traces: List[Optional[StepTrace]] = [None] * cfg.k
        self.q = round_bf16 if cfg.bf16 else _identity

    def draw_z(self, worker: int, sample: int = 0) -> np.ndarray:
        """Probe `sample` of the worker's next step: stream position t_i * n_samples + sample, so that one
        probe per step (n_samples = 1) is the stream at (seed, i, t_i)."""
        pos = int(self.t[worker]) * self.cfg.n_samples + sample
        words = rademacher_words(self.cfg.seed, worker, pos, self.P)
        return words_to_signs(words, self.P)

    def worker_step(self, x, y, z_signs=None, active=None, tie_band=0.0, tie_choice=None):
        """One local AdaHessian step per active worker.  x: [k,B,d0], y: [k,B] ints.
        z_signs: optional [k,P] of +-1 (else drawn from the counter-based stream at (seed, i, t_i)).
        tie_band / tie_choice[i]: see grad_and_hvp.
        Returns the per-worker mean losses (nan for inactive workers)."""
        cfg = self.cfg
        losses = np.full(cfg.k, np.nan)
        for i in range(cfg.k):
            if active is not None and not active[i]:
                continue
            if cfg.optimizer != OPT_ADAHESSIAN:
                # baseline worker step: the minibatch gradient alone, no Hessian-vector product
                tr = StepTrace()
                loss, g, _ = grad_and_hvp(self.theta[i], x[i], y[i], cfg.dims, None, self.q, tr, tie_band,
                                          None if tie_choice is None else tie_choice[i])
                self.traces[i] = tr
                self.t[i] += 1
                self._first_order(i, g)
                losses[i] = loss
                continue
            if cfg.n_samples == 1:
                z = self.draw_z(i) if z_signs is None else np.asarray(z_signs[i], dtype=F64)
                tr = StepTrace()
                loss, g, hz = grad_and_hvp(self.theta[i], x[i], y[i], cfg.dims, z, self.q, tr, tie_band,
                                           None if tie_choice is None else tie_choice[i])
            else:
                # n probes of the same minibatch: the loss and g do not depend on the probe
                assert z_signs is None, "caller-supplied probes are for n_samples = 1"
                zs, hzs = [], []
                for j in range(cfg.n_samples):
                    zj = self.draw_z(i, j)
                    tr = StepTrace()
                    loss, g, hzj = grad_and_hvp(self.theta[i], x[i], y[i], cfg.dims, zj, self.q, tr, tie_band,
                                                None if tie_choice is None else tie_choice[i])
                    zs.append(zj); hzs.append(hzj)
                z, hz = np.stack(zs), np.stack(hzs)
                tr.hz, tr.z = hz, z
            self.traces[i] = tr
            self.t[i] += 1
            self.theta[i], self.m[i], self.v[i] = adahessian_update(
                self.theta[i], self.m[i], self.v[i], g, hz, z, int(self.t[i]),
                lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, hpow=cfg.hpow,
                dims=cfg.dims, avg_block=cfg.avg_block)
            losses[i] = loss
        self.global_step += 1
        return losses

    def _first_order(self, i, g):
        cfg = self.cfg
        if cfg.optimizer == OPT_SGD:
            self.theta[i] = sgd_update(self.theta[i], g, lr=cfg.lr)
        else:
            self.theta[i], self.m[i] = momentum_update(self.theta[i], self.m[i], g, lr=cfg.lr, momentum=cfg.momentum)

    def update_only(self, g, hz, z_signs=None, active=None):
        """The optimizer part alone on caller-supplied g and Hz ([k,P] each; Hz is not used by the baselines)."""
        cfg = self.cfg
        for i in range(cfg.k):
            if active is not None and not active[i]:
                continue
            if cfg.optimizer != OPT_ADAHESSIAN:
                self.t[i] += 1
                self._first_order(i, np.asarray(g[i], dtype=F64))
                continue
            z = self.draw_z(i) if z_signs is None else np.asarray(z_signs[i], dtype=F64)
            self.t[i] += 1
            self.theta[i], self.m[i], self.v[i] = adahessian_update(
                self.theta[i], self.m[i], self.v[i], np.asarray(g[i], dtype=F64),
                np.asarray(hz[i], dtype=F64), z, int(self.t[i]),
                lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, hpow=cfg.hpow,
                dims=cfg.dims, avg_block=cfg.avg_block)
        self.global_step += 1

    def elastic_sync(self, mode: int, tau: int = 1, h1s=None, h2s=None, participate=None,
                     sequential: bool = False) -> bool:
        """Communication round, taken when the number of worker_step calls is a multiple of tau.

        Every worker (also one whose communication is suppressed) records its log-distance to the
        centre as it stands at the start of the round; the weights then come from the fixed rate
        alpha, from the caller, or from the raw score.  Returns True when a round took place."""
        cfg = self.cfg
        if tau > 1 and self.global_step % tau != 0:
            return False
        p = len(cfg.c)
        H1 = np.zeros(cfg.k)
        H2 = np.zeros(cfg.k)
        for i in range(cfg.k):
            u = log_distance(self.theta[i], self.centre)
            self.u_hist[i].append(u)
            self.u_hist[i] = self.u_hist[i][-(p + 1):]
            a = raw_score(self.u_hist[i], cfg.c)
            self.last_u[i], self.last_a[i] = u, a
            if mode == MODE_FIXED:
                H1[i], H2[i] = cfg.alpha, cfg.alpha
            elif mode == MODE_MANUAL:
                H1[i], H2[i] = h1s[i], h2s[i]
            else:
                H1[i], H2[i] = h1(a, cfg.alpha, cfg.kappa), h2(a, cfg.alpha, cfg.kappa)
        self.last_h1, self.last_h2 = H1, H2
        pull = elastic_sync_sequential if sequential else elastic_sync
        self.theta, self.centre = pull(self.theta, self.centre, H1, H2, participate)
        return True
