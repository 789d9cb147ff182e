"""Seeded synthetic inputs and the benchmark configurations.

This module serves both the CPU oracle's tests and the GPU library's tests/bench.  It holds no
arithmetic of the method itself: only shapes, hyper-parameters, random inputs, teacher labels and
the host-side communication schedules (which workers are suppressed in which round).

The paper trains on MNIST (Section VI); that data is not available here, so inputs are seeded
synthetic stand-ins with the same shapes and value ranges (784 features in [0,1], 10 classes).
Hyper-parameters follow Section VII: eta = 0.01, beta = (0.9, 0.999), one Hutchinson sample,
alpha = 0.1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    k: int                                  # number of worker replicas
    dims: Optional[Tuple[int, ...]]         # MLP layer widths d_0..d_L; None for the flat update-only case
    batch: int
    tau: int                                # communication period (Section VI footnote)
    input_dist: str                         # "normal" | "uniform01"
    teacher: str                            # "linear" | "mlp2"
    bf16: bool = False
    n_params: int = 0                       # flat case only
    steps: int = 20
    stale: str = "none"                     # "none" | "fixed3_last2" | "geometric0.3" | "third"
    lr: float = 0.01
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-4
    hpow: float = 1.0
    avg_block: int = 1
    alpha: float = 0.1
    kappa: float = -0.1
    c: Tuple[float, ...] = (0.4, 0.3, 0.2, 0.1)
    seed: int = 20240909
    img: Optional[Tuple[int, int, int]] = None   # convolutional front end: input image (H, W, C), channels last
    conv: Tuple[int, ...] = ()               # output channels of its 3x3 convolutions (dims[0] = the pooled, flattened map)
    conv_avg: int = 0                        # 3x3 window averaging of the Hutchinson estimate
    optimizer: int = 0                       # 0 AdaHessian; 1 SGD, 2 SGD with momentum (the baselines of Section VI)
    momentum: float = 0.5                    # Section VII

    @property
    def P(self) -> int:
        if self.dims is None:
            return self.n_params
        conv = sum(co * ((9 * ci + 3) // 4 * 4) + co for (_, ci, co) in self.conv_stages())   # rows padded to 4
        return conv + sum(self.dims[l] * self.dims[l - 1] + self.dims[l] for l in range(1, len(self.dims)))

    def conv_stages(self):
        """(output positions per sample, input channels, output channels) of every convolution."""
        out = []
        if self.conv:
            h, w, c = self.img
            for co in self.conv:
                h, w = h - 2, w - 2
                out.append((h * w, c, co))
                c = co
        return out

    def gemm_flops_by_class(self):
        """Multiply-add work (flop) of one worker step per GEMM class.  A layer costs 2 (rows)(fan-in)(fan-out) per
        product: forward 3 products (2 when its input does not depend on the parameters), weight gradient the same,
        data gradient 3 (none for the first layer of the model)."""
        layers = [(self.batch * pos, 9 * ci, co) for (pos, ci, co) in self.conv_stages()]
        layers += [(self.batch, self.dims[l - 1], self.dims[l]) for l in range(1, len(self.dims))]
        fwd = sum(2.0 * m * fi * fo * (3 if n > 0 else 2) for n, (m, fi, fo) in enumerate(layers))
        dgrad = sum(2.0 * m * fi * fo * 3 for n, (m, fi, fo) in enumerate(layers) if n > 0)
        return {"gemm_fwd": fwd, "gemm_wgrad": fwd, "gemm_dgrad": dgrad}

    def flops_per_worker_step(self) -> float:
        """Multiply-add work of one worker step including the Hessian-vector product:
        first layer 4 products (forward, V-term, weight-grad, Hz weight-grad), every later layer 9."""
        return sum(self.gemm_flops_by_class().values())


C1 = Workload("c1_tiny", k=4, dims=(32, 64, 10), batch=16, tau=1, input_dist="normal", teacher="linear",
              steps=20, seed=20240909 + 1)
C2 = Workload("c2_mnist_mlp", k=4, dims=(784, 512, 512, 10), batch=128, tau=4, input_dist="uniform01",
              teacher="mlp2", steps=16, seed=20240909 + 2)
C3 = Workload("c3_cifar_mlp", k=8, dims=(3072, 1024, 1024, 1024, 10), batch=256, tau=8, input_dist="normal",
              teacher="mlp2", steps=64, stale="fixed3_last2", seed=20240909 + 3)
C4 = Workload("c4_wide_bf16", k=16, dims=(4096, 4096, 4096, 4096, 10), batch=512, tau=4, input_dist="normal",
              teacher="mlp2", bf16=True, steps=8, stale="geometric0.3", seed=20240909 + 4)
# the model of the paper's experiments (Section VI: a small 2-convolution CNN on 28 x 28 images, k in {4, 8}), inputs
# U[0,1] shaped like its data set, batch 64, communication period 1, one third of the communications suppressed
CNN = Workload("cnn_paper_model", k=8, dims=(9216, 128, 10), batch=64, tau=1, input_dist="uniform01", teacher="mlp2",
               steps=8, stale="third", seed=20240909 + 6, img=(28, 28, 1), conv=(32, 64), conv_avg=1)
C5 = Workload("c5_update_only", k=16, dims=None, batch=0, tau=1, input_dist="normal", teacher="none",
              n_params=100_000_000, steps=20, seed=20240909 + 5)

WORKLOADS = {w.name.split("_")[0]: w for w in (C1, C2, C3, C4, C5, CNN)}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (used for reduced-size parity cases)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


def rng_for(seed: int, stream: int) -> np.random.Generator:
    """Counter-based generator keyed by (seed, stream): independent streams for theta, x, labels, ..."""
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def init_theta(dims: Sequence[int], seed: int) -> np.ndarray:
    """theta_0 ~ U(-1/sqrt(fan_in), 1/sqrt(fan_in)) per layer, float32, canonical flat layout."""
    rng = rng_for(seed, 11)
    parts = []
    for l in range(1, len(dims)):
        bound = 1.0 / np.sqrt(dims[l - 1])
        parts.append(rng.uniform(-bound, bound, size=dims[l] * dims[l - 1]))
        parts.append(rng.uniform(-bound, bound, size=dims[l]))
    return np.concatenate(parts).astype(np.float32)


def init_theta_workload(w: Workload) -> np.ndarray:
    """theta_0 of a workload in the library's layout: as init_theta, with the kernels of a convolutional front end
    first (rows padded with zeros to a multiple of 4 entries)."""
    if not w.conv:
        return init_theta(w.dims, w.seed)
    rng = rng_for(w.seed, 11)
    parts = []
    for (_, ci, co) in w.conv_stages():
        K = (9 * ci + 3) // 4 * 4
        bound = 1.0 / np.sqrt(9 * ci)
        kern = np.zeros((co, K))
        kern[:, :9 * ci] = rng.uniform(-bound, bound, size=(co, 9 * ci))
        parts.append(kern.reshape(-1))
        parts.append(rng.uniform(-bound, bound, size=co))
    for l in range(1, len(w.dims)):
        bound = 1.0 / np.sqrt(w.dims[l - 1])
        parts.append(rng.uniform(-bound, bound, size=w.dims[l] * w.dims[l - 1]))
        parts.append(rng.uniform(-bound, bound, size=w.dims[l]))
    return np.concatenate(parts).astype(np.float32)


def _teacher_labels(x: np.ndarray, kind: str, n_classes: int, seed: int) -> np.ndarray:
    rng = rng_for(seed, 13)
    d0 = x.shape[-1]
    if kind == "linear":
        T = rng.standard_normal((n_classes, d0))
        logits = x @ T.T
    else:
        T1 = rng.standard_normal((32, d0)) / np.sqrt(d0)
        T2 = rng.standard_normal((n_classes, 32)) / np.sqrt(32)
        logits = np.maximum(x @ T1.T, 0.0) @ T2.T
    return np.argmax(logits, axis=-1).astype(np.int32)


def minibatch_pool(w: Workload, n_batches: int, bf16_round=None) -> Tuple[np.ndarray, np.ndarray]:
    """A pool of minibatches: x [n_batches, k, B, d0] float32, y [n_batches, k, B] int32."""
    rng = rng_for(w.seed, 17)
    shape = (n_batches, w.k, w.batch) + (tuple(w.img) if w.conv else (w.dims[0],))
    if w.input_dist == "uniform01":
        x = rng.random(shape, dtype=np.float32)
    else:
        x = rng.standard_normal(shape, dtype=np.float32)
    if bf16_round is not None:
        x = bf16_round(x)
    y = _teacher_labels(x.reshape(shape[:3] + (-1,)).astype(np.float64), w.teacher, w.dims[-1], w.seed)
    return x.astype(np.float32), y


def to_bf16_f32(a: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest-even) and return them as float32 (input prep only)."""
    u = np.asarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(a))


def participation_schedule(w: Workload, n_rounds: int) -> np.ndarray:
    """[n_rounds, k] uint8: 1 where worker i communicates with the master in that round.

    The paper forces failure by suppressing a worker's communication (Section VI).  Here:
      "fixed3_last2":  the last two workers are absent for 3 rounds and present in the 4th, forever;
      "geometric0.3":  after each participation a worker draws s ~ Geometric(0.3) on {0,1,2,...}
                       and is absent for the next s rounds.
      "third":         every worker's communication is suppressed in a round with probability 1/3,
                       independently (the suppression rate of Section VI).
    Suppressed workers keep taking local steps.
    """
    part = np.ones((n_rounds, w.k), dtype=np.uint8)
    if w.stale == "fixed3_last2":
        for i in (w.k - 2, w.k - 1):
            for r in range(n_rounds):
                part[r, i] = 1 if (r % 4) == 3 else 0
    elif w.stale == "geometric0.3":
        rng = rng_for(w.seed, 19)
        for i in range(w.k):
            r = 0
            while r < n_rounds:
                s = int(rng.geometric(0.3)) - 1
                part[r:r + s, i] = 0
                r += s + 1
    elif w.stale == "third":
        rng = rng_for(w.seed, 23)
        part = (rng.random((n_rounds, w.k)) >= 1.0 / 3.0).astype(np.uint8)
    return part
