"""Helpers shared by the GPU parity tests: tolerance rule and oracle/GPU construction."""
import numpy as np

from oracle import dw_oracle as O
from paper_2409_09242_amd import binding as B

RTOL_UPDATE = 1e-4      # parameter updates, moments, centre, weights
RTOL_HV = 1e-3          # Hessian-vector products
RTOL_GRAD = 1e-4


def close(gpu, ref, rtol, what=""):
    """|gpu - ref| <= rtol * max(|ref|, rms(ref)) element by element.

    The floor rms(ref) is needed because single entries of a gradient or of Hz are sums with
    cancellation: their fp32 rounding error scales with the typical entry, not with the entry itself.
    """
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu)), what
    scale = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    bound = rtol * np.maximum(np.abs(ref), scale) + 1e-30
    err = np.abs(gpu - ref)
    worst = int(np.argmax(err / bound)) if ref.size else 0
    assert np.all(err <= bound), "%s: worst at %d: gpu %.9g ref %.9g (err/bound %.3g, rms %.3g)" % (
        what, worst, gpu.reshape(-1)[worst], ref.reshape(-1)[worst], (err / bound).reshape(-1)[worst], scale)


def per_layer(dims):
    offs, P = O.layer_offsets(dims)
    out = []
    for l, (w, b) in enumerate(offs, start=1):
        out.append(("W%d" % l, slice(w, b)))
        out.append(("b%d" % l, slice(b, b + dims[l])))
    return out


def close_layers(gpu, ref, dims, rtol, what):
    for name, sl in per_layer(dims):
        close(gpu[sl], ref[sl], rtol, "%s/%s" % (what, name))


def oracle_config(w, **kw):
    d = dict(dims=w.dims, k=w.k, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, hpow=w.hpow,
             avg_block=w.avg_block, alpha=w.alpha, kappa=w.kappa, c=w.c, seed=w.seed, bf16=w.bf16,
             n_params=w.n_params)
    d.update(kw)
    return O.OracleConfig(**d)
