"""Helpers shared by the GPU parity tests: tolerance rule and oracle/GPU construction."""
import numpy as np

from oracle import dw_oracle as O
from paper_2409_09242_amd import binding as B

RTOL_UPDATE = 1e-4      # parameter updates, moments, centre, weights
RTOL_HV = 1e-3          # Hessian-vector products
RTOL_GRAD = 1e-4


OBSERVED = {}            # worst err/bound seen per label, printed by tests for the record
HZ_INPUT_ERR = 5e-5      # allowed fp32 error of an Hz entry relative to the layer's rms when it is propagated
                         # into the update (20 times tighter than the tolerance on Hz itself)


def close(gpu, ref, rtol, what="", extra=None):
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
    if extra is not None:
        bound = bound + extra
    err = np.abs(gpu - ref)
    key = what.split("[")[0].split(" ")[-1] + ("/" + what.split("/")[-1] if "/" in what else "")
    OBSERVED[key] = max(OBSERVED.get(key, 0.0), float((err / bound).max()) if ref.size else 0.0)
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


G_INPUT_ERR = 2e-5       # same for an entry of g (5 times tighter than the tolerance on g itself)


def close_update(gpu_upd, ref_upd, tr, i, dims, rtol, what):
    """Parameter update of worker i after a network step.

    The step eta*m_hat/(sqrt(v_hat)^hpow + eps) divides by a quantity built from D = z*Hz.  Entries whose
    denominator is far below the layer's typical |Hz| (or whose numerator error meets a small denominator)
    amplify the fp32 rounding of Hz and g, which is relative to the layer's typical entry, not to the entry
    itself.  First-order propagation gives the extra allowance
        |update| * HZ_INPUT_ERR * rms(Hz) / denom  +  eta * (1-beta1)/(1-beta1^t) * G_INPUT_ERR * rms(g) / denom;
    the GPU also stores theta in fp32, so an update read back as a difference of two stored values carries
    one ulp of theta (2^-23 |theta|).  Everything else must hold to rtol.
    """
    cfg = tr.cfg
    t = int(tr.t[i])
    v_hat = tr.v[i] / (1.0 - cfg.beta2 ** t)
    denom = np.power(v_hat, 0.5 * cfg.hpow) + cfg.eps
    hz, g = tr.traces[i].hz, tr.traces[i].g
    for name, sl in per_layer(dims):
        rms_hz = float(np.sqrt(np.mean(hz[sl] ** 2)))
        rms_g = float(np.sqrt(np.mean(g[sl] ** 2)))
        extra = (np.abs(ref_upd[sl]) * HZ_INPUT_ERR * rms_hz
                 + cfg.lr * (1.0 - cfg.beta1) / (1.0 - cfg.beta1 ** t) * G_INPUT_ERR * rms_g) / denom[sl]
        extra = extra + 2.0 ** -23 * np.abs(tr.theta[i][sl])
        close(gpu_upd[sl], ref_upd[sl], rtol, "%s/%s" % (what, name), extra=extra)


def oracle_config(w, **kw):
    d = dict(dims=w.dims, k=w.k, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, hpow=w.hpow,
             avg_block=w.avg_block, alpha=w.alpha, kappa=w.kappa, c=w.c, seed=w.seed, bf16=w.bf16,
             n_params=w.n_params)
    d.update(kw)
    return O.OracleConfig(**d)
