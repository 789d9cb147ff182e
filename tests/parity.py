"""Helpers shared by the GPU parity tests: tolerance rule and oracle/GPU construction."""
import numpy as np

from oracle import dw_oracle as O
from paper_2409_09242_amd import binding as B

RTOL_UPDATE = 1e-4      # parameter updates, moments, centre, weights
RTOL_HV = 1e-3          # Hessian-vector products
RTOL_GRAD = 1e-4


OBSERVED = {}            # worst err/bound seen per label, printed by tests for the record
STATS = {}               # per label: entries compared, and how many of them needed the rms floor / an extra allowance
HZ_INPUT_ERR = 5e-5      # allowed fp32 error of an Hz entry relative to the layer's rms when it is propagated
                         # into the update (20 times tighter than the tolerance on Hz itself)


def close(gpu, ref, rtol, what="", extra=None):
    """|gpu - ref| <= rtol * max(|ref|, rms(ref)) element by element.

    The floor rms(ref) is needed because single entries of a gradient or of Hz are sums with
    cancellation: their fp32 rounding error scales with the typical entry, not with the entry itself.
    How the entries pass (on the relative tolerance alone, only thanks to the floor, only thanks to `extra`) is
    counted in STATS.
    """
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    key = what.split("[")[0].split(" ")[-1] + ("/" + what.split("/")[-1] if "/" in what else "")
    if ref.size == 0:
        return
    absref = np.abs(ref)
    scale = float(np.sqrt(np.dot(ref.reshape(-1), ref.reshape(-1)) / ref.size))
    err = np.abs(gpu - ref)
    n_strict = int(np.count_nonzero(err <= rtol * absref + 1e-30))
    floor_bound = rtol * np.maximum(absref, scale) + 1e-30
    if extra is None:
        bound, n_floor_ok = floor_bound, None
    else:
        n_floor_ok = int(np.count_nonzero(err <= floor_bound))
        bound = floor_bound + extra
    ratio = err / bound
    worst = float(ratio.max())                                  # nan if anything is not finite
    OBSERVED[key] = max(OBSERVED.get(key, 0.0), worst)
    if not worst <= 1.0:
        at = int(np.argmax(np.where(np.isfinite(ratio), ratio, np.inf)))
        raise AssertionError("%s: worst at %d: gpu %.9g ref %.9g (err/bound %.3g, rms %.3g)" % (
            what, at, gpu.reshape(-1)[at], ref.reshape(-1)[at], ratio.reshape(-1)[at], scale))
    st = STATS.setdefault(key.split("/")[0], {"n": 0, "floor": 0, "extra": 0})
    st["n"] += int(ref.size)
    if n_floor_ok is None:
        st["floor"] += int(ref.size) - n_strict
    else:
        st["floor"] += n_floor_ok - n_strict; st["extra"] += int(ref.size) - n_floor_ok


def reset():
    OBSERVED.clear(); STATS.clear()


def pass_fractions(prefix=""):
    """{label: (entries, fraction that needed the rms floor, fraction that needed an extra allowance)}."""
    return {k: (v["n"], v["floor"] / max(v["n"], 1), v["extra"] / max(v["n"], 1)) for k, v in STATS.items()
            if k.startswith(prefix) and v["n"]}


def bound_fractions(limits):
    """limits: {label: (largest fraction allowed through the floor, largest through an extra allowance)}; labels not
    compared in this process are skipped.  Prints the record."""
    fr = pass_fractions()
    print("entries passing only by the rms floor / an extra allowance:",
          {k: "%d: %.2e / %.2e" % v for k, v in sorted(fr.items())})
    for k, (fl, ex) in limits.items():
        if k in fr:
            assert fr[k][1] <= fl and fr[k][2] <= ex, (k, fr[k], (fl, ex))


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
             n_params=w.n_params, optimizer=getattr(w, "optimizer", 0), momentum=getattr(w, "momentum", 0.5))
    d.update(kw)
    return O.OracleConfig(**d)


# ---------------------------------------------------------------------------------------------------------
# ReLU pattern of the hidden layers.  The gradient of a ReLU network jumps where a pre-activation crosses zero, so a
# unit whose pre-activation lies within `band * rms(s_l)` of zero in the oracle may land on either side in lower
# precision.  For such tie units, and for no others, the oracle is run under the on/off pattern the library chose; the
# checks here make sure that this is all the library's pattern is used for: ties are rare, every other unit has the
# oracle's own pattern, and the activations themselves agree with the oracle's.
# ---------------------------------------------------------------------------------------------------------
TIE_BAND = 2e-5          # fp32: fraction of the layer's rms below which a pre-activation counts as a tie
TIE_BAND_BF16 = 1e-2     # bf16: upstream rounding flips move a pre-activation by up to 2e-3 of the layer's rms
MAX_TIE_FRACTION = 1e-4          # of the hidden units compared (a Gaussian layer has 1.6e-5 of them inside the fp32 band)
MAX_TIE_FRACTION_BF16 = 1.5e-2   # (0.8e-2 inside the bf16 band)
TIES = {"units": 0, "ties": 0, "choice_used": 0}


def gpu_hidden(h, w, workers=None):
    """Hidden activations of the last step as float64 arrays [B, d_l], per worker and hidden layer."""
    L = len(w.dims) - 1
    out = {}
    for i in (range(w.k) if workers is None else workers):
        per = []
        for l in range(1, L):
            a = h.get_state(B.DW_S_ACT + l, i)
            if a.dtype == np.uint16:
                a = (a.astype(np.uint32) << 16).view(np.float32)
            per.append(a.astype(np.float64))
        out[i] = per
    return out


def slopes_of(hidden):
    return {i: [a > 0 for a in per] for i, per in hidden.items()}


def check_hidden(hidden, traces, bf16, what=""):
    """hidden: gpu_hidden(...) of the step; traces: {worker: StepTrace of the oracle's step (run with the tie band)}."""
    for i, per in hidden.items():
        trc = traces[i]
        if trc is None:
            continue
        for l, a_gpu in enumerate(per):
            s = trc.pre_acts[l]
            tie = trc.ties[l] if trc.ties else np.zeros(s.shape, dtype=bool)
            on_ref = s > 0
            on_gpu = a_gpu > 0
            differ = on_gpu != on_ref
            assert not np.any(differ & ~tie), "%s worker %d layer %d: %d units outside the tie band differ" % (
                what, i, l + 1, int((differ & ~tie).sum()))
            TIES["units"] += s.size; TIES["ties"] += int(tie.sum()); TIES["choice_used"] += int(differ.sum())
            a_ref = np.maximum(s, 0.0)
            rms = float(np.sqrt(np.mean(a_ref ** 2)))
            if bf16:
                a_ref = O.round_bf16(a_ref)
                # stored values agree to one bf16 step (2^-8 relative, the next power of two up: 2^-7) on top of what
                # upstream rounding flips move the pre-activation by; in norm the flips average out
                err = np.abs(a_gpu - a_ref)
                assert np.all(err <= 2.0 ** -7 * np.abs(a_ref) + 1e-2 * rms), (what, i, l, float(err.max()), rms)
                rel = np.linalg.norm(a_gpu - a_ref) / max(np.linalg.norm(a_ref), 1e-300)
                OBSERVED["norm act"] = max(OBSERVED.get("norm act", 0.0), rel / 2e-3)
                assert rel <= 2e-3, (what, i, l, rel)
            else:
                close(a_gpu, a_ref, RTOL_GRAD, "%s act[%d]/a%d" % (what, i, l + 1))


def bound_ties(bf16):
    frac = TIES["ties"] / max(TIES["units"], 1)
    print("hidden units compared %d, inside the tie band %d (%.2e), of which the library chose the other side %d" % (
        TIES["units"], TIES["ties"], frac, TIES["choice_used"]))
    limit = MAX_TIE_FRACTION_BF16 if bf16 else MAX_TIE_FRACTION
    assert TIES["ties"] <= limit * TIES["units"] + 3, (TIES, limit)        # + 3: layers of a few hundred units
    for k_ in TIES:
        TIES[k_] = 0
