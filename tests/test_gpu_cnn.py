"""GPU parity of the convolutional model (Section VI) against the oracle: loss, gradient, Hessian-vector product
and the AdaHessian update with and without the 3x3 window averaging (Section IV-B); called through the C ABI."""
import functools

import numpy as np
import pytest
import torch

from oracle import dw_cnn as OC
from oracle import dw_oracle as O
from paper_2409_09242_amd import binding as B
from paper_2409_09242_amd import workloads as W
from parity import close, RTOL_GRAD, RTOL_HV, RTOL_UPDATE

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SPECS = {
    "two_conv": (OC.CnnSpec(img=(10, 10, 1), conv=(4, 8), fc=(16, 10)), 6, 3),
    "one_conv_rgb": (OC.CnnSpec(img=(12, 8, 3), conv=(8,), fc=(12, 5)), 5, 2),
    "paper_shape": (OC.CnnSpec(img=(28, 28, 1), conv=(32, 64), fc=(128, 10)), 16, 2),
    # maps that are not square and channel counts that are not powers of two (the second convolution reads its patches
    # in place and takes its data gradient as a sum over taps)
    "two_conv_odd": (OC.CnnSpec(img=(14, 12, 2), conv=(12, 20), fc=(24, 7)), 5, 2),
}


@functools.lru_cache(maxsize=None)
def _inputs(spec, batch, k, seed):
    """theta_0 (unpadded layout), minibatches and labels; the seed is advanced until every worker's first step is
    clear of ReLU and pooling kinks by more than fp32 rounding (fp32 and fp64 must take the same branches; with
    hundreds of thousands of pre-activations the closest one is never far from zero, so the bar scales down
    with the size)."""
    offs, P = spec.offsets()
    for s in range(seed, seed + 50):
        rng = W.rng_for(s, 3)
        theta = np.zeros(P)
        for (w, b, shape) in offs:
            fan_in = int(np.prod(shape[1:]))
            theta[w:b] = rng.uniform(-1, 1, size=b - w) / np.sqrt(fan_in)
            theta[b:b + shape[0]] = rng.uniform(-1, 1, size=shape[0]) / np.sqrt(fan_in)
        theta = theta.astype(np.float32).astype(np.float64)
        x = rng.uniform(0, 1, size=(k, batch) + spec.img).astype(np.float32)
        y = rng.integers(0, spec.fc[-1], size=(k, batch)).astype(np.int32)
        margins = [OC.grad_and_hvp(theta, x[i], y[i], spec)[3] for i in range(k)]
        if min(margins) > (1e-5 if P < 100000 else 3e-7):
            return theta, x, y
    raise AssertionError("no kink-free inputs found")


def _layers(spec):
    offs, _ = spec.offsets()
    out = []
    for n, (w, b, shape) in enumerate(offs):
        out.append(("W%d" % n, slice(w, b)))
        out.append(("b%d" % n, slice(b, b + shape[0])))
    return out


def _signs(bits, P_lib):
    return np.where((bits[np.arange(P_lib) >> 5] >> (np.arange(P_lib) & 31)) & 1, 1.0, -1.0)


@pytest.mark.parametrize("name", list(SPECS))
@pytest.mark.parametrize("conv_avg", [0, 1])
def test_cnn_step_matches_the_oracle(name, conv_avg):
    spec, batch, k = SPECS[name]
    print("cnn", name, "conv_avg", conv_avg, flush=True)
    theta0, x, y = _inputs(spec, batch, k, 100)
    idx, P_lib = B.conv_param_index(spec.img, spec.conv, spec.fc)
    cfg = B.make_config(dims=(spec.flat,) + spec.fc, k=k, batch=batch, img=spec.img, conv=spec.conv,
                        conv_avg=conv_avg, seed=77, lr=0.01, eps=1e-4)
    assert B.param_count(cfg) == P_lib
    th_lib = np.zeros(P_lib, dtype=np.float32); th_lib[idx] = theta0
    h = B.Handle(cfg, th_lib, DEV)
    loss = torch.zeros(k, device=DEV)
    active = None if name != "two_conv" else [1, 0, 1]
    h.worker_step(torch.from_numpy(x).to(DEV), torch.from_numpy(y).to(DEV), loss=loss, active=active)
    torch.cuda.synchronize()
    pad = np.ones(P_lib, dtype=bool); pad[idx] = False
    for i in range(k):
        th = h.get_state(B.DW_S_THETA, i)
        if active is not None and not active[i]:
            np.testing.assert_array_equal(th, th_lib)
            assert int(h.get_state(B.DW_S_STEPS, i)[0]) == 0
            continue
        z = _signs(h.get_state(B.DW_S_ZBITS, i), P_lib)[idx]
        ref_loss, g, hz, margin = OC.grad_and_hvp(theta0, x[i], y[i], spec, z)
        assert abs(loss[i].item() - ref_loss) <= 1e-5 * abs(ref_loss)
        gg, gh = h.get_state(B.DW_S_G, i), h.get_state(B.DW_S_HZ, i)
        assert not gg[pad].any() and not th[pad].any()              # padding entries never move
        if not conv_avg:
            assert not gh[pad].any()
        for lname, sl in _layers(spec):
            close(gg[idx][sl], g[sl], RTOL_GRAD, "cnn g[%s]/%s" % (name, lname))
            if not conv_avg:                                         # with averaging Hz of the kernels is rewritten in place
                close(gh[idx][sl], hz[sl], RTOL_HV, "cnn hz[%s]/%s" % (name, lname))
        # the update, from the GPU's own g and Hz (so that only the optimizer arithmetic is compared here) ...
        hz_in = gh[idx].astype(np.float64) if not conv_avg else None
        avg = (lambda D: OC.spatial_average(D, spec)) if conv_avg else (lambda D: D)
        if conv_avg:
            # ... with averaging the GPU's Hz buffer holds z * mean(z * Hz): the mean of the oracle's D must equal z * it
            Dbar = OC.spatial_average(z * hz, spec)
            for lname, sl in _layers(spec):
                close(z[sl] * gh[idx][sl], Dbar[sl], RTOL_HV, "cnn Dbar[%s]/%s" % (name, lname))
            hz_in = gh[idx].astype(np.float64)
            avg = lambda D: D
        t_new, m_new, v_new = O.adahessian_update(theta0, np.zeros_like(theta0), np.zeros_like(theta0),
                                                  gg[idx].astype(np.float64), hz_in, z, 1, lr=0.01, beta1=0.9,
                                                  beta2=0.999, eps=1e-4, hpow=1.0, average=avg)
        close(h.get_state(B.DW_S_M, i)[idx], m_new, RTOL_UPDATE, "cnn m[%s]" % name)
        close(h.get_state(B.DW_S_V, i)[idx], v_new, RTOL_UPDATE, "cnn v[%s]" % name)
        close(th[idx] - theta0, t_new - theta0, RTOL_UPDATE, "cnn update[%s]" % name,
              extra=2.0 ** -23 * np.abs(theta0))
    # a communication round works on the padded vectors as on any other
    assert h.elastic_sync(B.DW_DYNAMIC, tau=1)
    c = h.get_state(B.DW_S_CENTRE)
    assert not c[pad].any() and np.all(np.isfinite(c))
    h.close()


def test_cnn_configuration_errors():
    import ctypes as C
    n = C.c_int64()
    ok = dict(dims=(72, 16, 10), k=2, batch=4, img=(10, 10, 1), conv=(4, 8))
    assert B.lib().dw_param_count(C.byref(B.make_config(**ok)), C.byref(n)) == 0
    bad = [dict(ok, dims=(64, 16, 10)),                 # flatten size does not match
           dict(ok, conv=(4, 6)),                       # channels not a multiple of 4
           dict(ok, img=(9, 10, 1)),                    # odd map before the pooling
           dict(ok, bf16=True), dict(ok, fuse_update=1), dict(ok, conv_avg=2)]
    for kw in bad:
        assert B.lib().dw_param_count(C.byref(B.make_config(**kw)), C.byref(n)) == -2, kw
    assert B.lib().dw_param_count(C.byref(B.make_config(**dict(ok, avg_block=2))), C.byref(n)) == -3


def test_cnn_steps_and_rounds_follow_the_oracle():
    """Three local steps with a dynamic-weighted round after each (one worker's communication suppressed once):
    the oracle side is its flat trainer fed with the convolutional oracle's g and Hz."""
    spec, batch, k = SPECS["two_conv"]
    theta0, _, _ = _inputs(spec, batch, k, 100)
    offs, P = spec.offsets()
    idx, P_lib = B.conv_param_index(spec.img, spec.conv, spec.fc)
    cfg = B.make_config(dims=(spec.flat,) + spec.fc, k=k, batch=batch, img=spec.img, conv=spec.conv, conv_avg=1,
                        seed=5, lr=0.01, eps=1e-4)
    th_lib = np.zeros(P_lib, dtype=np.float32); th_lib[idx] = theta0
    h = B.Handle(cfg, th_lib, DEV)
    tr = O.OracleTrainer(O.OracleConfig(dims=None, k=k, n_params=P, lr=0.01, eps=1e-4, seed=5), theta0.copy())
    rng = W.rng_for(26, 1)       # a data seed under which no pre-activation of the three steps comes within 2e-5 of a kink
    for step in range(3):
        x = rng.uniform(0, 1, size=(k, batch) + spec.img).astype(np.float32)
        y = rng.integers(0, spec.fc[-1], size=(k, batch)).astype(np.int32)
        h.worker_step(torch.from_numpy(x).to(DEV), torch.from_numpy(y).to(DEV))
        g_all, hz_all, z_all = [], [], []
        for i in range(k):
            z = _signs(h.get_state(B.DW_S_ZBITS, i), P_lib)[idx]
            _, g, hz, margin = OC.grad_and_hvp(tr.theta[i], x[i], y[i], spec, z)
            assert margin > 1e-6
            g_all.append(g); hz_all.append(z * OC.spatial_average(z * hz, spec)); z_all.append(z)
        tr.update_only(np.stack(g_all), np.stack(hz_all), z_signs=np.stack(z_all))
        part = [1, 0, 1] if step == 1 else None
        assert h.elastic_sync(B.DW_DYNAMIC, tau=1, participate=part)
        assert tr.elastic_sync(O.MODE_DYNAMIC, tau=1, participate=part)
    for i in range(k):
        th = h.get_state(B.DW_S_THETA, i)[idx]
        assert np.linalg.norm(th - tr.theta[i]) <= 2e-3 * np.linalg.norm(tr.theta[i] - theta0), i
        sc = h.get_state(B.DW_S_SCORE, i)
        # free-running: u is the log of a distance that carries the steps' rounding, a a difference of such logs,
        # h1 and h2 a (1-alpha)/|kappa| = 9 times amplified function of a (the end-to-end bounds of the MLP tests)
        want = [tr.last_u[i], tr.last_a[i], tr.last_h1[i], tr.last_h2[i]]
        assert abs(sc[0] - want[0]) <= 5e-4 and abs(sc[1] - want[1]) <= 1e-3, (sc, want)
        np.testing.assert_allclose(sc[2:], want[2:], rtol=5e-3)
    c = h.get_state(B.DW_S_CENTRE)[idx]
    assert np.linalg.norm(c - tr.centre) <= 2e-3 * np.linalg.norm(tr.centre - theta0)
    h.close()


def test_cnn_step_with_two_hutchinson_probes_follows_the_oracle():
    """n = 2 probes of the same minibatch through the convolutional model: D is the mean over the probes of the
    window-averaged z_j * Hz_j (the averaging is linear, so it can be taken per probe), then one update and a round."""
    spec, batch, k = SPECS["two_conv"]
    theta0, _, _ = _inputs(spec, batch, k, 100)
    offs, P = spec.offsets()
    idx, P_lib = B.conv_param_index(spec.img, spec.conv, spec.fc)
    n, seed = 2, 11
    cfg = B.make_config(dims=(spec.flat,) + spec.fc, k=k, batch=batch, img=spec.img, conv=spec.conv, conv_avg=1,
                        seed=seed, lr=0.01, eps=1e-4, n_samples=n)
    th_lib = np.zeros(P_lib, dtype=np.float32); th_lib[idx] = theta0
    h = B.Handle(cfg, th_lib, DEV)
    tr = O.OracleTrainer(O.OracleConfig(dims=None, k=k, n_params=P, lr=0.01, eps=1e-4, seed=seed), theta0.copy())
    rng = W.rng_for(26, 1)
    for step in range(2):
        x = rng.uniform(0, 1, size=(k, batch) + spec.img).astype(np.float32)
        y = rng.integers(0, spec.fc[-1], size=(k, batch)).astype(np.int32)
        h.worker_step(torch.from_numpy(x).to(DEV), torch.from_numpy(y).to(DEV))
        g_all, d_all = [], []
        for i in range(k):
            D = np.zeros(P)
            for j in range(n):
                # probe j of the worker's step t sits at position t*n + j of its stream (library index space)
                z = O.words_to_signs(O.rademacher_words(seed, i, step * n + j, P_lib), P_lib)[idx]
                _, g, hz, margin = OC.grad_and_hvp(tr.theta[i], x[i], y[i], spec, z)
                assert margin > 1e-6
                D += OC.spatial_average(z * hz, spec) / n
            np.testing.assert_array_equal(_signs(h.get_state(B.DW_S_ZBITS, i), P_lib)[idx], z)   # the last probe's bits
            g_all.append(g); d_all.append(D)
        tr.update_only(np.stack(g_all), np.stack(d_all), z_signs=np.ones((k, P)))
        assert h.elastic_sync(B.DW_DYNAMIC, tau=1) and tr.elastic_sync(O.MODE_DYNAMIC, tau=1)
    for i in range(k):
        th = h.get_state(B.DW_S_THETA, i)[idx]
        assert np.linalg.norm(th - tr.theta[i]) <= 2e-3 * np.linalg.norm(tr.theta[i] - theta0), i
        sc = h.get_state(B.DW_S_SCORE, i)
        assert abs(sc[0] - tr.last_u[i]) <= 5e-4 and abs(sc[1] - tr.last_a[i]) <= 1e-3, (sc, tr.last_u[i], tr.last_a[i])
    h.close()
