"""Pins for the oracle's AdaHessian update, Rademacher stream, dynamic weights and elastic pull.

Section IV-B (Hutchinson / spatial averaging / Adam-like moments), Section V-B (u, a, h1, h2,
eq.(10)-(13)), Section IV-A (EASGD, eq.(8)-(9) read with the signs of eq.(12)-(13)).
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import dw_oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


# ------------------------------------------------------------------ Rademacher stream
def test_splitmix_reference_outputs():
    want = [int(l, 16) for l in open(os.path.join(HERE, "golden", "splitmix64_seed0.txt"))
            if not l.startswith("#") and l.strip()]
    got = O.splitmix_stream(0, len(want))
    assert [int(v) for v in got] == want


def test_rademacher_words_vectorised_equals_scalar_stream_and_is_balanced():
    P = 100_003
    w = O.rademacher_words(42, 3, 7, P)
    key = O.rademacher_key(42, 3, 7)
    np.testing.assert_array_equal(w[:50], O.splitmix_stream(key, 50))
    z = O.words_to_signs(w, P)
    assert set(np.unique(z)) == {-1.0, 1.0}
    assert abs(z.mean()) < 4.0 / math.sqrt(P)
    # different (worker, step) give different, uncorrelated streams
    z2 = O.words_to_signs(O.rademacher_words(42, 3, 8, P), P)
    z3 = O.words_to_signs(O.rademacher_words(42, 4, 7, P), P)
    assert abs((z * z2).mean()) < 4.0 / math.sqrt(P) and abs((z * z3).mean()) < 4.0 / math.sqrt(P)
    # bit order: element j is bit (j mod 64) of word j // 64; the 32-bit view is low half first
    j = 64 * 5 + 37
    assert z[j] == (1.0 if (int(w[5]) >> 37) & 1 else -1.0)
    u32 = O.words_to_u32(w)
    assert (int(u32[11]) >> 5) & 1 == (int(w[5]) >> 37) & 1


# ------------------------------------------------------------------ AdaHessian update
HP = dict(lr=0.01, beta1=0.9, beta2=0.999, eps=1e-4, hpow=1.0)


def test_update_reduces_to_torch_adam_when_hz_is_z_times_g():
    """With Hz := z*g the Hutchinson estimate z*Hz equals g, so the second moment is Adam's and the
    whole step must coincide with the library's Adam (no block averaging, Hessian power 1)."""
    rng = np.random.default_rng(0)
    P = 257
    theta0 = rng.standard_normal(P)
    p = torch.nn.Parameter(torch.tensor(theta0))
    opt = torch.optim.Adam([p], lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"])
    theta, m, v = theta0.copy(), np.zeros(P), np.zeros(P)
    for t in range(1, 8):
        g = rng.standard_normal(P) * 0.1
        z = rng.choice([-1.0, 1.0], size=P)
        theta, m, v = O.adahessian_update(theta, m, v, g, z * g, z, t, **HP)
        p.grad = torch.tensor(g)
        opt.step()
        np.testing.assert_allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_update_first_step_closed_form_and_power_zero():
    rng = np.random.default_rng(1)
    P = 64
    theta0, g, hz = rng.standard_normal(P), rng.standard_normal(P), rng.standard_normal(P)
    z = rng.choice([-1.0, 1.0], size=P)
    th, m, v = O.adahessian_update(theta0, np.zeros(P), np.zeros(P), g, hz, z, 1, **HP)
    # t = 1: m_hat = g, v_hat = D^2  ->  theta - lr * g / (|D| + eps)
    np.testing.assert_allclose(th, theta0 - 0.01 * g / (np.abs(hz) + 1e-4), rtol=1e-12)
    hp0 = dict(HP, hpow=0.0)
    th0, _, _ = O.adahessian_update(theta0, np.zeros(P), np.zeros(P), g, hz, z, 1, **hp0)
    np.testing.assert_allclose(th0, theta0 - 0.01 * g / (1.0 + 1e-4), rtol=1e-12)
    # the sign of z matters only through D = z*Hz: flipping z and Hz together changes nothing
    th2, _, _ = O.adahessian_update(theta0, np.zeros(P), np.zeros(P), g, -hz, -z, 1, **HP)
    np.testing.assert_array_equal(th, th2)


def test_spatial_average_blocks():
    dims = (8, 4, 2)
    offs, P = O.layer_offsets(dims)
    D = np.random.default_rng(2).standard_normal(P)
    A = O.spatial_average(D, dims, 4)
    # block sums are preserved; every block is constant; biases untouched; b=1 is the identity
    (w1, b1), (w2, b2) = offs
    np.testing.assert_allclose(A[w1:b1].reshape(-1, 4).sum(1), D[w1:b1].reshape(-1, 4).sum(1), atol=1e-14)
    assert np.all(np.ptp(A[w1:b1].reshape(-1, 4), axis=1) < 1e-15)
    assert np.all(np.ptp(A[w2:b2].reshape(-1, 4), axis=1) < 1e-15)
    np.testing.assert_array_equal(A[b1:b1 + 4], D[b1:b1 + 4])
    np.testing.assert_array_equal(A[b2:], D[b2:])
    np.testing.assert_array_equal(O.spatial_average(D, dims, 1), D)
    # hand example: the mean is signed
    flat = O.spatial_average(np.array([1.0, -3.0, 2.0, 2.0]), None, 2)
    np.testing.assert_array_equal(flat, [-1.0, -1.0, 2.0, 2.0])
    # blocks run along the fan-in axis and never straddle two rows of W
    dims8 = (8, 8, 2)
    Dw = np.zeros(O.layer_offsets(dims8)[1]); Dw[0:8] = 1.0            # first row of W_1 only
    Aw = O.spatial_average(Dw, dims8, 8)
    assert Aw[0:8].tolist() == [1.0] * 8 and np.all(Aw[8:] == 0.0)


def test_update_with_constant_D_is_unchanged_by_averaging():
    rng = np.random.default_rng(3)
    P = 32
    theta0, g = rng.standard_normal(P), rng.standard_normal(P)
    z = rng.choice([-1.0, 1.0], size=P)
    hz = 0.7 * z                                        # D = z*Hz = 0.7 everywhere
    a = O.adahessian_update(theta0, np.zeros(P), np.zeros(P), g, hz, z, 1, avg_block=1, **HP)
    b = O.adahessian_update(theta0, np.zeros(P), np.zeros(P), g, hz, z, 1, avg_block=8, **HP)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-15)


# ------------------------------------------------------------------ dynamic weights
@pytest.mark.parametrize("alpha,kappa", [(0.1, -0.1), (0.25, -0.5), (0.05, -2.0)])
def test_h1_h2_branches_continuity_and_closed_form(alpha, kappa):
    # the three branches of the paper's displays
    assert O.h1(kappa - 1e-9, alpha, kappa) == 1.0 and O.h2(kappa - 1e-9, alpha, kappa) == 0.0
    assert O.h1(1e-9, alpha, kappa) == alpha and O.h2(1e-9, alpha, kappa) == alpha
    # continuity at a = kappa (1, 0) and a = 0 (alpha, alpha)
    assert abs(O.h1(kappa, alpha, kappa) - 1.0) < 1e-15 and abs(O.h2(kappa, alpha, kappa)) < 1e-15
    assert abs(O.h1(0.0, alpha, kappa) - alpha) < 1e-15 and abs(O.h2(0.0, alpha, kappa) - alpha) < 1e-15
    # single-parameter form: s = clamp(a/kappa, 0, 1), h1 = alpha + (1-alpha)s, h2 = alpha(1-s)
    for a in np.linspace(2 * kappa, -kappa, 41):
        s = min(max(a / kappa, 0.0), 1.0)
        assert abs(O.h1(a, alpha, kappa) - (alpha + (1 - alpha) * s)) < 1e-14
        assert abs(O.h2(a, alpha, kappa) - alpha * (1 - s)) < 1e-14
    # a failing worker (negative score) is pulled harder and pulls less
    mid = 0.5 * kappa
    assert O.h1(mid, alpha, kappa) > alpha and O.h2(mid, alpha, kappa) < alpha


def test_raw_score_hand_examples_and_warm_up():
    c = (0.4, 0.3, 0.2, 0.1)
    assert O.raw_score([], c) == 0.0 and O.raw_score([1.7], c) == 0.0
    assert abs(O.raw_score([1.0, 1.5], c) - 0.4 * 0.5) < 1e-15               # only the newest difference
    # full history, differences (oldest..newest) 1, 2, 3, 4 -> 0.1*1 + 0.2*2 + 0.3*3 + 0.4*4
    assert abs(O.raw_score([0.0, 1.0, 3.0, 6.0, 10.0], c) - 3.0) < 1e-15
    # values older than p+1 are ignored
    assert abs(O.raw_score([99.0, 0.0, 1.0, 3.0, 6.0, 10.0], c) - 3.0) < 1e-15
    # a straight line u_t = t*d scores d because the weights sum to one
    assert abs(O.raw_score([0.3 * t for t in range(5)], c) - 0.3) < 1e-15


def test_log_distance():
    a = np.array([3.0, 0.0, 4.0]); b = np.zeros(3)
    assert abs(O.log_distance(a, b) - math.log(5.0)) < 1e-15
    assert O.log_distance(a, a) == 0.5 * math.log(1e-30)       # floor for identical vectors


# ------------------------------------------------------------------ elastic pull
def _state(k=5, P=40, seed=0):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((k, P)), rng.standard_normal(P)


def test_equal_weights_is_easgd():
    th, c = _state()
    alpha = 0.1
    nt, nc = O.elastic_sync(th, c, [alpha] * 5, [alpha] * 5)
    # EASGD: worker moves alpha of the way to the centre, centre moves alpha of the way to each worker
    np.testing.assert_allclose(nt, (1 - alpha) * th + alpha * c, rtol=1e-14)
    np.testing.assert_allclose(nc, c + alpha * (th.sum(0) - 5 * c), rtol=1e-13)
    # centre + sum of workers is conserved when h1_i == h2_i
    np.testing.assert_allclose(nc + nt.sum(0), c + th.sum(0), rtol=1e-13)
    # each pair ends closer together
    assert np.all(np.linalg.norm(nt - nc, axis=1) < np.linalg.norm(th - c, axis=1))


def test_zero_weight_or_absent_worker_leaves_centre_independent_of_it():
    th, c = _state()
    h1s = [0.1, 0.2, 1.0, 0.1, 0.3]
    h2s = [0.1, 0.05, 0.0, 0.1, 0.02]
    _, nc = O.elastic_sync(th, c, h1s, h2s)
    th2 = th.copy(); th2[2] += 100.0
    nt2, nc2 = O.elastic_sync(th2, c, h1s, h2s)
    np.testing.assert_array_equal(nc, nc2)                     # h2 = 0: centre never sees worker 2
    np.testing.assert_allclose(nt2[2], c, atol=1e-12)          # h1 = 1: the worker is reset to the centre
    part = [1, 1, 1, 0, 1]
    nt3, nc3 = O.elastic_sync(th, c, h1s, h2s, part)
    th4 = th.copy(); th4[3] -= 55.0
    nt4, nc4 = O.elastic_sync(th4, c, h1s, h2s, part)
    np.testing.assert_array_equal(nc3, nc4)
    np.testing.assert_array_equal(nt3[3], th[3])               # a suppressed worker keeps its parameters


def test_fixed_point_and_single_worker_contraction():
    _, c = _state()
    th = np.tile(c, (3, 1))
    nt, nc = O.elastic_sync(th, c, [0.3, 0.1, 1.0], [0.2, 0.1, 0.0])
    np.testing.assert_array_equal(nt, th); np.testing.assert_array_equal(nc, c)
    th1, c1 = _state(k=1, seed=3)
    nt, nc = O.elastic_sync(th1, c1, [0.3], [0.2])
    np.testing.assert_allclose(nt[0] - nc, (1 - 0.3 - 0.2) * (th1[0] - c1), rtol=1e-13)


def test_trainer_modes_and_dynamic_round():
    cfg = O.OracleConfig(dims=None, k=3, n_params=16, alpha=0.1, kappa=-0.1)
    rng = np.random.default_rng(5)
    tr = O.OracleTrainer(cfg, rng.standard_normal(16))
    g = rng.standard_normal((3, 16)); hz = rng.standard_normal((3, 16))
    tr.update_only(g, hz)
    assert tr.t.tolist() == [1, 1, 1]
    c0, t0 = tr.centre.copy(), tr.theta.copy()
    assert tr.elastic_sync(O.MODE_DYNAMIC, tau=1)
    # first round: history too short, a = 0 -> both weights alpha (equal initial weights)
    np.testing.assert_array_equal(tr.last_a, 0.0)
    np.testing.assert_allclose(tr.last_h1, 0.1); np.testing.assert_allclose(tr.last_h2, 0.1)
    np.testing.assert_allclose(tr.theta, 0.9 * t0 + 0.1 * c0, rtol=1e-13)
    # worker 2 does not step and is pulled: its distance shrinks, its score goes negative,
    # so next round h1 rises above alpha and h2 falls below it; the others stepped away (a > 0 -> alpha)
    tr.update_only(g, hz, active=[1, 1, 0])
    tr.elastic_sync(O.MODE_DYNAMIC, tau=1)
    assert tr.last_a[2] < 0 and tr.last_h1[2] > 0.1 and tr.last_h2[2] < 0.1
    # tau gating: rounds only when the step count is a multiple of tau
    tr.update_only(g, hz)
    assert tr.global_step == 3 and not tr.elastic_sync(O.MODE_FIXED, tau=2)
    tr.update_only(g, hz)
    assert tr.elastic_sync(O.MODE_FIXED, tau=2)


# ---------------------------------------------------------------------------------------------------------
# Sequential form of a round: a chain of single-worker exchanges, each eq.(12)-(13) as printed.
# ---------------------------------------------------------------------------------------------------------
def _exchange_matrix(k, i, h1, h2):
    """Linear map of one exchange of worker i on the state (theta_0 .. theta_{k-1}, centre), one coordinate."""
    M = np.eye(k + 1)
    M[i, i] = 1.0 - h1; M[i, k] = h1            # theta_i <- theta_i - h1 (theta_i - c)
    M[k, k] = 1.0 - h2; M[k, i] = h2            # c       <- c + h2 (theta_i - c)
    return M


def test_sequential_round_is_the_product_of_single_exchanges():
    rng = np.random.default_rng(5)
    k, P = 5, 7
    th, c = rng.normal(size=(k, P)), rng.normal(size=P)
    h1s, h2s = rng.uniform(0.05, 1.0, k), rng.uniform(0.0, 0.6, k)
    part = np.array([1, 0, 1, 1, 0], dtype=np.uint8)
    new_t, new_c = O.elastic_sync_sequential(th, c, h1s, h2s, part)
    M = np.eye(k + 1)
    for i in range(k):
        if part[i]:
            M = _exchange_matrix(k, i, h1s[i], h2s[i]) @ M      # later exchanges act on the earlier ones' result
    state = M @ np.vstack([th, c[None, :]])
    np.testing.assert_allclose(new_t, state[:k], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(new_c, state[k], rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(new_t[1], th[1]); np.testing.assert_array_equal(new_t[4], th[4])


def test_sequential_round_special_cases():
    rng = np.random.default_rng(6)
    k, P = 4, 9
    th, c = rng.normal(size=(k, P)), rng.normal(size=P)
    h1s, h2s = rng.uniform(0.1, 0.9, k), rng.uniform(0.1, 0.5, k)
    # a single participant: both forms are eq.(12)-(13) for that worker
    one = np.array([0, 0, 1, 0], dtype=np.uint8)
    ta, ca = O.elastic_sync(th, c, h1s, h2s, one)
    tb, cb = O.elastic_sync_sequential(th, c, h1s, h2s, one)
    np.testing.assert_allclose(ta, tb, rtol=0, atol=1e-15); np.testing.assert_allclose(ca, cb, rtol=0, atol=1e-15)
    np.testing.assert_allclose(cb, c + h2s[2] * (th[2] - c), rtol=1e-14)
    np.testing.assert_allclose(tb[2], th[2] - h1s[2] * (th[2] - c), rtol=1e-14)
    # h2 = 0: the centre never moves, so the order of the exchanges cannot matter
    ta, ca = O.elastic_sync(th, c, h1s, np.zeros(k))
    tb, cb = O.elastic_sync_sequential(th, c, h1s, np.zeros(k))
    np.testing.assert_allclose(ta, tb, rtol=0, atol=1e-15); np.testing.assert_array_equal(cb, c)
    # symmetric rate (plain elastic averaging): every exchange conserves theta_i + centre
    a = np.full(k, 0.3)
    tb, cb = O.elastic_sync_sequential(th, c, a, a)
    np.testing.assert_allclose(tb.sum(0) + cb, th.sum(0) + c, rtol=1e-13)
    # consensus is a fixed point; and with several participants the order does matter
    same = np.tile(c, (k, 1))
    tb, cb = O.elastic_sync_sequential(same, c, h1s, h2s)
    np.testing.assert_array_equal(tb, same); np.testing.assert_array_equal(cb, c)
    tj, cj = O.elastic_sync(th, c, h1s, h2s)
    ts, cs = O.elastic_sync_sequential(th, c, h1s, h2s)
    assert np.max(np.abs(cj - cs)) > 1e-3
    # two workers, written out: the second one sees the centre the first one moved
    c1 = c + h2s[0] * (th[0] - c)
    ts2, cs2 = O.elastic_sync_sequential(th[:2], c, h1s[:2], h2s[:2])
    np.testing.assert_allclose(ts2[1], th[1] - h1s[1] * (th[1] - c1), rtol=1e-14)
    np.testing.assert_allclose(cs2, c1 + h2s[1] * (th[1] - c1), rtol=1e-14)


def test_trainer_sequential_round_uses_the_scores_of_the_round_start():
    cfg = O.OracleConfig(dims=None, k=3, n_params=16, seed=3)
    rng = np.random.default_rng(8)
    ta = O.OracleTrainer(cfg, rng.normal(size=16)); tb = O.OracleTrainer(cfg, ta.centre.copy())
    pert = rng.normal(size=(3, 16)) * 0.1
    ta.theta = ta.theta + pert; tb.theta = tb.theta + pert
    assert ta.elastic_sync(O.MODE_DYNAMIC) and tb.elastic_sync(O.MODE_DYNAMIC, sequential=True)
    np.testing.assert_array_equal(ta.last_u, tb.last_u)          # same u, a, h1, h2 ...
    np.testing.assert_array_equal(ta.last_h1, tb.last_h1)
    assert np.max(np.abs(ta.centre - tb.centre)) > 0             # ... different pull


# ---------------------------------------------------------------------------------------------------------
# Baseline worker steps (Section II eq.(3); EASGD and EASGD with momentum of Section VI, delta = 0.5 in Section VII)
# ---------------------------------------------------------------------------------------------------------
def test_sgd_step_closed_forms():
    # eq.(3) on f = a/2 theta^2 (g = a theta): theta_t = (1 - eta a)^t theta_0
    a, eta = np.array([0.5, 2.0, 30.0]), 0.01
    th = np.array([1.0, -2.0, 0.25])
    th0 = th.copy()
    for _ in range(7):
        th = O.sgd_update(th, a * th, lr=eta)
    np.testing.assert_allclose(th, (1.0 - eta * a) ** 7 * th0, rtol=1e-14)
    # a constant gradient moves the parameters along a straight line
    g = np.array([3.0, -1.0, 0.0])
    np.testing.assert_array_equal(O.sgd_update(th0, g, lr=0.5), th0 - 0.5 * g)


def test_momentum_step_against_torch_sgd_and_its_closed_form():
    import torch
    rng = np.random.default_rng(12)
    P, steps, eta, delta = 50, 9, 0.01, 0.5
    th0 = rng.standard_normal(P)
    gs = rng.standard_normal((steps, P))
    th, buf = th0.copy(), np.zeros(P)
    t = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([t], lr=eta, momentum=delta)
    for s in range(steps):
        th, buf = O.momentum_update(th, buf, gs[s], lr=eta, momentum=delta)
        t.grad = torch.tensor(gs[s])
        opt.step()
        np.testing.assert_allclose(th, t.detach().numpy(), rtol=1e-13, atol=1e-15)
    # constant gradient: velocity g (1 - delta^t)/(1 - delta), position theta_0 - eta g sum_s (1 - delta^s)/(1 - delta)
    g = rng.standard_normal(P)
    th, buf = th0.copy(), np.zeros(P)
    for s in range(1, 6):
        th, buf = O.momentum_update(th, buf, g, lr=eta, momentum=delta)
    np.testing.assert_allclose(buf, g * (1 - delta ** 5) / (1 - delta), rtol=1e-14)
    np.testing.assert_allclose(th, th0 - eta * g * sum((1 - delta ** s) / (1 - delta) for s in range(1, 6)), rtol=1e-13)
    # delta = 0 is plain SGD
    np.testing.assert_array_equal(O.momentum_update(th0, buf, g, lr=eta, momentum=0.0)[0], O.sgd_update(th0, g, lr=eta))


@pytest.mark.parametrize("opt", [O.OPT_SGD, O.OPT_MOMENTUM])
def test_easgd_trainer_is_first_order_steps_plus_the_fixed_rate_pull(opt):
    """EASGD / EAMSGD as the trainer runs them against a loop written out here with torch's autograd for the gradients:
    k = 2 workers of a tiny ReLU classifier, a fixed-rate round (eq.(8)-(9) with the signs of eq.(12)-(13)) every
    second step, worker 1 suppressed in the first round."""
    import torch
    dims, B, k, eta, delta, alpha = (5, 6, 3), 7, 2, 0.01, 0.5, 0.1
    rng = np.random.default_rng(77)
    _, P = O.layer_offsets(dims)
    theta0 = rng.standard_normal(P) * 0.3
    xs = rng.standard_normal((4, k, B, dims[0])); ys = rng.integers(0, dims[-1], size=(4, k, B))
    tr = O.OracleTrainer(O.OracleConfig(dims=dims, k=k, lr=eta, alpha=alpha, optimizer=opt, momentum=delta), theta0)

    def torch_grad(theta, x, y):
        t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
        W1 = t[:30].reshape(6, 5); b1 = t[30:36]; W2 = t[36:54].reshape(3, 6); b2 = t[54:57]
        out = torch.relu(torch.tensor(x) @ W1.T + b1) @ W2.T + b2
        torch.nn.functional.cross_entropy(out, torch.tensor(y)).backward()
        return t.grad.numpy()

    th = np.tile(theta0, (k, 1)); buf = np.zeros((k, P)); centre = theta0.copy()
    for step in range(4):
        tr.worker_step(xs[step], ys[step])
        for i in range(k):
            g = torch_grad(th[i], xs[step][i], ys[step][i])
            if opt == O.OPT_SGD:
                th[i] = th[i] - eta * g
            else:
                buf[i] = delta * buf[i] + g
                th[i] = th[i] - eta * buf[i]
        part = [1, 0] if step == 1 else [1, 1]
        did = tr.elastic_sync(O.MODE_FIXED, tau=2, participate=part)
        assert did == (step % 2 == 1)
        if did:
            d = [th[i] - centre for i in range(k)]
            for i in range(k):
                if part[i]:
                    th[i] = th[i] - alpha * d[i]
                    centre = centre + alpha * d[i]
        np.testing.assert_allclose(tr.theta, th, rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(tr.centre, centre, rtol=1e-11, atol=1e-14)
    assert np.all(tr.v == 0.0) and (np.all(tr.m == 0.0) == (opt == O.OPT_SGD))       # no second moment; velocity in m
    assert list(tr.t) == [4, 4]
