"""Pins for the oracle's loss, gradient and Hessian-vector product (CPU only).

Each check compares the oracle with something it does not compute itself: finite differences,
a Hessian assembled by brute force, the textbook closed form for softmax regression, torch's
autograd, or an algebraic identity (Section II eq.(2); Section IV-B Hutchinson display).
"""
import math

import numpy as np
import pytest
import torch

from oracle import dw_oracle as O

DIMS_TINY = (3, 4, 2)          # P = 3*4+4 + 4*2+2 = 26
DIMS_DEEP = (5, 7, 6, 4)


def _problem(dims, B, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    _, P = O.layer_offsets(dims)
    theta = rng.standard_normal(P) * scale / math.sqrt(dims[0])
    x = rng.standard_normal((B, dims[0]))
    y = rng.integers(0, dims[-1], size=B)
    return theta, x, y, P


def _kink_margin(theta, x, y, dims):
    tr = O.StepTrace()
    O.grad_and_hvp(theta, x, y, dims, None, trace=tr)
    return tr.min_abs_preact


def test_layout_offsets():
    offs, P = O.layer_offsets((3, 4, 2))
    assert offs == [(0, 12), (16, 24)] and P == 26
    th = np.arange(P, dtype=float)
    (W1, b1), (W2, b2) = O.unpack(th, (3, 4, 2))
    assert W1.shape == (4, 3) and W1[1, 0] == 3 and b1[0] == 12 and W2[1, 3] == 23 and b2[1] == 25


def test_loss_zero_weights_is_log_classes():
    dims = (6, 5, 3)
    _, P = O.layer_offsets(dims)
    x = np.random.default_rng(0).standard_normal((9, 6))
    y = np.arange(9) % 3
    assert abs(O.loss_only(np.zeros(P), x, y, dims) - math.log(3)) < 1e-14
    loss, g, _ = O.grad_and_hvp(np.zeros(P), x, y, dims)
    assert abs(loss - math.log(3)) < 1e-14


@pytest.mark.parametrize("dims,B,seed", [(DIMS_TINY, 5, 1), (DIMS_DEEP, 6, 2), ((4, 3), 7, 3)])
def test_gradient_matches_finite_difference_of_loss(dims, B, seed):
    theta, x, y, P = _problem(dims, B, seed)
    assert _kink_margin(theta, x, y, dims) > 1e-3
    _, g, _ = O.grad_and_hvp(theta, x, y, dims)
    h = 1e-6
    for j in range(P):
        e = np.zeros(P); e[j] = h
        fd = (O.loss_only(theta + e, x, y, dims) - O.loss_only(theta - e, x, y, dims)) / (2 * h)
        assert abs(fd - g[j]) < 1e-8 + 1e-6 * abs(g[j]), j


@pytest.mark.parametrize("dims,B,seed", [(DIMS_TINY, 5, 1), (DIMS_DEEP, 6, 2)])
def test_gradient_matches_torch_autograd(dims, B, seed):
    theta, x, y, P = _problem(dims, B, seed)
    _, g, _ = O.grad_and_hvp(theta, x, y, dims)
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    a = torch.tensor(x)
    pos = 0
    L = len(dims) - 1
    for l in range(1, L + 1):
        W = t[pos:pos + dims[l] * dims[l - 1]].reshape(dims[l], dims[l - 1]); pos += dims[l] * dims[l - 1]
        b = t[pos:pos + dims[l]]; pos += dims[l]
        a = a @ W.T + b
        if l < L:
            a = torch.relu(a)
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(y), reduction="mean")
    loss.backward()
    np.testing.assert_allclose(g, t.grad.numpy(), rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("dims,B,seed", [(DIMS_TINY, 5, 1), (DIMS_DEEP, 6, 2)])
def test_hvp_matches_central_differences_of_gradient(dims, B, seed):
    theta, x, y, P = _problem(dims, B, seed)
    assert _kink_margin(theta, x, y, dims) > 1e-3
    rng = np.random.default_rng(seed + 100)
    for trial in range(4):
        z = rng.choice([-1.0, 1.0], size=P) if trial < 3 else rng.standard_normal(P)
        _, _, hz = O.grad_and_hvp(theta, x, y, dims, z)
        h = 1e-5
        gp = O.grad_and_hvp(theta + h * z, x, y, dims)[1]
        gm = O.grad_and_hvp(theta - h * z, x, y, dims)[1]
        fd = (gp - gm) / (2 * h)
        np.testing.assert_allclose(hz, fd, rtol=1e-5, atol=1e-8 * np.abs(hz).max() + 1e-10)


def _brute_force_hessian(theta, x, y, dims, h=1e-5):
    """Hessian by central differences of the gradient along unit vectors (no R-operator involved)."""
    P = theta.size
    H = np.zeros((P, P))
    for j in range(P):
        e = np.zeros(P); e[j] = h
        H[:, j] = (O.grad_and_hvp(theta + e, x, y, dims)[1] - O.grad_and_hvp(theta - e, x, y, dims)[1]) / (2 * h)
    return H


def test_hvp_on_unit_vectors_rebuilds_brute_force_hessian_and_is_symmetric():
    theta, x, y, P = _problem(DIMS_TINY, 6, 4)
    assert _kink_margin(theta, x, y, DIMS_TINY) > 1e-3
    H_fd = _brute_force_hessian(theta, x, y, DIMS_TINY)
    H_r = np.stack([O.grad_and_hvp(theta, x, y, DIMS_TINY, np.eye(P)[j])[2] for j in range(P)], axis=1)
    np.testing.assert_allclose(H_r, H_fd, atol=2e-8)
    np.testing.assert_allclose(H_r, H_r.T, atol=1e-13)          # u^T H v = v^T H u
    # within one layer's weights the logits are linear in theta for fixed masks, so that diagonal
    # block is positive semi-definite; in particular the exact diagonal is non-negative
    assert H_r.diagonal().min() > -1e-14
    offs, _ = O.layer_offsets(DIMS_TINY)
    for (w_off, b_off), d in zip(offs, DIMS_TINY[1:]):
        blk = H_r[w_off:b_off + d, w_off:b_off + d]
        assert np.linalg.eigvalsh(blk).min() > -1e-12


def test_hvp_linearity_and_zero():
    theta, x, y, P = _problem(DIMS_DEEP, 5, 7)
    rng = np.random.default_rng(0)
    u, v = rng.standard_normal(P), rng.standard_normal(P)
    Hu = O.grad_and_hvp(theta, x, y, DIMS_DEEP, u)[2]
    Hv = O.grad_and_hvp(theta, x, y, DIMS_DEEP, v)[2]
    Huv = O.grad_and_hvp(theta, x, y, DIMS_DEEP, 2.0 * u - 3.0 * v)[2]
    np.testing.assert_allclose(Huv, 2.0 * Hu - 3.0 * Hv, atol=1e-13)
    assert np.all(O.grad_and_hvp(theta, x, y, DIMS_DEEP, np.zeros(P))[2] == 0.0)
    assert abs(u @ Hv - v @ Hu) < 1e-12


def test_hvp_softmax_regression_closed_form():
    """No hidden layer: H = (1/B) sum_n (diag(p_n) - p_n p_n^T) kron x~_n x~_n^T, x~ = (x, 1)."""
    dims = (4, 3)
    theta, x, y, P = _problem(dims, 8, 9)
    d, C = dims
    (W, b), = O.unpack(theta, dims)
    p = O.softmax_rows(x @ W.T + b)
    B = x.shape[0]
    # index map of the canonical layout: W[c, j] -> c*d + j ; b[c] -> C*d + c
    H = np.zeros((P, P))
    for n in range(B):
        S = np.diag(p[n]) - np.outer(p[n], p[n])
        xt = np.append(x[n], 1.0)
        for c1 in range(C):
            for c2 in range(C):
                for j1 in range(d + 1):
                    for j2 in range(d + 1):
                        i1 = c1 * d + j1 if j1 < d else C * d + c1
                        i2 = c2 * d + j2 if j2 < d else C * d + c2
                        H[i1, i2] += S[c1, c2] * xt[j1] * xt[j2] / B
    rng = np.random.default_rng(1)
    for _ in range(3):
        z = rng.choice([-1.0, 1.0], size=P)
        np.testing.assert_allclose(O.grad_and_hvp(theta, x, y, dims, z)[2], H @ z, atol=1e-13)


def test_hutchinson_exact_with_hadamard_probes_and_monte_carlo_rate():
    """(1/n) sum z_i * (H z_i) equals diag(H) exactly when (1/n) sum z_i z_i^T = I, which holds for
    the rows of a Sylvester Hadamard matrix restricted to P columns; random Rademacher probes
    converge to the same diagonal at the Monte-Carlo rate."""
    theta, x, y, P = _problem(DIMS_TINY, 6, 4)
    H = _brute_force_hessian(theta, x, y, DIMS_TINY)
    n = 32
    Had = np.array([[1.0]])
    while Had.shape[0] < n:
        Had = np.block([[Had, Had], [Had, -Had]])
    est = np.zeros(P)
    for i in range(n):
        z = Had[i, :P]
        est += z * O.grad_and_hvp(theta, x, y, DIMS_TINY, z)[2]
    est /= n
    np.testing.assert_allclose(est, H.diagonal(), atol=2e-8)

    words = O.rademacher_words(5, 0, 0, P)
    errs = []
    for N in (64, 4096):
        acc = np.zeros(P)
        for i in range(N):
            z = O.words_to_signs(O.rademacher_words(5, 0, i, P), P)
            acc += z * O.grad_and_hvp(theta, x, y, DIMS_TINY, z)[2]
        errs.append(np.abs(acc / N - H.diagonal()).max())
    offdiag = np.sqrt((H ** 2).sum(axis=1) - H.diagonal() ** 2).max()
    assert errs[1] < 4.0 * offdiag / math.sqrt(4096)
    assert errs[1] < errs[0]


def test_bf16_rounding_helper():
    v = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.3, 3.0e38, 0.0])
    r = O.round_bf16(v)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == 1.0 + 2 ** -7 and r[3] == 1.0 + 2 ** -6
    t = torch.tensor(v, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(r, t)
    big = np.random.default_rng(0).standard_normal(10000)
    np.testing.assert_array_equal(O.round_bf16(big),
                                  torch.tensor(big, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy())


def test_hutchinson_diagonal_of_n_probes_and_the_update_that_uses_it():
    """Section IV-B with n probes: the estimate is the mean of z_j * (H z_j); with the P-column restriction of a
    Hadamard matrix as probes it is diag(H) exactly, and the update takes D from it."""
    theta, x, y, P = _problem(DIMS_TINY, 6, 4)
    H = _brute_force_hessian(theta, x, y, DIMS_TINY)
    n = 32
    Had = np.array([[1.0]])
    while Had.shape[0] < n:
        Had = np.block([[Had, Had], [Had, -Had]])
    zs = Had[:, :P]
    hzs = np.stack([O.grad_and_hvp(theta, x, y, DIMS_TINY, z)[2] for z in zs])
    np.testing.assert_allclose(O.hutchinson_diagonal(zs, hzs), H.diagonal(), atol=2e-8)
    # one probe: the plain product; two probes: the mean of the two single-probe estimates
    np.testing.assert_array_equal(O.hutchinson_diagonal(zs[3], hzs[3]), zs[3] * hzs[3])
    np.testing.assert_allclose(O.hutchinson_diagonal(zs[:2], hzs[:2]), 0.5 * (zs[0] * hzs[0] + zs[1] * hzs[1]), rtol=1e-15)
    g = O.grad_and_hvp(theta, x, y, DIMS_TINY, zs[0])[1]
    hp = dict(lr=0.01, beta1=0.9, beta2=0.999, eps=1e-4, hpow=1.0)
    th_n, m_n, v_n = O.adahessian_update(theta, np.zeros(P), np.zeros(P), g, hzs, zs, 1, **hp)
    # with the exact diagonal, the first step is lr * g / (|diag(H)| + eps) (bias corrections cancel at t = 1)
    np.testing.assert_allclose(theta - th_n, 0.01 * g / (np.abs(H.diagonal()) + 1e-4), rtol=1e-6, atol=1e-12)
    np.testing.assert_allclose(v_n, 0.001 * H.diagonal() ** 2, rtol=1e-6, atol=1e-18)


def test_trainer_draws_distinct_probes_per_step_and_keeps_the_single_probe_stream():
    dims = DIMS_TINY
    P = O.layer_offsets(dims)[-1] if hasattr(O, "layer_offsets") else None
    theta, x, y, P = _problem(dims, 6, 4)
    one = O.OracleTrainer(O.OracleConfig(dims=dims, k=1, seed=9), theta)
    three = O.OracleTrainer(O.OracleConfig(dims=dims, k=1, seed=9, n_samples=3), theta)
    np.testing.assert_array_equal(one.draw_z(0), O.words_to_signs(O.rademacher_words(9, 0, 0, P), P))
    zs = [three.draw_z(0, j) for j in range(3)]
    np.testing.assert_array_equal(zs[0], one.draw_z(0))                     # position 0 either way
    assert not np.array_equal(zs[0], zs[1]) and not np.array_equal(zs[1], zs[2])
    three.worker_step(x[None], y[None]); one.worker_step(x[None], y[None])
    # second step: positions 3, 4, 5 against position 1
    np.testing.assert_array_equal(three.draw_z(0, 0), O.words_to_signs(O.rademacher_words(9, 0, 3, P), P))
    np.testing.assert_array_equal(one.draw_z(0), O.words_to_signs(O.rademacher_words(9, 0, 1, P), P))
    # the 3-probe step used the mean of the three single-probe estimates
    hz = three.traces[0].hz
    assert hz.shape == (3, P)
    D = (np.stack(zs) * hz).mean(axis=0)
    np.testing.assert_allclose(three.v[0], 0.001 * D ** 2, rtol=1e-12, atol=1e-30)
