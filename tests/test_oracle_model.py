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


# ---------------------------------------------------------------------------------------------------------
# ReLU ties: the only place where a caller may dictate anything to the oracle.  The pins below fix what that
# is: nothing outside the band, and inside it one of the two one-sided derivatives.
# ---------------------------------------------------------------------------------------------------------
def test_tie_choice_cannot_touch_a_unit_outside_the_band():
    dims = DIMS_DEEP
    theta, x, y, P = _problem(dims, 40, 11)
    z = np.random.default_rng(3).choice([-1.0, 1.0], size=P)
    plain = O.grad_and_hvp(theta, x, y, dims, z)
    band = 0.05
    tr = O.StepTrace()
    O.grad_and_hvp(theta, x, y, dims, z, trace=tr, tie_band=band)
    # the reported ties are exactly the units with |s| < band * rms(s_l), counted here from the pre-activations
    n_ties = 0
    for l, s_l in enumerate(tr.pre_acts[:-1]):
        want = np.abs(s_l) < band * np.sqrt(np.mean(s_l ** 2))
        np.testing.assert_array_equal(tr.ties[l], want)
        n_ties += int(want.sum())
    assert 0 < n_ties < 0.1 * sum(s.size for s in tr.pre_acts[:-1])
    rng = np.random.default_rng(4)
    natural = [s_l > 0 for s_l in tr.pre_acts[:-1]]
    # any choice that agrees with the natural slopes inside the band gives the plain result, whatever it says outside
    noise = [np.where(t, n, rng.random(n.shape) < 0.5) for t, n in zip(tr.ties, natural)]
    got = O.grad_and_hvp(theta, x, y, dims, z, tie_band=band, tie_choice=noise)
    for a, b in zip(got, plain):
        np.testing.assert_array_equal(a, b)
    # without a band a choice is ignored altogether
    got = O.grad_and_hvp(theta, x, y, dims, z, tie_band=0.0, tie_choice=[~n for n in natural])
    for a, b in zip(got, plain):
        np.testing.assert_array_equal(a, b)
    # flipping the units inside the band does change the result (the band is not a dead letter)
    flipped = [np.where(t, ~n, n) for t, n in zip(tr.ties, natural)]
    got = O.grad_and_hvp(theta, x, y, dims, z, tie_band=band, tie_choice=flipped)
    assert np.abs(got[1] - plain[1]).max() > 1e-6 and np.abs(got[2] - plain[2]).max() > 1e-6
    assert got[0] == plain[0]                                   # the loss never depends on the slope chosen


@pytest.mark.parametrize("side", ["on", "off"])
def test_a_dictated_tie_is_the_one_sided_derivative(side):
    """A hidden unit a hair's breadth from its kink, its slope dictated through tie_choice: g and Hz must be those of
    the network with that unit moved just across the kink (bias shifted by twice the distance), where no tie exists."""
    dims = DIMS_DEEP
    theta, x, y, P = _problem(dims, 6, 21)
    z = np.random.default_rng(5).choice([-1.0, 1.0], size=P)
    offs, _ = O.layer_offsets(dims)
    n, j, gap = 2, 3, 1e-10
    tr = O.StepTrace()
    O.grad_and_hvp(theta, x, y, dims, z, trace=tr)
    theta = theta.copy()
    # put s_1[n, j] at -gap (natural slope off) or +gap (natural slope on) by moving the unit's bias
    theta[offs[0][1] + j] += (gap if side == "off" else -gap) - tr.pre_acts[0][n, j]
    tr = O.StepTrace()
    O.grad_and_hvp(theta, x, y, dims, z, trace=tr)
    assert abs(abs(tr.pre_acts[0][n, j]) - gap) < 1e-14 and (tr.pre_acts[0][n, j] > 0) == (side == "off")
    others = min(np.abs(np.delete(tr.pre_acts[0].reshape(-1), n * dims[1] + j)).min(), np.abs(tr.pre_acts[1]).min())
    band = 1e-8 / np.sqrt(np.mean(tr.pre_acts[0] ** 2))
    assert others > 1e-6                                         # the band below holds this one unit only
    choice = [s_l > 0 for s_l in tr.pre_acts[:-1]]
    choice[0][n, j] = side == "on"
    tr2 = O.StepTrace()
    forced = O.grad_and_hvp(theta, x, y, dims, z, trace=tr2, tie_band=band, tie_choice=choice)
    assert int(tr2.ties[0].sum()) == 1 and tr2.ties[0][n, j] and int(tr2.ties[1].sum()) == 0
    across = theta.copy()
    across[offs[0][1] + j] += 2 * gap if side == "on" else -2 * gap
    want = O.grad_and_hvp(across, x, y, dims, z)
    natural = O.grad_and_hvp(theta, x, y, dims, z)
    for a, b, c in zip(forced[1:], want[1:], natural[1:]):
        assert np.abs(a - b).max() < 1e-8 and np.abs(a - c).max() > 1e-5


# ---------------------------------------------------------------------------------------------------------
# Mixed precision: where the oracle rounds to bfloat16.  The pipeline stores x, the weights, a_l, Ra_l and the
# back-propagated d_l, Rd_l in bf16 and keeps every sum, g and Hz wider.
# ---------------------------------------------------------------------------------------------------------
class _Rounder:
    """round_bf16 that can leave one of its call sites out; records what went through it."""

    def __init__(self, skip=None):
        self.skip, self.calls = skip, []

    def __call__(self, a):
        idx = len(self.calls)
        self.calls.append(np.shape(a))
        return np.asarray(a, dtype=np.float64) if idx == self.skip else O.round_bf16(a)


def test_bf16_mode_rounds_at_the_stored_tensors_and_every_rounding_point_matters():
    dims, B = (8, 12, 6, 4), 10                 # L = 3: two hidden layers
    theta, x, y, P = _problem(dims, B, 33)
    z = np.random.default_rng(6).choice([-1.0, 1.0], size=P)
    L = len(dims) - 1
    q = _Rounder()
    loss, g, hz = O.grad_and_hvp(theta, x, y, dims, z, q)
    # what is rounded, by shape: x once; every W_l (read by the forward pass and again by the R- and backward passes);
    # a_l and Ra_l of the hidden layers; d_l and Rd_l of every layer
    shapes = q.calls
    assert shapes.count((B, dims[0])) == 1
    for l in range(1, L + 1):
        assert shapes.count((dims[l], dims[l - 1])) == 2
    hidden = sum(shapes.count((B, dims[l])) for l in range(1, L))
    assert hidden == 4 * (L - 1)                                 # a_l, Ra_l, d_l, Rd_l per hidden layer
    assert shapes.count((B, dims[L])) == 2                       # d_L, Rd_L
    assert len(shapes) == 1 + 2 * L + 4 * (L - 1) + 2
    # every result is computed from rounded operands only: the same call on inputs that are already bf16 values
    # and with the weights pre-rounded gives the same bits
    offs, _ = O.layer_offsets(dims)
    th_r = theta.copy()
    for l, (w_off, b_off) in enumerate(offs):
        th_r[w_off:b_off] = O.round_bf16(theta[w_off:b_off])
    same = O.grad_and_hvp(th_r, O.round_bf16(x), y, dims, z, O.round_bf16)
    assert same[0] == loss
    np.testing.assert_array_equal(same[1], g); np.testing.assert_array_equal(same[2], hz)
    # the biases are not rounded (fp32 state added in the epilogue): rounding them as well changes the result
    th_b = th_r.copy()
    for l, (w_off, b_off) in enumerate(offs):
        th_b[b_off:b_off + dims[l + 1]] = O.round_bf16(th_b[b_off:b_off + dims[l + 1]])
    assert np.abs(O.grad_and_hvp(th_b, x, y, dims, z, O.round_bf16)[1] - g).max() > 0
    # leaving out any single rounding point changes g or Hz.  The one exception: the copy of W_1 read after the
    # forward pass multiplies Ra_0 = 0 only (the input does not depend on the parameters) and no error is propagated
    # below the first layer, so its rounding cannot show
    w1_again = [i for i, sh in enumerate(shapes) if sh == (dims[1], dims[0])][1]
    for skip, shape in enumerate(shapes):
        q2 = _Rounder(skip)
        l2, g2, hz2 = O.grad_and_hvp(theta, x, y, dims, z, q2)
        assert q2.calls == shapes
        dg, dh = np.abs(g2 - g).max(), np.abs(hz2 - hz).max()
        assert (dg > 0 or dh > 0) == (skip != w1_again), (skip, shape)
    # identity rounding is the full-precision oracle
    full = O.grad_and_hvp(theta, x, y, dims, z)
    ident = O.grad_and_hvp(theta, x, y, dims, z, lambda a: a)
    for a, b in zip(full, ident):
        np.testing.assert_array_equal(a, b)
    # and bf16 results sit within bf16 rounding of it: a few 2^-9 per rounding point, far from equal
    rel = np.linalg.norm(g - full[1]) / np.linalg.norm(full[1])
    assert 1e-4 < rel < 3e-2, rel


def test_r_pass_rounding_points_leave_the_gradient_alone():
    """Ra_l and Rd_l feed only the Hessian-vector product: leaving their rounding out must not move g or the loss."""
    dims, B = (8, 12, 6, 4), 10
    theta, x, y, P = _problem(dims, B, 34)
    z = np.random.default_rng(7).choice([-1.0, 1.0], size=P)
    q = _Rounder()
    loss, g, hz = O.grad_and_hvp(theta, x, y, dims, z, q)
    q_none = _Rounder()
    loss_n, g_n, _ = O.grad_and_hvp(theta, x, y, dims, None, q_none)          # no z: no R-pass, fewer roundings
    assert loss_n == loss
    np.testing.assert_array_equal(g_n, g)
    L = len(dims) - 1
    assert len(q.calls) - len(q_none.calls) == (L - 1) + L                    # Ra_l of the hidden layers, Rd_l of all


def test_trainer_bf16_flag_selects_the_rounding():
    dims, B = (8, 12, 4), 6
    theta, x, y, P = _problem(dims, B, 35)
    theta32 = theta.astype(np.float32).astype(np.float64)
    a = O.OracleTrainer(O.OracleConfig(dims=dims, k=1, seed=2, bf16=True), theta32)
    b = O.OracleTrainer(O.OracleConfig(dims=dims, k=1, seed=2, bf16=False), theta32)
    a.worker_step(x[None], y[None]); b.worker_step(x[None], y[None])
    zz = a.traces[0].z
    want = O.grad_and_hvp(theta32, x, y, dims, zz, O.round_bf16)
    np.testing.assert_array_equal(a.traces[0].g, want[1]); np.testing.assert_array_equal(a.traces[0].hz, want[2])
    a.q = lambda v: v                                                          # identity rounding = the fp32 trainer
    a.theta[0] = theta32; a.m[:] = 0; a.v[:] = 0; a.t[:] = 0
    a.worker_step(x[None], y[None])
    np.testing.assert_array_equal(a.traces[0].g, b.traces[0].g)
    np.testing.assert_array_equal(a.traces[0].hz, b.traces[0].hz)
    np.testing.assert_array_equal(a.theta[0], b.theta[0])
