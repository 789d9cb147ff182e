"""Pins for the convolutional oracle (CPU only): each layer against a library routine or its adjoint identity,
the gradient and the Hessian-vector product against finite differences and against torch's autograd (an
independent implementation), the averaging against its definition (Section IV-B; Section VI for the model)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F
from scipy.signal import correlate2d

from oracle import dw_cnn as C

TINY = C.CnnSpec(img=(6, 6, 1), conv=(2, 3), fc=(4, 3))           # 2x2 map -> pooled 1x1x3
SMALL = C.CnnSpec(img=(10, 8, 2), conv=(4, 6), fc=(8, 5))         # 6x4 map -> pooled 3x2x6 = 36
ONE = C.CnnSpec(img=(6, 6, 3), conv=(4,), fc=(5,))                # a single convolution, a single linear layer


def _problem(spec, B, seed, scale=0.7):
    rng = np.random.default_rng(seed)
    offs, P = spec.offsets()
    theta = rng.standard_normal(P) * scale / 3.0
    x = rng.standard_normal((B,) + spec.img)
    y = rng.integers(0, spec.fc[-1], size=B)
    return theta, x, y, P


def test_offsets_and_sizes():
    spec = C.CnnSpec(img=(28, 28, 1), conv=(32, 64), fc=(128, 10))
    offs, P = spec.offsets()
    assert spec.conv_shapes() == [(28, 28, 1), (26, 26, 32), (24, 24, 64)] and spec.flat == 9216
    assert P == 32 * 9 + 32 + 64 * 288 + 64 + 9216 * 128 + 128 + 1280 + 10 == 1199882
    assert offs[0][:2] == (0, 288) and offs[1][0] == 320 and offs[2][0] == 320 + 18432 + 64


def test_convolution_is_cross_correlation():
    rng = np.random.default_rng(0)
    a = rng.standard_normal((2, 7, 9, 3)); W = rng.standard_normal((4, 3, 3, 3))
    s = C.conv3x3(a, W)
    assert s.shape == (2, 5, 7, 4)
    for b in range(2):
        for co in range(4):
            want = sum(correlate2d(a[b, :, :, ci], W[co, ci], mode="valid") for ci in range(3))
            np.testing.assert_allclose(s[b, :, :, co], want, rtol=1e-12, atol=1e-12)


def test_convolution_adjoints():
    rng = np.random.default_rng(1)
    a = rng.standard_normal((3, 6, 5, 2)); W = rng.standard_normal((4, 2, 3, 3)); d = rng.standard_normal((3, 4, 3, 4))
    lhs = np.sum(C.conv3x3(a, W) * d)
    assert abs(lhs - np.sum(a * C.conv3x3_input_grad(d, W))) < 1e-11 * abs(lhs) + 1e-12
    assert abs(lhs - np.sum(W * C.conv3x3_weight_grad(d, a))) < 1e-11 * abs(lhs) + 1e-12


def test_maxpool_selection_ties_and_adjoint():
    a = np.zeros((1, 4, 4, 1))
    a[0, :, :, 0] = [[1, 5, 2, 2], [3, 4, 2, 2], [0, 0, 7, 1], [0, 0, 1, 9]]
    p, idx = C.maxpool2(a)
    assert p[0, :, :, 0].tolist() == [[5, 2], [0, 9]]
    assert idx[0, :, :, 0].tolist() == [[1, 0], [0, 3]]             # ties: the first of the four
    rng = np.random.default_rng(2)
    b = rng.standard_normal((2, 4, 6, 3)); d = rng.standard_normal((2, 2, 3, 3))
    _, idx = C.maxpool2(b)
    assert abs(np.sum(C.pool_select(b, idx) * d) - np.sum(b * C.unpool2(d, idx))) < 1e-12
    tp = F.max_pool2d(torch.from_numpy(b).permute(0, 3, 1, 2), 2).permute(0, 2, 3, 1).numpy()
    np.testing.assert_array_equal(C.maxpool2(b)[0], tp)


def test_loss_at_zero_weights_is_log_classes():
    _, x, y, P = _problem(SMALL, 4, 3)
    assert abs(C.loss_only(np.zeros(P), x, y, SMALL) - math.log(5)) < 1e-14
    loss, g, _, _ = C.grad_and_hvp(np.zeros(P), x, y, SMALL)
    assert abs(loss - math.log(5)) < 1e-14


@pytest.mark.parametrize("spec,B,seed", [(TINY, 3, 4), (ONE, 2, 5)])
def test_gradient_matches_finite_difference_of_loss(spec, B, seed):
    theta, x, y, P = _problem(spec, B, seed)
    loss, g, _, margin = C.grad_and_hvp(theta, x, y, spec)
    assert margin > 1e-4 and abs(loss - C.loss_only(theta, x, y, spec)) < 1e-14
    h = 1e-6
    for j in range(P):
        e = np.zeros(P); e[j] = h
        fd = (C.loss_only(theta + e, x, y, spec) - C.loss_only(theta - e, x, y, spec)) / (2 * h)
        assert abs(fd - g[j]) < 1e-7 * max(1.0, abs(g[j])), j


@pytest.mark.parametrize("spec,B,seed", [(TINY, 3, 6), (ONE, 2, 11)])
def test_hvp_matches_finite_difference_of_gradient_and_is_symmetric(spec, B, seed):
    theta, x, y, P = _problem(spec, B, seed)
    rng = np.random.default_rng(seed + 100)
    z = rng.choice([-1.0, 1.0], size=P); w = rng.standard_normal(P)
    _, _, hz, margin = C.grad_and_hvp(theta, x, y, spec, z)
    assert margin > 1e-3
    h = 1e-5
    gp = C.grad_and_hvp(theta + h * z, x, y, spec)[1]; gm = C.grad_and_hvp(theta - h * z, x, y, spec)[1]
    np.testing.assert_allclose(hz, (gp - gm) / (2 * h), rtol=2e-6, atol=2e-8)
    hw = C.grad_and_hvp(theta, x, y, spec, w)[2]
    assert abs(z @ hw - w @ hz) < 1e-10 * (abs(z @ hw) + 1.0)


def _torch_net(theta_t, x_t, y_t, spec):
    offs, _ = spec.offsets()
    a = x_t.permute(0, 3, 1, 2)
    nc = len(spec.conv)
    for j in range(nc):
        w, b, shape = offs[j]
        a = F.relu(F.conv2d(a, theta_t[w:b].reshape(shape), theta_t[b:b + shape[0]]))
    a = F.max_pool2d(a, 2).permute(0, 2, 3, 1).reshape(x_t.shape[0], -1)
    for l in range(len(spec.fc)):
        w, b, shape = offs[nc + l]
        a = F.linear(a, theta_t[w:b].reshape(shape), theta_t[b:b + shape[0]])
        if l < len(spec.fc) - 1:
            a = F.relu(a)
    return F.cross_entropy(a, y_t)


@pytest.mark.parametrize("spec,B,seed", [(SMALL, 5, 8), (C.CnnSpec(img=(12, 12, 1), conv=(3, 5), fc=(7, 4)), 4, 9)])
def test_gradient_and_hvp_match_torch_autograd(spec, B, seed):
    theta, x, y, P = _problem(spec, B, seed)
    z = np.random.default_rng(seed + 50).choice([-1.0, 1.0], size=P)
    loss, g, hz, margin = C.grad_and_hvp(theta, x, y, spec, z)
    assert margin > 1e-6
    th = torch.from_numpy(theta).requires_grad_(True)
    lt = _torch_net(th, torch.from_numpy(x), torch.from_numpy(y), spec)
    (gt,) = torch.autograd.grad(lt, th, create_graph=True)
    (hzt,) = torch.autograd.grad(gt, th, grad_outputs=torch.from_numpy(z))
    assert abs(loss - lt.item()) < 1e-12
    np.testing.assert_allclose(g, gt.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(hz, hzt.numpy(), rtol=1e-9, atol=1e-11)


def test_spatial_average_is_the_window_mean_for_kernels_only():
    offs, P = SMALL.offsets()
    D = np.random.default_rng(10).standard_normal(P)
    A = C.spatial_average(D, SMALL)
    for j in range(2):
        w, b, shape = offs[j]
        want = D[w:b].reshape(shape[0], shape[1], 9).mean(axis=2)
        got = A[w:b].reshape(shape[0], shape[1], 9)
        np.testing.assert_allclose(got, np.repeat(want[:, :, None], 9, axis=2), rtol=1e-15)
        np.testing.assert_array_equal(A[b:b + shape[0]], D[b:b + shape[0]])          # biases untouched
    w = offs[2][0]
    np.testing.assert_array_equal(A[w:], D[w:])                                       # linear layers untouched
    const = np.ones(P)
    np.testing.assert_array_equal(C.spatial_average(const, SMALL), const)
