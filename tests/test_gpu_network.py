"""GPU parity of the network part (gradient and Hessian-vector product) and of whole trajectories."""
import numpy as np
import pytest
import torch

from oracle import dw_oracle as O
from paper_2409_09242_amd import binding as B
from paper_2409_09242_amd import workloads as W
from parity import RTOL_GRAD, RTOL_HV, RTOL_UPDATE, close, close_layers, oracle_config

pytestmark = pytest.mark.gpu


def _setup(w):
    theta0 = W.init_theta(w.dims, w.seed)
    h = B.Handle(B.config_from_workload(w), theta0)
    tr = O.OracleTrainer(oracle_config(w), theta0.astype(np.float64))
    return h, tr, theta0


SHAPES = [
    # dims, batch, k  -- chosen to cover every tile shape, several tiles and ragged tails
    ((32, 64, 10), 16, 4),
    ((36, 10), 7, 2),                      # no hidden layer: softmax regression
    ((200, 136, 72, 10), 150, 2),
    ((64, 260, 132, 12), 70, 3),
    ((256, 1024, 1024, 10), 160, 8),       # large tiles
    ((48, 40, 36, 28, 24, 4), 33, 2),      # deep and narrow
]


@pytest.mark.parametrize("dims,batch,k", SHAPES)
def test_gradient_and_hvp_match_the_oracle(dims, batch, k):
    w = W.scaled(W.C1, dims=dims, batch=batch, k=k, seed=1000 + batch)
    h, tr, theta0 = _setup(w)
    x, y = W.minibatch_pool(w, 1)
    loss = torch.zeros(k, device="cuda")
    h.worker_step(torch.from_numpy(x[0]).cuda(), torch.from_numpy(y[0]).cuda(), loss=loss)
    ref_loss = tr.worker_step(x[0], y[0])
    margin = min(t.min_abs_preact for t in tr.traces)
    print("kink margin", margin)
    close(loss.cpu().numpy(), ref_loss, 1e-5, "loss")
    for i in range(k):
        z = O.words_to_u32(O.rademacher_words(w.seed, i, 0, w.P))
        np.testing.assert_array_equal(h.get_state(B.DW_S_ZBITS, i), z)
        close_layers(h.get_state(B.DW_S_G, i), tr.traces[i].g, dims, RTOL_GRAD, "g[%d]" % i)
        close_layers(h.get_state(B.DW_S_HZ, i), tr.traces[i].hz, dims, RTOL_HV, "hz[%d]" % i)
        upd = h.get_state(B.DW_S_THETA, i) - theta0
        close_layers(upd, tr.theta[i] - theta0.astype(np.float64), dims, RTOL_UPDATE, "update[%d]" % i)


def test_caller_supplied_z_and_frozen_worker():
    w = W.scaled(W.C1, dims=(40, 48, 8), batch=21, k=3, seed=31)
    h, tr, theta0 = _setup(w)
    x, y = W.minibatch_pool(w, 1)
    rng = W.rng_for(5, 29)
    words = rng.integers(0, 2 ** 63, size=(3, (w.P + 63) // 64), dtype=np.uint64)
    zb = np.stack([O.words_to_u32(words[i]) for i in range(3)])
    zs = np.stack([O.words_to_signs(words[i], w.P) for i in range(3)])
    active = [1, 0, 1]
    h.worker_step(torch.from_numpy(x[0]).cuda(), torch.from_numpy(y[0]).cuda(),
                  zbits=torch.from_numpy(zb.view(np.int32)).cuda(), active=active)
    tr.worker_step(x[0], y[0], z_signs=zs, active=active)
    for i in (0, 2):
        close_layers(h.get_state(B.DW_S_HZ, i), tr.traces[i].hz, w.dims, RTOL_HV, "hz[%d]" % i)
        close_layers(h.get_state(B.DW_S_THETA, i) - theta0, tr.theta[i] - theta0, w.dims, RTOL_UPDATE, "upd")
    np.testing.assert_array_equal(h.get_state(B.DW_S_THETA, 1), theta0)
    assert int(h.get_state(B.DW_S_STEPS, 1)[0]) == 0


def _run_trajectory(w, steps, rtol_scale=1.0):
    h, tr, theta0 = _setup(w)
    n_pool = 4
    x, y = W.minibatch_pool(w, n_pool)
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    sched = W.participation_schedule(w, steps // w.tau + 1)
    rounds = 0
    for step in range(1, steps + 1):
        b = (step - 1) % n_pool
        prev = tr.theta.copy()
        prev_gpu = h.all_state(B.DW_S_THETA)
        h.worker_step(xd[b], yd[b])
        tr.worker_step(x[b], y[b])
        margin = min(t.min_abs_preact for t in tr.traces)
        now_gpu = h.all_state(B.DW_S_THETA)
        for i in range(w.k):
            close_layers(now_gpu[i] - prev_gpu[i], tr.theta[i] - prev[i], w.dims, RTOL_UPDATE * rtol_scale,
                         "step %d update[%d] (kink margin %.2e)" % (step, i, margin))
        part = sched[rounds]
        did = h.elastic_sync(B.DW_DYNAMIC, tau=w.tau, participate=part)
        assert did == tr.elastic_sync(O.MODE_DYNAMIC, tau=w.tau, participate=part)
        if did:
            rounds += 1
            for i in range(w.k):
                sc = h.get_state(B.DW_S_SCORE, i)
                assert abs(sc[2] - tr.last_h1[i]) < 1e-3 and abs(sc[3] - tr.last_h2[i]) < 1e-3, (step, i, sc)
            close(h.get_state(B.DW_S_CENTRE), tr.centre, RTOL_UPDATE * rtol_scale * 10, "centre after round %d" % rounds)
    for i in range(w.k):
        close(h.get_state(B.DW_S_THETA, i), tr.theta[i], 1e-3, "final theta[%d]" % i)
    return h, tr


def test_trajectory_c1_tiny():
    _run_trajectory(W.C1, W.C1.steps)


def test_trajectory_c2():
    _run_trajectory(W.C2, W.C2.steps)
