"""GPU parity of the data side: the overlap partition (Section V-A) and the minibatch draws, against the
oracle, bit for bit (index work); the library is called through its C ABI."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import dw_data as OD
from paper_2409_09242_amd import binding as B
from paper_2409_09242_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("n,o,k", [
    (60000, 7500, 8),        # the paper's data set size with r = 12.5 % and 8 workers
    (60000, 15000, 4),       # r = 25 % and 4 workers
    (60000, 0, 8), (60000, 30000, 4),
    (103, 10, 4),            # a remainder point goes to no worker
    (257, 1, 3), (1000, 0, 16), (16, 16, 4), (16, 0, 1), (3, 0, 8), (1, 1, 1),
    (300001, 1234, 64),      # several slices of the ranking, ragged tail, the largest k
])
def test_partition_matches_the_oracle(n, o, k):
    print("partition", n, o, k, flush=True)
    seed = 1000 + n + o
    got = B.overlap_partition(n, o, k, seed, DEV).cpu().numpy()
    want = OD.worker_datasets(n, o, k, seed)
    assert got.shape == want.shape
    np.testing.assert_array_equal(got, want)


def test_partition_rejects_bad_arguments():
    lib = B.lib()
    scratch = torch.empty(4096 + 256, dtype=torch.uint8, device=DEV)
    sp = (scratch.data_ptr() + 255) // 256 * 256
    idx = torch.empty(64, dtype=torch.int32, device=DEV)
    ip = C.c_void_p(idx.data_ptr())
    assert lib.dw_overlap_partition(0, 0, 1, 1, ip, C.c_void_p(sp), 4096, None) == -5
    assert lib.dw_overlap_partition(16, 17, 1, 1, ip, C.c_void_p(sp), 4096, None) == -5
    assert lib.dw_overlap_partition(16, 0, 0, 1, ip, C.c_void_p(sp), 4096, None) == -5
    assert lib.dw_overlap_partition(16, 0, 65, 1, ip, C.c_void_p(sp), 4096, None) == -5
    assert lib.dw_overlap_partition(16, 0, 2, 1, None, C.c_void_p(sp), 4096, None) == -1
    assert lib.dw_overlap_partition(16, 0, 2, 1, ip, C.c_void_p(sp), 16, None) == -4          # scratch too small
    assert lib.dw_overlap_partition(16, 0, 2, 1, ip, C.c_void_p(sp + 8), 4096, None) == -4     # misaligned
    assert lib.dw_overlap_partition(16, 4, 2, 1, ip, C.c_void_p(sp), 4096, None) == 6


def _bits(t):
    return t.cpu().view(torch.int16 if t.dtype == torch.bfloat16 else torch.int32).numpy()


@pytest.mark.parametrize("bf16", [False, True])
def test_draw_batch_matches_the_oracle_and_follows_the_local_steps(bf16):
    print("draw_batch bf16=%s" % bf16, flush=True)
    k, Bsz, d0, n, o = 4, 24, 64, 500, 60
    w = W.scaled(W.C1, k=k, dims=(d0, 32, 10), batch=Bsz, bf16=bf16)
    h = B.Handle(B.config_from_workload(w), W.init_theta(w.dims, w.seed), DEV)
    rng = W.rng_for(5, 1)
    data_np = rng.standard_normal((n, d0)).astype(np.float32)
    labels_np = rng.integers(0, 10, size=n).astype(np.int32)
    data = torch.from_numpy(data_np).to(DEV)
    if bf16:
        data = data.to(torch.bfloat16)
    labels = torch.from_numpy(labels_np).to(DEV)
    index = B.overlap_partition(n, o, k, 31, DEV)
    Dj = OD.worker_datasets(n, o, k, 31)
    x = torch.zeros((k, Bsz, d0), dtype=data.dtype, device=DEV)
    y = torch.full((k, Bsz), -7, dtype=torch.int32, device=DEV)
    data_bits = _bits(data)
    steps = [0] * k
    schedule = [None, [1, 0, 1, 1], [1, 1, 0, 1], None, [0, 0, 0, 1]]
    for active in schedule:
        act = [1] * k if active is None else active
        before_x, before_y = _bits(x).copy(), y.cpu().numpy().copy()
        h.draw_batch(data, labels, index, 77, x, y, active=active)
        torch.cuda.synchronize()
        gx, gy = _bits(x), y.cpu().numpy()
        for j in range(k):
            if not act[j]:                                   # a frozen worker's rows are left alone
                np.testing.assert_array_equal(gx[j], before_x[j])
                np.testing.assert_array_equal(gy[j], before_y[j])
                continue
            idx = Dj[j][OD.batch_positions(77, j, steps[j], Bsz, Dj.shape[1])]
            np.testing.assert_array_equal(gx[j], data_bits[idx])
            np.testing.assert_array_equal(gy[j], labels_np[idx])
        h.worker_step(x, y, active=active)                   # consumes the batch, advances the active workers' steps
        for j in range(k):
            steps[j] += act[j]
        assert [int(h.get_state(B.DW_S_STEPS, j)[0]) for j in range(k)] == steps
    h.close()


def test_draw_batch_marks_indices_outside_the_data_set_and_rejects_bad_calls():
    k, Bsz, d0, n = 2, 8, 32, 40
    w = W.scaled(W.C1, k=k, dims=(d0, 16, 10), batch=Bsz)
    h = B.Handle(B.config_from_workload(w), W.init_theta(w.dims, w.seed), DEV)
    data = torch.ones((n, d0), dtype=torch.float32, device=DEV)
    labels = torch.arange(n, dtype=torch.int32, device=DEV)
    index = torch.tensor([[3, 5], [40, -1]], dtype=torch.int32, device=DEV)     # worker 1's points do not exist
    x = torch.full((k, Bsz, d0), 9.0, device=DEV)
    y = torch.zeros((k, Bsz), dtype=torch.int32, device=DEV)
    h.draw_batch(data, labels, index, 1, x, y)
    torch.cuda.synchronize()
    assert torch.all(x[0] == 1.0) and set(y[0].tolist()) <= {3, 5}
    assert torch.all(x[1] == 0.0) and torch.all(y[1] == -1)
    lib = B.lib()
    args = lambda **kw: [kw.get("h", h._h), kw.get("data", C.c_void_p(data.data_ptr())), C.c_void_p(labels.data_ptr()),
                         kw.get("n", n), C.c_void_p(index.data_ptr()), kw.get("m", 2), 1, None,
                         kw.get("x", C.c_void_p(x.data_ptr())), C.c_void_p(y.data_ptr()), None]
    assert lib.dw_draw_batch(*args(m=0)) == -5
    assert lib.dw_draw_batch(*args(m=n + 1)) == -5
    assert lib.dw_draw_batch(*args(n=0)) == -5
    assert lib.dw_draw_batch(*args(data=None)) == -1
    assert lib.dw_draw_batch(*args(x=C.c_void_p(x.data_ptr() + 4))) == -5
    flat = B.Handle(B.make_config(dims=None, k=2, n_params=64), np.zeros(64, np.float32), DEV)
    assert lib.dw_draw_batch(*args(h=flat._h)) == -7
    flat.close()
    h.close()


def test_draw_batch_at_the_largest_configuration_shape():
    """k = 16, B = 512, d_0 = 4096 in bf16 from 60000 resident points: every row and label against the oracle."""
    print("draw_batch full size", flush=True)
    w = W.C4
    k, Bsz, d0, n, o = w.k, w.batch, w.dims[0], 60000, 7500
    cfg = B.make_config(dims=(d0, 8, 10), k=k, batch=Bsz, bf16=True)          # the draw only uses k, B, d_0 and dtype
    h = B.Handle(cfg, W.init_theta((d0, 8, 10), 3), DEV)
    g = torch.Generator(device=DEV); g.manual_seed(11)
    data = torch.randn((n, d0), device=DEV, generator=g).to(torch.bfloat16)
    labels = torch.randint(0, 10, (n,), device=DEV, generator=g, dtype=torch.int32)
    index = B.overlap_partition(n, o, k, 99, DEV)
    Dj = OD.worker_datasets(n, o, k, 99)
    np.testing.assert_array_equal(index.cpu().numpy(), Dj)
    for j in range(k):
        h.set_state(B.DW_S_STEPS, j, np.array([j * 3], dtype=np.int64))
    x = torch.empty((k, Bsz, d0), dtype=torch.bfloat16, device=DEV)
    y = torch.empty((k, Bsz), dtype=torch.int32, device=DEV)
    h.draw_batch(data, labels, index, 5, x, y)
    torch.cuda.synchronize()
    lab = labels.cpu().numpy()
    for j in range(k):
        idx = Dj[j][OD.batch_positions(5, j, j * 3, Bsz, Dj.shape[1])]
        want = data[torch.from_numpy(idx).to(DEV)]
        assert torch.equal(x[j].view(torch.int16), want.view(torch.int16))
        np.testing.assert_array_equal(y[j].cpu().numpy(), lab[idx])
    h.close()


def test_draw_batch_feeds_a_convolutional_model_with_whole_images():
    from oracle import dw_cnn as OC
    spec = OC.CnnSpec(img=(10, 10, 1), conv=(4, 8), fc=(16, 10))
    k, Bsz, n = 2, 6, 50
    idx, P_lib = B.conv_param_index(spec.img, spec.conv, spec.fc)
    cfg = B.make_config(dims=(spec.flat,) + spec.fc, k=k, batch=Bsz, img=spec.img, conv=spec.conv)
    h = B.Handle(cfg, np.zeros(P_lib, dtype=np.float32), DEV)
    data = torch.rand((n, 10, 10, 1), device=DEV)
    labels = torch.randint(0, 10, (n,), device=DEV, dtype=torch.int32)
    index = B.overlap_partition(n, 10, k, 3, DEV)
    Dj = OD.worker_datasets(n, 10, k, 3)
    x = torch.zeros((k, Bsz, 10, 10, 1), device=DEV); y = torch.zeros((k, Bsz), dtype=torch.int32, device=DEV)
    h.draw_batch(data, labels, index, 8, x, y)
    torch.cuda.synchronize()
    for j in range(k):
        pos = Dj[j][OD.batch_positions(8, j, 0, Bsz, Dj.shape[1])]
        assert torch.equal(x[j], data[torch.from_numpy(pos).to(DEV)])
        np.testing.assert_array_equal(y[j].cpu().numpy(), labels.cpu().numpy()[pos])
    h.worker_step(x, y)                                       # the drawn images are a valid minibatch of the model
    torch.cuda.synchronize()
    h.close()
