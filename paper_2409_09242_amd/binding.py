"""Thin ctypes binding over libdw.so (declared in include/dw.h).

Argument marshalling only: every step of the method runs in the library's HIP kernels.  PyTorch is used
for device memory (the workspace and the caller's tensors) and for the current stream.  There is no CPU
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdw.so")

DW_MAX_LAYERS, DW_MAX_K, DW_MAX_P, DW_MAX_CLASSES, DW_MAX_CONV = 8, 64, 8, 16, 2
DW_STATIC_MAX_POINTS = 1 << 17
DW_F32, DW_BF16 = 0, 1
DW_FIXED, DW_MANUAL, DW_DYNAMIC = 0, 1, 2
DW_OPT_ADAHESSIAN, DW_OPT_SGD, DW_OPT_MOMENTUM = 0, 1, 2
DW_SEQUENTIAL = 16      # OR-ed into the mode of elastic_sync: exchanges one after the other, in index order
(DW_S_THETA, DW_S_M, DW_S_V, DW_S_G, DW_S_HZ, DW_S_CENTRE, DW_S_ZBITS, DW_S_SCORE, DW_S_U_HIST,
 DW_S_STEPS, DW_S_ZBITS_T, DW_S_COUNTERS) = range(12)
DW_S_ACT = 16

EXPORTS = ("dw_strerror", "dw_last_hip_error", "dw_param_count", "dw_workspace_bytes", "dw_init", "dw_destroy",
           "dw_worker_step", "dw_update_only", "dw_elastic_sync", "dw_get_state", "dw_set_state",
           "dw_profile", "dw_profile_read", "dw_partition_scratch_bytes", "dw_overlap_partition", "dw_draw_batch",
           "dw_overlap_partition_static")
KERNEL_CLASSES = ("rademacher", "gemm_fwd", "head", "gemm_wgrad", "gemm_dgrad", "update", "weights", "pull", "gather", "step")


class dw_config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("dims", C.c_int32 * (DW_MAX_LAYERS + 1)), ("n_params", C.c_int64),
        ("k", C.c_int32), ("batch", C.c_int32), ("dtype", C.c_int32),
        ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
        ("hpow", C.c_float), ("avg_block", C.c_int32),
        ("alpha", C.c_float), ("kappa", C.c_float), ("p", C.c_int32), ("c", C.c_float * DW_MAX_P),
        ("seed", C.c_uint64), ("n_samples", C.c_int32), ("fuse_update", C.c_int32),
        ("n_conv", C.c_int32), ("img_h", C.c_int32), ("img_w", C.c_int32), ("img_c", C.c_int32),
        ("conv_c", C.c_int32 * DW_MAX_CONV), ("conv_avg", C.c_int32),
        ("optimizer", C.c_int32), ("momentum", C.c_float),
    ]


class DwError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (status %d, hip error %d)" % (
            where, lib().dw_strerror(status).decode(), status, lib().dw_last_hip_error()))


_LIB = None


def lib() -> C.CDLL:
    """Load libdw.so once and declare the prototypes of include/dw.h."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libdw.so is missing: build it with `python -m paper_2409_09242_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    L.dw_strerror.restype = C.c_char_p; L.dw_strerror.argtypes = [i32]
    L.dw_last_hip_error.restype = i32; L.dw_last_hip_error.argtypes = []
    L.dw_param_count.restype = i32; L.dw_param_count.argtypes = [C.POINTER(dw_config), C.POINTER(i64)]
    L.dw_workspace_bytes.restype = C.c_size_t; L.dw_workspace_bytes.argtypes = [C.POINTER(dw_config)]
    L.dw_init.restype = i32
    L.dw_init.argtypes = [C.POINTER(vp), C.POINTER(dw_config), vp, C.c_size_t, vp, i32, vp]
    L.dw_destroy.restype = i32; L.dw_destroy.argtypes = [vp]
    L.dw_worker_step.restype = i32; L.dw_worker_step.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    L.dw_update_only.restype = i32; L.dw_update_only.argtypes = [vp, vp, vp, vp, vp, vp]
    L.dw_elastic_sync.restype = i32; L.dw_elastic_sync.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    L.dw_get_state.restype = i32; L.dw_get_state.argtypes = [vp, i32, i32, i64, i64, vp, vp]
    L.dw_set_state.restype = i32; L.dw_set_state.argtypes = [vp, i32, i32, i64, i64, vp, vp]
    L.dw_profile.restype = i32; L.dw_profile.argtypes = [vp, i32]
    L.dw_profile_read.restype = i32; L.dw_profile_read.argtypes = [vp, vp, vp, vp, vp]
    L.dw_partition_scratch_bytes.restype = C.c_size_t; L.dw_partition_scratch_bytes.argtypes = [i64]
    L.dw_overlap_partition.restype = i64
    L.dw_overlap_partition.argtypes = [i64, i64, i32, C.c_uint64, vp, vp, C.c_size_t, vp]
    L.dw_overlap_partition_static.restype = i64
    L.dw_overlap_partition_static.argtypes = [i64, i64, i32, C.c_uint64, vp, vp]
    L.dw_draw_batch.restype = i32
    L.dw_draw_batch.argtypes = [vp, vp, vp, i64, vp, i64, C.c_uint64, vp, vp, vp, vp]
    _LIB = L
    return L


def make_config(*, dims: Optional[Sequence[int]], k: int, batch: int = 0, bf16: bool = False, n_params: int = 0,
                lr=0.01, beta1=0.9, beta2=0.999, eps=1e-4, hpow=1.0, avg_block=1, alpha=0.1, kappa=-0.1,
                c: Sequence[float] = (0.4, 0.3, 0.2, 0.1), seed: int = 0, fuse_update: int = 0,
                n_samples: int = 1, img: Optional[Sequence[int]] = None, conv: Sequence[int] = (),
                conv_avg: int = 0, optimizer: int = DW_OPT_ADAHESSIAN, momentum: float = 0.5) -> dw_config:
    cfg = dw_config()
    if dims is None:
        cfg.n_layers = 0
        cfg.n_params = n_params
    else:
        cfg.n_layers = len(dims) - 1
        for i, d in enumerate(dims):
            cfg.dims[i] = d
        cfg.n_params = 0
    cfg.k, cfg.batch, cfg.dtype = k, batch, (DW_BF16 if bf16 else DW_F32)
    cfg.lr, cfg.beta1, cfg.beta2, cfg.eps, cfg.hpow, cfg.avg_block = lr, beta1, beta2, eps, hpow, avg_block
    cfg.alpha, cfg.kappa, cfg.p = alpha, kappa, len(c)
    for j, cj in enumerate(c):
        cfg.c[j] = cj
    cfg.seed = seed
    cfg.fuse_update = fuse_update
    cfg.n_samples = n_samples
    cfg.n_conv = len(conv)
    if conv:
        cfg.img_h, cfg.img_w, cfg.img_c = img
        for j, cj in enumerate(conv):
            cfg.conv_c[j] = cj
    cfg.conv_avg = conv_avg
    cfg.optimizer, cfg.momentum = optimizer, momentum
    return cfg


def config_from_workload(w, **overrides) -> dw_config:
    kw = dict(dims=w.dims, k=w.k, batch=w.batch, bf16=w.bf16, n_params=w.n_params if w.dims is None else 0,
              lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, hpow=w.hpow, avg_block=w.avg_block,
              alpha=w.alpha, kappa=w.kappa, c=w.c, seed=w.seed, optimizer=getattr(w, "optimizer", 0),
              momentum=getattr(w, "momentum", 0.5))
    if getattr(w, "conv", ()):
        kw.update(img=w.img, conv=w.conv, conv_avg=w.conv_avg)
    kw.update(overrides)
    return make_config(**kw)


def conv_param_index(img: Sequence[int], conv: Sequence[int], fc: Sequence[int]):
    """Where the parameters of a convolutional model sit in the library's layout.

    Returns (idx, P_lib): idx[j] is the library position of parameter j of the unpadded layout (kernels
    [C_out][C_in][3][3] and biases of the convolutions, then W_l, b_l of the linear layers); the library rows of a
    kernel run over (tap, input channel) and are padded to a multiple of 4 entries, which adds zeros that never
    change (see dw_config.n_conv)."""
    h, w, c_in = img
    idx, pos = [], 0
    for co in conv:
        K = (9 * c_in + 3) // 4 * 4
        # unpadded entry (co, ci, tap) -> library entry co*K + tap*C_in + ci
        rows = pos + np.arange(co)[:, None, None] * K + np.arange(c_in)[None, :, None] + np.arange(9)[None, None, :] * c_in
        idx.append(rows.reshape(-1)); pos += co * K
        idx.append(pos + np.arange(co)); pos += co
        h, w, c_in = h - 2, w - 2, co
    d_in = (h // 2) * (w // 2) * c_in
    for d in fc:
        n = d * d_in + d
        idx.append(pos + np.arange(n)); pos += n
        d_in = d
    return np.concatenate(idx).astype(np.int64), pos


def param_count(cfg: dw_config) -> int:
    n = C.c_int64(0)
    st = lib().dw_param_count(C.byref(cfg), C.byref(n))
    if st != 0:
        raise DwError(st, "dw_param_count")
    return n.value


def _u8(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.uint8))


def _ptr(a):
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        return a.ctypes.data_as(C.c_void_p)
    return C.c_void_p(a.data_ptr())        # torch tensor


def overlap_partition(n: int, o: int, k: int, seed: int, device="cuda:0"):
    """Section V-A on the device: an int32 tensor [k][o + floor((n-o)/k)], row j = D_j (O first)."""
    import torch
    dev = torch.device(device)
    nbytes = lib().dw_partition_scratch_bytes(n)
    if nbytes == 0:
        raise DwError(-5, "dw_partition_scratch_bytes")
    scratch = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
    sp = (scratch.data_ptr() + 255) // 256 * 256
    m = o + (n - o) // k if 0 <= o <= n and k >= 1 else 0
    index = torch.empty((max(k, 1), max(m, 0)), dtype=torch.int32, device=dev)
    stream = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    s = lib().dw_overlap_partition(n, o, k, seed, C.c_void_p(index.data_ptr()) if index.numel() else None,
                                   C.c_void_p(sp), nbytes, stream)
    if s < 0:
        raise DwError(int(s), "dw_overlap_partition")
    torch.cuda.current_stream(dev).synchronize()          # the scratch tensor goes away with this frame
    return index


def overlap_partition_static(n: int, o: int, k: int, seed: int, index) -> int:
    """dw_overlap_partition_static into a caller-allocated int32 tensor [k][o + floor((n-o)/k)]; returns floor((n-o)/k).
    Nothing is allocated here or in the library; the work is enqueued on the current stream of the tensor's device."""
    import torch
    stream = C.c_void_p(torch.cuda.current_stream(index.device).cuda_stream)
    s = lib().dw_overlap_partition_static(n, o, k, seed, C.c_void_p(index.data_ptr()) if index.numel() else None, stream)
    if s < 0:
        raise DwError(int(s), "dw_overlap_partition_static")
    return int(s)


class Handle:
    """One master + k workers on the current CUDA device; owns the workspace tensor."""

    def __init__(self, cfg: dw_config, theta0, device="cuda:0"):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.k = cfg.k
        self.P = param_count(cfg)
        self.zwords = 2 * ((self.P + 63) // 64)
        nbytes = lib().dw_workspace_bytes(C.byref(cfg))
        if nbytes == 0:
            raise DwError(-2, "dw_workspace_bytes")
        self.device = torch.device(device)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        self._h = C.c_void_p()
        if isinstance(theta0, np.ndarray):
            t0 = np.ascontiguousarray(theta0, dtype=np.float32)
            assert t0.shape == (self.P,)
            st = lib().dw_init(C.byref(self._h), C.byref(cfg), self._ws_ptr, nbytes, _ptr(t0), 0, self._stream())
        else:
            assert theta0.is_cuda and theta0.dtype == torch.float32 and theta0.numel() == self.P
            st = lib().dw_init(C.byref(self._h), C.byref(cfg), self._ws_ptr, nbytes, _ptr(theta0), 1, self._stream())
        if st != 0:
            raise DwError(st, "dw_init")

    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def close(self):
        if self._h:
            lib().dw_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the three hot calls -------------------------------------------------------------------------
    def worker_step(self, x, y, zbits=None, active=None, loss=None):
        act = _u8(active)
        st = lib().dw_worker_step(self._h, _ptr(x), _ptr(y), _ptr(zbits), _ptr(act), _ptr(loss), self._stream())
        if st != 0:
            raise DwError(st, "dw_worker_step")

    def update_only(self, g, hz, zbits=None, active=None):
        act = _u8(active)
        st = lib().dw_update_only(self._h, _ptr(g), _ptr(hz), _ptr(zbits), _ptr(act), self._stream())
        if st != 0:
            raise DwError(st, "dw_update_only")

    def elastic_sync(self, mode=DW_DYNAMIC, tau=1, h1=None, h2=None, participate=None) -> bool:
        a1 = None if h1 is None else np.ascontiguousarray(h1, dtype=np.float32)
        a2 = None if h2 is None else np.ascontiguousarray(h2, dtype=np.float32)
        part = _u8(participate)
        st = lib().dw_elastic_sync(self._h, mode, _ptr(a1), _ptr(a2), _ptr(part), tau, self._stream())
        if st < 0:
            raise DwError(st, "dw_elastic_sync")
        return st == 1

    def draw_batch(self, data, labels, index, seed: int, x, y, active=None):
        """Fill x [k][B][d0], y [k][B] with every active worker's minibatch at its current local step."""
        act = _u8(active)
        st = lib().dw_draw_batch(self._h, _ptr(data), _ptr(labels), data.shape[0], _ptr(index), index.shape[1], seed,
                                 _ptr(act), _ptr(x), _ptr(y), self._stream())
        if st != 0:
            raise DwError(st, "dw_draw_batch")

    # ---- state access --------------------------------------------------------------------------------
    _DT = {DW_S_ZBITS: np.uint32, DW_S_ZBITS_T: np.uint32, DW_S_SCORE: np.float64, DW_S_U_HIST: np.float64, DW_S_STEPS: np.int64,
           DW_S_COUNTERS: np.int64}

    def get_state(self, what: int, worker: int = 0, offset: int = 0, count: Optional[int] = None) -> np.ndarray:
        if what > DW_S_ACT:
            l = what - DW_S_ACT
            n = self.cfg.batch * self.cfg.dims[l]
            out = np.empty(n, dtype=np.uint16 if self.cfg.dtype == DW_BF16 else np.float32)
            st = lib().dw_get_state(self._h, what, worker, 0, n, _ptr(out), self._stream())
            if st != 0:
                raise DwError(st, "dw_get_state")
            return out.reshape(self.cfg.batch, self.cfg.dims[l])
        if count is None:
            count = {DW_S_ZBITS: self.zwords, DW_S_ZBITS_T: self.zwords, DW_S_SCORE: 4, DW_S_U_HIST: 2 + DW_MAX_P, DW_S_STEPS: 1,
                     DW_S_COUNTERS: 3}.get(
                what, self.P) - offset
        out = np.empty(count, dtype=self._DT.get(what, np.float32))
        st = lib().dw_get_state(self._h, what, worker, offset, count, _ptr(out), self._stream())
        if st != 0:
            raise DwError(st, "dw_get_state")
        return out

    def set_state(self, what: int, worker: int, values, offset: int = 0):
        arr = np.ascontiguousarray(values, dtype=self._DT.get(what, np.float32))
        st = lib().dw_set_state(self._h, what, worker, offset, arr.size, _ptr(arr), self._stream())
        if st != 0:
            raise DwError(st, "dw_set_state")

    # ---- per-kernel timing -----------------------------------------------------------------------------
    def profile(self, enable: bool):
        st = lib().dw_profile(self._h, 1 if enable else 0)
        if st != 0:
            raise DwError(st, "dw_profile")

    def profile_read(self) -> dict:
        """{class name: (launches, total ms)} since the last read; synchronises the stream."""
        n = np.zeros(len(KERNEL_CLASSES), dtype=np.int64)
        ms = np.zeros(len(KERNEL_CLASSES), dtype=np.float64)
        dropped = np.zeros(1, dtype=np.int64)
        st = lib().dw_profile_read(self._h, _ptr(n), _ptr(ms), _ptr(dropped), self._stream())
        if st != 0:
            raise DwError(st, "dw_profile_read")
        out = {name: (int(n[i]), float(ms[i])) for i, name in enumerate(KERNEL_CLASSES)}
        out["dropped"] = int(dropped[0])
        return out

    def all_state(self, what: int) -> np.ndarray:
        return np.stack([self.get_state(what, i) for i in range(self.k)])

    # ---- checkpoint: plain copies through dw_get_state / dw_set_state ------------------------------------
    def checkpoint(self) -> dict:
        """Everything a run needs to go on elsewhere: parameters, moments and step counts of every worker, the
        centre, the handle's counters and every worker's history of u."""
        return {"theta": self.all_state(DW_S_THETA), "m": self.all_state(DW_S_M), "v": self.all_state(DW_S_V),
                "centre": self.get_state(DW_S_CENTRE), "steps": self.all_state(DW_S_STEPS),
                "counters": self.get_state(DW_S_COUNTERS), "u_hist": self.all_state(DW_S_U_HIST)}

    def restore(self, ck: dict):
        """Put a checkpoint into this handle (created with the same configuration); the counters go in before the
        histories, as dw_set_state asks."""
        self.set_state(DW_S_COUNTERS, 0, ck["counters"])
        for i in range(self.k):
            self.set_state(DW_S_THETA, i, ck["theta"][i])
            self.set_state(DW_S_M, i, ck["m"][i])
            self.set_state(DW_S_V, i, ck["v"][i])
            self.set_state(DW_S_STEPS, i, ck["steps"][i])
            self.set_state(DW_S_U_HIST, i, ck["u_hist"][i])
        self.set_state(DW_S_CENTRE, 0, ck["centre"])
