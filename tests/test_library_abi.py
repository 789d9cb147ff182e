"""CPU-only checks of the C-ABI library: it loads, exports what include/dw.h declares, and validates
configurations on the host (no kernel is launched here)."""
import ctypes as C
import os
import re
import shutil
import subprocess

import numpy as np
import pytest

from paper_2409_09242_amd import binding as B
from paper_2409_09242_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "dw.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dw_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared()
    assert set(names) == set(B.EXPORTS), names
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_and_param_count():
    lib = B.lib()
    assert lib.dw_strerror(0) == b"ok"
    assert b"workspace" in lib.dw_strerror(-4)
    for w in (W.C1, W.C2, W.C3, W.C4, W.C5):
        cfg = B.config_from_workload(w)
        assert B.param_count(cfg) == w.P
        assert lib.dw_workspace_bytes(C.byref(cfg)) > 4 * w.P * w.k * 3


@pytest.mark.parametrize("field,value,status", [
    ("k", 0, -2), ("k", 65, -2), ("batch", 0, -2), ("dtype", 7, -2), ("fuse_update", 2, -2), ("n_samples", 9, -2), ("n_samples", -1, -2),
    ("lr", 0.0, -3), ("beta1", 1.0, -3), ("eps", 0.0, -3), ("avg_block", 3, -3), ("avg_block", 512, -3),
    ("alpha", 0.0, -3), ("alpha", 1.5, -3), ("kappa", 0.0, -3), ("kappa", 0.2, -3), ("p", 0, -3), ("p", 9, -3),
])
def test_bad_config_is_rejected(field, value, status):
    cfg = B.config_from_workload(W.C1)
    setattr(cfg, field, value)
    n = C.c_int64()
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == status
    assert B.lib().dw_workspace_bytes(C.byref(cfg)) == 0


def test_bad_dims_and_weights():
    n = C.c_int64()
    cfg = B.make_config(dims=(30, 64, 10), k=2, batch=4)            # d_0 not a multiple of 4
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == -2
    cfg = B.make_config(dims=(32, 64, 17), k=2, batch=4)            # too many classes
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == -2
    cfg = B.make_config(dims=(32, 64, 10), k=2, batch=4, bf16=True)
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == 0
    cfg = B.make_config(dims=(36, 64, 10), k=2, batch=4, bf16=True)  # bf16 needs multiples of 8
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == -2
    cfg = B.make_config(dims=(32, 64, 10), k=2, batch=4, c=(0.5, 0.4))   # weights must sum to one
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == -3
    cfg = B.make_config(dims=(32, 48, 10), k=2, batch=4, avg_block=32)   # block must divide fan-in 48
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == -3
    cfg = B.make_config(dims=None, k=2, n_params=1002)                    # flat P must be a multiple of 4
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == -2
    assert B.lib().dw_param_count(None, C.byref(n)) == -1


def test_null_handles_are_rejected_without_a_gpu():
    lib = B.lib()
    assert lib.dw_destroy(None) == -1
    assert lib.dw_worker_step(None, None, None, None, None, None, None) == -1
    assert lib.dw_elastic_sync(None, 0, None, None, None, 1, None) == -1
    h = C.c_void_p()
    cfg = B.config_from_workload(W.C1)
    assert lib.dw_init(C.byref(h), C.byref(cfg), None, 0, None, 0, None) == -1


def test_fused_update_is_an_option_of_large_layers_only():
    """fuse_update = 1 is accepted everywhere; it only adds partial-sum slots (workspace) where a layer qualifies."""
    lib = B.lib()
    for w in (W.C1, W.C3, W.C4):
        plain = lib.dw_workspace_bytes(C.byref(B.config_from_workload(w)))
        fused = lib.dw_workspace_bytes(C.byref(B.config_from_workload(w, fuse_update=1)))
        assert plain > 0
        if w is W.C4:
            # three 4096 x 4096 layers, 32 x 32 tiles of 128 x 128 each, one double per tile and worker
            assert fused - plain == 3 * 32 * 32 * 8 * w.k
        elif w is W.C3:
            # fp32: 1024 x 3072 and two 1024 x 1024 layers in 128 x 128 tiles, one double per tile and worker
            assert fused - plain == (8 * 24 + 2 * 8 * 8) * 8 * w.k
        else:
            assert fused == plain


def test_two_probes_with_fused_bf16_layers_keep_the_earlier_probe():
    """n_samples = 2 in bf16 with fused layers: the fused weight-gradient kernels take both probes in one launch, so the
    workspace holds the earlier probe's sign bits and its Ra_l, Rd_l of the hidden layers next to the later probe's.
    Three probes (running sum through memory) and the unfused handle have no such buffers."""
    lib = B.lib()
    w = W.C4

    def size(**kw):
        return lib.dw_workspace_bytes(C.byref(B.config_from_workload(w, **kw)))

    def up(n, a):
        return (n + a - 1) // a * a
    z_bytes = w.k * up(2 * ((w.P + 63) // 64), 64) * 4
    hidden = sum(2 * up(w.k * w.batch * d * 2, 256) for d in w.dims[1:-1])
    assert size(n_samples=2, fuse_update=1) - size(n_samples=3, fuse_update=1) == up(z_bytes, 256) + hidden
    assert size(n_samples=2) == size(n_samples=3)


def test_participation_schedules():
    """Host-side recipes of the failure patterns (Section VI: communication suppressed, here per round)."""
    w = W.scaled(W.C2, k=6, stale="third", seed=4)
    p = W.participation_schedule(w, 6000)
    assert p.shape == (6000, 6) and p.dtype == np.uint8 and set(np.unique(p)) == {0, 1}
    assert abs(p.mean() - 2.0 / 3.0) < 0.02                       # suppressed one third of the time
    assert np.array_equal(p, W.participation_schedule(w, 6000))   # seeded
    assert np.all(np.abs(p.mean(axis=0) - 2.0 / 3.0) < 0.03)      # every worker alike
    f = W.participation_schedule(W.scaled(W.C3, k=5), 8)
    assert f[:, :3].all() and list(f[:, 3]) == [0, 0, 0, 1, 0, 0, 0, 1] and list(f[:, 4]) == list(f[:, 3])
    g = W.participation_schedule(W.C4, 400)
    # absent for Geometric(0.3) - 1 rounds (7/3 on average) after each turn: present 3 rounds in 10
    assert g.shape == (400, 16) and 0.25 < g.mean() < 0.35
    assert W.participation_schedule(W.C1, 3).all()


def test_data_calls_validate_on_the_host():
    lib = B.lib()
    assert lib.dw_partition_scratch_bytes(0) == 0
    assert lib.dw_partition_scratch_bytes((1 << 21) + 1) == 0
    assert lib.dw_partition_scratch_bytes(60000) >= 60000 * 12
    assert lib.dw_partition_scratch_bytes(60000) % 256 == 0
    # argument errors are reported before anything touches a device
    assert lib.dw_overlap_partition(0, 0, 1, 1, None, None, 0, None) == -5
    assert lib.dw_overlap_partition(10, 11, 1, 1, None, None, 0, None) == -5
    assert lib.dw_overlap_partition(10, 0, 65, 1, None, None, 0, None) == -5
    assert lib.dw_overlap_partition(10, 0, 2, 1, None, None, 0, None) == -1
    assert lib.dw_draw_batch(None, None, None, 1, None, 1, 0, None, None, None, None) == -1


def test_convolutional_configuration_is_validated_on_the_host():
    n = C.c_int64()
    ok = dict(dims=(72, 16, 10), k=2, batch=4, img=(10, 10, 1), conv=(4, 8))
    cfg = B.make_config(**ok)
    assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == 0
    idx, P_lib = B.conv_param_index((10, 10, 1), (4, 8), (16, 10))
    assert n.value == P_lib == 4 * 12 + 4 + 8 * 36 + 8 + 72 * 16 + 16 + 160 + 10
    assert idx.size == 4 * 9 + 4 + 8 * 36 + 8 + 72 * 16 + 16 + 160 + 10 and len(set(idx.tolist())) == idx.size
    assert idx[:10].tolist() == [0, 1, 2, 3, 4, 5, 6, 7, 8, 12]        # three padding entries after nine taps
    second = 4 * 12 + 4                                                # the second kernel: rows of 9 taps x 4 channels
    assert idx[40:50].tolist() == [second + t * 4 for t in range(9)] + [second + 1]
    assert B.lib().dw_workspace_bytes(C.byref(cfg)) > 0
    for kw in (dict(ok, dims=(64, 16, 10)), dict(ok, conv=(4, 6)), dict(ok, img=(9, 10, 1)), dict(ok, bf16=True)):
        assert B.lib().dw_param_count(C.byref(B.make_config(**kw)), C.byref(n)) == -2


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")
def test_header_is_plain_c_and_a_c_program_can_call_the_library(tmp_path):
    """include/dw.h compiles as C99, and a C program linked against the library reaches the host-side calls."""
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                    os.path.join(inc, "dw.h")], check=True)
    libdir = os.path.dirname(B.LIB_PATH)
    src = tmp_path / "use_dw.c"
    src.write_text(
        '#include <stdio.h>\n#include <string.h>\n#include "dw.h"\n'
        'int main(void) {\n'
        '  dw_config c; memset(&c, 0, sizeof c);\n'
        '  c.n_layers = 2; c.dims[0] = 32; c.dims[1] = 64; c.dims[2] = 10; c.k = 4; c.batch = 16; c.dtype = DW_F32;\n'
        '  c.lr = 0.01f; c.beta1 = 0.9f; c.beta2 = 0.999f; c.eps = 1e-4f; c.hpow = 1.0f; c.avg_block = 1;\n'
        '  c.alpha = 0.1f; c.kappa = -0.1f; c.p = 1; c.c[0] = 1.0f; c.seed = 1;\n'
        '  int64_t n = 0; int st = dw_param_count(&c, &n);\n'
        '  printf("%d %lld %s %zu\\n", st, (long long)n, dw_strerror(DW_ERR_WORKSPACE), dw_workspace_bytes(&c));\n'
        '  c.k = 0; return dw_param_count(&c, &n) == DW_ERR_CONFIG ? 0 : 1;\n}\n')
    exe = tmp_path / "use_dw"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-l:" +
                    os.path.basename(B.LIB_PATH), "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out[0] == "0" and int(out[1]) == 32 * 64 + 64 + 64 * 10 + 10 and int(out[-1]) > 0


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")
def test_binding_lays_the_configuration_out_as_the_header_does(tmp_path):
    """The ctypes mirror of dw_config against the C compiler's own layout of the header's struct: size and the offset
    of every field."""
    names = [f[0] for f in B.dw_config._fields_]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "dw.h"\nint main(void) {\n'
                   '  printf("%zu\\n", sizeof(dw_config));\n' +
                   "".join('  printf("%%zu\\n", offsetof(dw_config, %s));\n' % n for n in names) + "  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = [int(v) for v in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert out[0] == C.sizeof(B.dw_config)
    assert out[1:] == [getattr(B.dw_config, n).offset for n in names]


def test_baseline_optimizers_are_validated_on_the_host():
    n = C.c_int64()
    for kw, status in ((dict(optimizer=B.DW_OPT_SGD), 0), (dict(optimizer=B.DW_OPT_MOMENTUM, momentum=0.5), 0),
                       (dict(optimizer=3), -2), (dict(optimizer=B.DW_OPT_MOMENTUM, momentum=1.0), -3),
                       (dict(optimizer=B.DW_OPT_SGD, fuse_update=1), -2), (dict(optimizer=B.DW_OPT_SGD, n_samples=2), -2)):
        cfg = B.make_config(dims=(32, 64, 10), k=2, batch=4, **kw)
        assert B.lib().dw_param_count(C.byref(cfg), C.byref(n)) == status, kw


def test_transposed_lds_reads_are_not_touched_before_their_wait():
    """The data-gradient kernel reads LDS with transpose reads issued from inline assembly; the build checks in the
    kernels' own assembly that nothing touches their destination registers before the wait for LDS.  Here: the
    checker finds a planted copy, and the assembly of the current sources is clean."""
    from paper_2409_09242_amd import build as BLD
    planted = ("\n_ZN2dw4b16d18dual_gemm_bf16_dmaILb1ELb1ELb0EEEvNS_8GemmArgsE: ; @kernel\n"
               "\tds_read_b64_tr_b16 v[60:61], v7\n\tv_mfma_f32_32x32x16_bf16 a[0:15], v[2:5], v[8:11], a[0:15]\n"
               "\tv_mov_b32_e32 v14, v60\n\ts_waitcnt lgkmcnt(0)\n\tv_mov_b32_e32 v15, v61\n\ts_endpgm\n")
    found, n = BLD.premature_uses_of_transposed_reads(planted)
    assert n == 1 and [f[2] for f in found] == ["v_mov_b32_e32 v14, v60"]
    asm = os.path.join(BLD.OBJ, BLD.ASM_CHECKED + ".s")
    src = os.path.join(BLD.CSRC, BLD.ASM_CHECKED)
    if not (os.path.exists(asm) and os.path.getmtime(asm) >= os.path.getmtime(src)):
        asm = BLD.check_transposed_reads()              # compiles (about a minute)
    found, n = BLD.premature_uses_of_transposed_reads(open(asm).read())
    assert n >= 8 and found == []


def test_bench_reads_the_traffic_figure_only_for_the_kernel_it_was_measured_on(tmp_path, monkeypatch):
    """bench.py takes roofline.traffic from the counter summary under profiles/ and drops it (None) as soon as the
    sources of the kernel differ from the digest recorded with the counters."""
    import sys
    sys.path.insert(0, ROOT)
    import bench
    f = tmp_path / "summary.txt"
    f.write_text("some text\ntraffic_bytes_per_launch: 8.25e9\nkernel_sources_digest: %s\nmore text\n" % bench.kernel_sources_digest())
    monkeypatch.setattr(bench, "TRAFFIC_SUMMARY", str(f))
    assert bench.measured_traffic() == 8.25e9
    f.write_text("traffic_bytes_per_launch: 8.25e9\nkernel_sources_digest: 0123456789abcdef\n")
    assert bench.measured_traffic() is None
    f.write_text("no figures here\n")
    assert bench.measured_traffic() is None
    monkeypatch.setattr(bench, "TRAFFIC_SUMMARY", str(tmp_path / "absent.txt"))
    assert bench.measured_traffic() is None
    # the summary that is committed belongs to the sources that are committed
    monkeypatch.undo()
    assert bench.measured_traffic() is not None
