"""Host-side checks of the C boundary that need no GPU: the library loads, exports every symbol
include/lopt.h declares, and rejects bad configurations before touching the device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    src = open(os.path.join(ROOT, "include", "lopt.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(lopt_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    import paper_2506_10315_amd as P
    L = P.lib()
    syms = _declared_symbols()
    assert "lopt_step" in syms and "lopt_create" in syms and len(syms) >= 9
    for s in syms:
        assert hasattr(L, s), f"liblopt.so does not export {s}"
    from paper_2506_10315_amd import binding
    assert sorted(binding.EXPORTS) == syms


def test_default_config_and_weight_counts():
    import paper_2506_10315_amd as P
    import workloads as W
    c = P.default_config(P.LOPT_SMALL_FC)
    assert c.struct_size == C.sizeof(P.lopt_config)
    assert (c.hidden, c.kind) == (32, 0)
    assert P.weights_count(c) == 39 * 32 + 32 + 32 * 32 + 32 + 64 + 2 == W.small_fc_weights(0).size
    v = P.default_config(P.LOPT_VELO)
    assert (v.hidden, v.lstm_hidden, v.n_bank) == (4, 512, 256)
    assert P.weights_count(v) == W.velo_weights(0).size
    assert [round(float(x), 6) for x in c.mom_decay] == [0.9, 0.99, 0.999]
    assert float(c.exp_mult) == pytest.approx(0.01) and float(c.step_mult) == pytest.approx(0.01)


def test_create_rejects_bad_configurations_without_a_device():
    import paper_2506_10315_amd as P
    L = P.lib()
    w = np.zeros(2402, np.float32)
    wp = w.ctypes.data_as(C.POINTER(C.c_float))
    ctx = C.c_void_p()

    def create(cfg, n=2402, ptr=wp):
        return L.lopt_create(C.byref(cfg), ptr, n, C.byref(ctx))

    c = P.default_config(0)
    c.hidden = 0
    assert create(c) == 1 and b"hidden" in L.lopt_last_error(None)
    c = P.default_config(0)
    c.hidden = 33
    assert create(c) == 1
    c = P.default_config(0)
    c.struct_size = 8
    assert create(c) == 1 and b"struct_size" in L.lopt_last_error(None)
    c = P.default_config(0)
    c.rms_decay = 1.0
    assert create(c) == 1 and b"decay" in L.lopt_last_error(None)
    c = P.default_config(0)
    c.eps_acc = -1.0
    assert create(c) == 1
    c = P.default_config(0)
    c.kind = 7
    assert create(c) == 1
    c = P.default_config(0)
    assert create(c, n=100) == 3 and b"2402" in L.lopt_last_error(None)      # LOPT_ESTATE
    assert create(c, ptr=None) == 1
    v = P.default_config(1)
    v.lstm_hidden = 0
    assert create(v) == 1
    assert ctx.value is None
    assert L.lopt_default_config(9, C.byref(c)) == 1
    assert L.lopt_weights_count(None) == 0
    L.lopt_destroy(None)     # null is ignored
    assert L.lopt_pass_name(6) == b"apply" and L.lopt_pass_name(7) is None


def test_flatten_shape_convention():
    from paper_2506_10315_amd.binding import flatten_shape
    import workloads as W
    for shp in [(768,), (1, 1, 768), (1, 197, 768), (768, 3, 16, 16), (2304, 768), (1,), (3, 1)]:
        assert flatten_shape(shp) == W.TensorSpec("x", shp).as_2d()
    assert flatten_shape((768, 3, 16, 16)) == (4, 768, 768)
    assert flatten_shape((1, 197, 768)) == (2, 197, 768)
    assert flatten_shape((5,)) == (1, 1, 5)


def test_workload_shapes_match_the_named_models():
    import workloads as W
    assert (len(W.vit_b16_shapes()), W.get_workload(2).numel) == (152, 86_567_656)   # paper: 86.57 M
    assert (len(W.gpt2_medium_shapes()), W.get_workload(4).numel) == (388, 354_823_168)
    w5 = W.get_workload(5)
    assert len(w5.tensors) == 219 + 2000
    assert sum(t.numel for t in w5.tensors[:219]) == 1_345_423_360
    assert all(1 <= t.numel <= 512 for t in w5.tensors[219:])


def test_bench_refuses_more_than_one_gpu():
    # one GPU only: a request for more ends with a message before anything touches a device
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_create_refuses_unknown_tuning_knob_values_and_non_finite_weights(monkeypatch):
    import paper_2506_10315_amd as P
    L = P.lib()
    w = np.zeros(2402, np.float32)
    wp = w.ctypes.data_as(C.POINTER(C.c_float))
    ctx = C.c_void_p()
    c = P.default_config(0)
    c.apply_kernel = 4
    assert L.lopt_create(C.byref(c), wp, 2402, C.byref(ctx)) == 1 and b"apply_kernel" in L.lopt_last_error(None)
    c = P.default_config(0)
    c.groups = 17
    assert L.lopt_create(C.byref(c), wp, 2402, C.byref(ctx)) == 1 and b"groups" in L.lopt_last_error(None)
    c = P.default_config(0)
    c.state_pass = 3
    assert L.lopt_create(C.byref(c), wp, 2402, C.byref(ctx)) == 1 and b"state_pass" in L.lopt_last_error(None)
    c = P.default_config(0)
    monkeypatch.setenv("LOPT_STATE_PASS", "1")              # names only: auto, stats, apply
    assert L.lopt_create(C.byref(c), wp, 2402, C.byref(ctx)) == 1 and b"LOPT_STATE_PASS" in L.lopt_last_error(None)
    monkeypatch.delenv("LOPT_STATE_PASS")
    monkeypatch.setenv("LOPT_APPLY", "mfma_f16")            # a misspelt variant must not silently mean "auto"
    assert L.lopt_create(C.byref(c), wp, 2402, C.byref(ctx)) == 1 and b"LOPT_APPLY" in L.lopt_last_error(None)
    monkeypatch.delenv("LOPT_APPLY")
    for bad in ("17", "-1", "four", ""):
        monkeypatch.setenv("LOPT_GROUPS", bad)
        assert L.lopt_create(C.byref(c), wp, 2402, C.byref(ctx)) == 1 and b"LOPT_GROUPS" in L.lopt_last_error(None)
    monkeypatch.delenv("LOPT_GROUPS")
    w[100] = np.inf
    assert L.lopt_create(C.byref(c), wp, 2402, C.byref(ctx)) == 1 and b"non-finite" in L.lopt_last_error(None)
    assert not ctx.value


def test_set_loss_validates_its_arguments():
    import paper_2506_10315_amd as P
    L = P.lib()
    assert L.lopt_set_loss(None, 1.0) == 1
