"""GPU behaviour that is not numerical parity: determinism (doubles as the race detector), checkpoint /
resume through the documented state layout, argument validation on the step path, empty lists."""
import ctypes as C

import numpy as np
import pytest

import workloads as W
from tests import harness as Hn

pytestmark = pytest.mark.gpu

SHAPES = [(300, 257), (64, 256), (1030,), (5,), (520, 768)]


def _run(kind, steps, device="cuda:0", resume_at=None, seed=0):
    import torch
    import paper_2506_10315_amd as P
    cfg = Hn.make_cfg(kind) if kind == "small_fc_lopt" else Hn.make_cfg(kind, lstm_hidden=64, n_bank=32)
    w = Hn.random_weights(cfg, seed)
    specs = [W.TensorSpec(f"t{i}", s) for i, s in enumerate(SHAPES)]
    case = Hn.Case(201, specs, "gauss_logscale")
    opt = P.LearnedOptimizer(cfg, w, SHAPES, device=device)
    p = [torch.from_numpy(case.p0(i)).to(device) for i in range(len(specs))]
    for t in range(steps):
        if resume_at is not None and t == resume_at:
            # checkpoint = plain copies of params and state blobs; resume into a NEW context
            torch.cuda.synchronize()
            saved_p = [x.clone() for x in p]
            saved_s = [x.clone() for x in opt.state]
            opt.close()
            opt = P.LearnedOptimizer(cfg, w, SHAPES, device=device)
            for dst, src in zip(opt.state, saved_s):
                dst.copy_(src)
            p = saved_p
        g = [torch.from_numpy(case.grad(i, t)).to(device) for i in range(len(specs))]
        opt.step(p, g, lr=0.7, weight_decay=0.01, step=t)
    torch.cuda.synchronize()
    out = [x.cpu().numpy().copy() for x in p] + [x.cpu().numpy().copy() for x in opt.state]
    opt.close()
    return out


@pytest.mark.parametrize("kind", ["small_fc_lopt", "velo"])
def test_two_runs_are_bit_identical(kind):
    a = _run(kind, 5)
    b = _run(kind, 5)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))


def test_groups_field_of_the_configuration_selects_the_plan_per_context():
    # two contexts in one process, one with every pass over the whole list on one stream, one with three tensor groups
    # on two streams: same bits (the selection is per context, no environment involved)
    import torch
    import paper_2506_10315_amd as P
    outs = []
    for groups in (1, 3):
        cfg = Hn.make_cfg("small_fc_lopt", groups=groups)
        w = Hn.random_weights(cfg, 0)
        specs = [W.TensorSpec(f"t{i}", s) for i, s in enumerate(SHAPES)]
        case = Hn.Case(201, specs, "gauss_logscale")
        opt = P.LearnedOptimizer(cfg, w, SHAPES)
        p = [torch.from_numpy(case.p0(i)).to("cuda:0") for i in range(len(specs))]
        for t in range(3):
            g = [torch.from_numpy(case.grad(i, t)).to("cuda:0") for i in range(len(specs))]
            opt.step(p, g, lr=0.7, weight_decay=0.01, step=t)
        torch.cuda.synchronize()
        outs.append([x.cpu().numpy().copy() for x in p] + [x.cpu().numpy().copy() for x in opt.state])
        opt.close()
    for x, y in zip(*outs):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))


@pytest.mark.parametrize("kind,groups", [("small_fc_lopt", 1), ("small_fc_lopt", 3), ("velo", 1)])
def test_state_pass_field_moves_the_accumulator_update_without_changing_a_bit(kind, groups):
    # The new M_1..3 and V are written either by the statistics pass or by the default apply kernels (split-fp16 strip
    # kernel of small_fc_lopt, width-4 kernel of VeLO), which then form them a second time with the same fp32
    # operations: parameters AND every word of the state must agree bit for bit, ragged and unaligned shapes included,
    # with and without the tensor-group pipeline.
    import torch
    import paper_2506_10315_amd as P
    shapes = SHAPES + [(300, 257), (2, 1000), (1, 77), (129, 64)]
    outs = []
    for state_pass in ("stats", "apply"):
        if kind == "small_fc_lopt":
            cfg = Hn.make_cfg(kind, groups=groups, state_pass=state_pass)
        else:
            cfg = Hn.make_cfg(kind, lstm_hidden=32, n_bank=8, state_pass=state_pass)
        w = Hn.random_weights(cfg, 0)
        specs = [W.TensorSpec(f"t{i}", s) for i, s in enumerate(shapes)]
        case = Hn.Case(202, specs, "gauss_logscale")
        opt = P.LearnedOptimizer(cfg, w, shapes)
        p = [torch.from_numpy(case.p0(i)).to("cuda:0") for i in range(len(specs))]
        for t in range(4):
            g = [torch.from_numpy(case.grad(i, t)).to("cuda:0") for i in range(len(specs))]
            opt.step(p, g, lr=0.7, weight_decay=0.01, step=t, loss=1.5 - 0.1 * t)
        torch.cuda.synchronize()
        outs.append([x.cpu().numpy().copy() for x in p] + [x.cpu().numpy().copy() for x in opt.state])
        opt.close()
    for x, y in zip(*outs):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))


@pytest.mark.parametrize("groups", [2, 3, 16])
def test_group_pipeline_is_bit_identical_to_one_stream(groups, monkeypatch):
    # LOPT_GROUPS (read when the context is created) cuts the list into tensor groups whose HBM-bound passes run on
    # the library's second stream beside the previous group's apply pass. The same kernels see the same tiles, so
    # the results must not change by a single bit, on the default stream and on a stream of the caller's.
    import torch
    monkeypatch.setenv("LOPT_GROUPS", "1")
    ref = _run("small_fc_lopt", 4)
    monkeypatch.setenv("LOPT_GROUPS", str(groups))
    out = _run("small_fc_lopt", 4)
    for x, y in zip(ref, out):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        out2 = _run("small_fc_lopt", 4)
    for x, y in zip(ref, out2):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))


@pytest.mark.parametrize("kind", ["small_fc_lopt", "velo"])
def test_per_pass_timing_changes_no_result_and_names_every_pass(kind, monkeypatch):
    # With lopt_profile_enable the step runs pass after pass on one stream with events in between (no tensor groups);
    # results must be bit-identical to the default launch plan, here forced to three groups.
    import torch
    import paper_2506_10315_amd as P
    monkeypatch.setenv("LOPT_GROUPS", "3")
    ref = _run(kind, 3)
    cfg = Hn.make_cfg(kind) if kind == "small_fc_lopt" else Hn.make_cfg(kind, lstm_hidden=64, n_bank=32)
    w = Hn.random_weights(cfg, 0)
    specs = [W.TensorSpec(f"t{i}", s) for i, s in enumerate(SHAPES)]
    case = Hn.Case(201, specs, "gauss_logscale")
    opt = P.LearnedOptimizer(cfg, w, SHAPES, device="cuda:0")
    opt.profile_enable(True)
    p = [torch.from_numpy(case.p0(i)).to("cuda:0") for i in range(len(specs))]
    for t in range(3):
        g = [torch.from_numpy(case.grad(i, t)).to("cuda:0") for i in range(len(specs))]
        opt.step(p, g, lr=0.7, weight_decay=0.01, step=t)
    pass_ms, k = opt.profile_read()
    torch.cuda.synchronize()
    out = [x.cpu().numpy().copy() for x in p] + [x.cpu().numpy().copy() for x in opt.state]
    opt.close()
    assert k == 3 and set(pass_ms) == {"rowcol_sums", "rc_update", "accum_stats", "finalize", "velo_lstm", "velo_head", "apply"}
    assert all(v >= 0.0 for v in pass_ms.values()) and pass_ms["apply"] > 0.0 and pass_ms["accum_stats"] > 0.0
    if kind == "velo":
        assert pass_ms["velo_lstm"] > 0.0 and pass_ms["velo_head"] > 0.0
    for x, y in zip(ref, out):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))


@pytest.mark.parametrize("kind", ["small_fc_lopt", "velo"])
def test_checkpoint_resume_is_bit_identical(kind):
    a = _run(kind, 6)
    b = _run(kind, 6, resume_at=3)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))


def test_step_argument_validation_leaves_everything_untouched():
    import torch
    import paper_2506_10315_amd as P
    from paper_2506_10315_amd import binding as B
    cfg = Hn.make_cfg("small_fc_lopt")
    opt = P.LearnedOptimizer(cfg, W.small_fc_weights(0), [(8, 12)])
    p = torch.full((8, 12), 0.5, device="cuda:0")
    g = torch.full((8, 12), 1e-3, device="cuda:0")
    L = P.lib()
    ws = C.c_void_p(opt.workspace.data_ptr())
    descs = opt._descs

    def step(pp, gp, sp, workspace=ws, step=0, lr=1.0, wd=0.0, d=descs, n=1):
        arr = lambda x: (C.c_void_p * 1)(x)
        return L.lopt_step(opt._ctx, n, d, arr(pp), arr(gp), arr(sp), workspace, step, lr, wd, None)

    sp = opt.state[0].data_ptr()
    assert step(None, g.data_ptr(), sp) == 1
    assert step(p.data_ptr(), None, sp) == 1
    assert step(p.data_ptr(), g.data_ptr(), None) == 1
    assert step(p.data_ptr() + 4, g.data_ptr(), sp) == 1 and b"aligned" in L.lopt_last_error(opt._ctx)
    assert step(p.data_ptr(), g.data_ptr(), sp, workspace=None) == 1
    assert step(p.data_ptr(), g.data_ptr(), sp, step=-1) == 1
    assert step(p.data_ptr(), g.data_ptr(), sp, lr=float("nan")) == 1
    assert step(p.data_ptr(), g.data_ptr(), sp, wd=float("inf")) == 1
    bad = (B.lopt_tensor_desc * 1)()
    bad[0].ndim, bad[0].rows, bad[0].cols = 2, 0, 12
    assert step(p.data_ptr(), g.data_ptr(), sp, d=bad) == 2          # LOPT_ESHAPE
    bad[0].rows, bad[0].cols = 1 << 20, 1 << 20
    assert step(p.data_ptr(), g.data_ptr(), sp, d=bad) == 2
    bad[0].ndim, bad[0].rows, bad[0].cols = 0, 8, 12
    assert step(p.data_ptr(), g.data_ptr(), sp, d=bad) == 1
    # an empty list is a valid no-op
    assert L.lopt_step(opt._ctx, 0, None, None, None, None, None, 0, 1.0, 0.0, None) == 0
    torch.cuda.synchronize()
    assert bool((p == 0.5).all()) and bool((opt.state[0] == 0).all())
    # and the context still works afterwards
    assert step(p.data_ptr(), g.data_ptr(), sp) == 0
    torch.cuda.synchronize()
    assert not bool((p == 0.5).all())
    opt.close()


def test_context_reused_across_different_tensor_lists_and_streams():
    import torch
    import paper_2506_10315_amd as P
    cfg = Hn.make_cfg("small_fc_lopt")
    w = W.small_fc_weights(0)
    res = []
    for use_side_stream in (False, True):
        opt = P.LearnedOptimizer(cfg, w, [(64, 256), (33,)])
        p = [torch.full((64, 256), 0.1, device="cuda:0"), torch.full((1, 33), 0.1, device="cuda:0")]
        g = [torch.linspace(-1e-3, 1e-3, 64 * 256, device="cuda:0").view(64, 256).contiguous(),
             torch.linspace(-1e-3, 1e-3, 33, device="cuda:0").view(1, 33).contiguous()]
        torch.cuda.synchronize()
        if use_side_stream:
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                opt.step(p, g)
                opt.step(p, g)
            s.synchronize()
        else:
            opt.step(p, g)
            opt.step(p, g)
        torch.cuda.synchronize()
        res.append([x.cpu().numpy().copy() for x in p])
        opt.close()
    for x, y in zip(*res):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("kind,shapes,static", [
    ("small_fc_lopt", [(300, 257), (64, 256), (1030,), (5,)], True),
    ("velo", [(300, 257), (64, 256), (1030,), (5,)], True),
    ("small_fc_lopt", [(1000, 1000)], False),
    ("small_fc_lopt", [(4096, 2560)] * 4 + [(2560,)] * 4, True),       # 42 M elements: the two-stream group pipeline
])
def test_a_step_captured_in_a_hip_graph_replays_bit_identically(kind, shapes, static):
    # After one warm-up call (tables uploaded, nothing left to allocate) a step is captured into a HIP graph: no
    # allocation, no host synchronization and no memset node inside the capture (tile counters are cleared by a kernel).
    # Replays are checked against the eager step from the same state, three times, with eager work and
    # synchronizations of the program's own in between.
    import torch
    import paper_2506_10315_amd as P
    dev = "cuda:0"
    cfg = Hn.make_cfg(kind) if kind == "small_fc_lopt" else Hn.make_cfg(kind, lstm_hidden=64, n_bank=32)
    w = Hn.random_weights(cfg, 2)
    specs = [W.TensorSpec(f"t{i}", s) for i, s in enumerate(shapes)]
    case = Hn.Case(202, specs, "gauss_logscale")
    opt = P.LearnedOptimizer(cfg, w, shapes, device=dev)
    n = len(specs)
    p = [torch.from_numpy(case.p0(i)).to(dev) for i in range(n)]
    g = [torch.from_numpy(case.grad(i, 0)).to(dev) for i in range(n)]
    kw = dict(lr=0.7, weight_decay=0.01, static=static, loss=1.5)
    for t in range(2):                                   # warm-up: two real steps, so the state is not trivial
        opt.step(p, g, step=t, **kw)
    torch.cuda.synchronize()
    p0 = [x.clone() for x in p]
    s0 = [x.clone() for x in opt.state]

    def restore():
        for dst, src in zip(p, p0):
            dst.copy_(src)
        for dst, src in zip(opt.state, s0):
            dst.copy_(src)

    opt.step(p, g, step=2, **kw)                         # the eager result of step 2 from (p0, s0)
    torch.cuda.synchronize()
    want = [x.clone() for x in p] + [x.clone() for x in opt.state]
    restore()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        opt.step(p, g, step=2, **kw)
    torch.cuda.synchronize()
    junk = torch.zeros(1 << 20, device=dev)
    for rep in range(3):
        restore()
        junk.add_(1.0)                                   # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = list(p) + list(opt.state)
        for a, b in zip(want, got):
            assert torch.equal(a.view(torch.int32), b.view(torch.int32)), f"replay {rep} differs from the eager step"
    del graph
    opt.close()
