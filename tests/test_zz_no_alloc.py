"""lopt_step_static (the entry point for callers that cannot allocate: tables and workspace in the library's fixed
per-GPU scratch array) against lopt_step, through the C boundary: bit-identical parameters and state on two calls
in a row, the second on a smaller list; two contexts taking turns on the array; refusal of a list beyond the limit."""
import ctypes as C

import numpy as np
import pytest

import workloads as W
from tests import harness as Hn

pytestmark = pytest.mark.gpu

BIG = [(300, 257), (64, 256), (1030,), (5,), (520, 768), (2048, 512)]
SMALL = [(33, 100), (7,), (64, 256)]


def _inputs(shapes, case_id, step):
    import torch
    specs = [W.TensorSpec(f"t{i}", s) for i, s in enumerate(shapes)]
    case = Hn.Case(case_id, specs, "gauss_logscale")
    p = [torch.from_numpy(case.p0(i)).to("cuda:0") for i in range(len(specs))]
    g = [torch.from_numpy(case.grad(i, step)).to("cuda:0") for i in range(len(specs))]
    return p, g


def _make(kind, shapes):
    import paper_2506_10315_amd as P
    cfg = Hn.make_cfg(kind) if kind == "small_fc_lopt" else Hn.make_cfg(kind, lstm_hidden=64, n_bank=32)
    return P.LearnedOptimizer(cfg, Hn.random_weights(cfg, 7), shapes)


def _bits(ts):
    import torch
    torch.cuda.synchronize()
    return [t.detach().cpu().numpy().view(np.uint32).copy() for t in ts]


@pytest.mark.parametrize("kind", ["small_fc_lopt", "velo"])
def test_static_scratch_step_matches_lopt_step_on_two_calls_the_second_smaller(kind):
    out = {}
    for static in (False, True):
        res = []
        # first call: the larger list, two steps (the second runs on non-zero state and re-uses the cached tables)
        opt = _make(kind, BIG)
        p, _ = _inputs(BIG, 301, 0)
        for t in range(2):
            _, g = _inputs(BIG, 301, t)
            opt.step(p, g, lr=0.7, weight_decay=0.01, step=t, static=static)
        res += _bits(p) + _bits(opt.state)
        # second call, right after, on a smaller list through a new context: the array still holds the first call's data
        opt2 = _make(kind, SMALL)
        p2, g2 = _inputs(SMALL, 302, 0)
        opt2.step(p2, g2, lr=0.7, weight_decay=0.01, step=0, static=static)
        res += _bits(p2) + _bits(opt2.state)
        # and the first context again, after the other one has overwritten its tables
        _, g = _inputs(BIG, 301, 2)
        opt.step(p, g, lr=0.7, weight_decay=0.01, step=2, static=static)
        res += _bits(p) + _bits(opt.state)
        opt.close()
        opt2.close()
        out[static] = res
    assert len(out[False]) == len(out[True])
    for a, b in zip(out[False], out[True]):
        assert np.array_equal(a, b)


def test_static_scratch_step_refuses_a_list_beyond_its_limit_and_leaves_everything_untouched():
    import torch
    import paper_2506_10315_amd as P
    from paper_2506_10315_amd import binding as B
    cfg = Hn.make_cfg("small_fc_lopt")
    opt = P.LearnedOptimizer(cfg, W.small_fc_weights(0), [(8, 12)])
    L = P.lib()
    # eight tensors of 46340 x 46340 need far more than 64 MiB of row/column partials; the refusal comes from the
    # host-side size check, before any pointer is touched
    n = 8
    descs = (B.lopt_tensor_desc * n)()
    for i in range(n):
        descs[i].ndim, descs[i].rows, descs[i].cols = 2, 46340, 46340
    fake = (C.c_void_p * n)(*[0x1000 * (i + 1) for i in range(n)])
    st = L.lopt_step_static(opt._ctx, n, descs, fake, fake, fake, 0, 1.0, 0.0, None)
    assert st == 6 and b"scratch" in L.lopt_last_error(opt._ctx)
    # the context still works
    p = torch.full((8, 12), 0.5, device="cuda:0")
    g = torch.full((8, 12), 1e-3, device="cuda:0")
    opt.step([p], [g], static=True)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(p).all()) and not bool((p == 0.5).all())
    opt.close()
