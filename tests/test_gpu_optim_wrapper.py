"""The torch.optim.Optimizer veneer: same numbers as the raw binding, state_dict resume, LR scheduler and
decoupled weight decay through param-group fields, and the paper's `optimizer.step(loss)` call form."""
import numpy as np
import pytest

import workloads as W
from tests import harness as Hn

pytestmark = pytest.mark.gpu


def _model(seed=0):
    import torch
    torch.manual_seed(seed)
    m = torch.nn.Sequential(torch.nn.Linear(40, 64), torch.nn.ReLU(), torch.nn.Linear(64, 10)).cuda()
    return m


def _batch(step):
    import torch
    g = torch.Generator(device="cuda").manual_seed(100 + step)
    return torch.randn(32, 40, device="cuda", generator=g), torch.randint(0, 10, (32,), device="cuda", generator=g)


@pytest.mark.parametrize("kind", ["small_fc_lopt", "velo"])
def test_wrapper_matches_oracle_and_resumes(kind):
    import torch
    from paper_2506_10315_amd.optim import LearnedOptTorch
    from oracle import lopt_oracle as O
    cfg = Hn.make_cfg(kind) if kind == "small_fc_lopt" else Hn.make_cfg(kind, lstm_hidden=32, n_bank=16)
    w = Hn.random_weights(cfg, 7)
    ocfg = Hn.oracle_config_from(cfg)
    model = _model()
    opt = LearnedOptTorch(model.parameters(), w, kind=kind, lr=0.5, weight_decay=0.01, cfg=cfg)
    sched = torch.optim.lr_scheduler.StepLR(opt, step_size=2, gamma=0.5)
    params = list(model.parameters())
    p_ora = [p.detach().cpu().numpy().astype(np.float64).reshape(Hn_shape(p)) for p in params]
    st_ora = [O.init_state(*p.shape, ocfg) for p in p_ora]
    saved = None
    for t in range(5):
        x, y = _batch(t)
        opt.zero_grad()
        loss = torch.nn.functional.cross_entropy(model(x), y)
        loss.backward()
        lr = float(np.float32(opt.param_groups[0]["lr"]))
        grads = [p.grad.detach().cpu().numpy().reshape(q.shape) for p, q in zip(params, p_ora)]
        opt.step(loss)                           # the paper's call form for VeLO: the loss value is an input
        sched.step()
        p_ora = O.list_step(p_ora, grads, st_ora, w, ocfg, t, lr, float(np.float32(0.01)),
                            [max(1, p.dim()) for p in params], loss=float(np.float32(loss.item())))
        for i, p in enumerate(params):
            e = O.rel_err(p.detach().cpu().numpy().reshape(p_ora[i].shape), p_ora[i])
            assert e <= Hn.TOL_PARAM, f"step {t} param {i}: {e:.2e}"
        if t == 2:
            saved = ({k: v.clone() for k, v in model.state_dict().items()}, opt.state_dict(), sched.state_dict())
    final = [p.detach().clone() for p in params]
    # resume from the checkpoint taken after step 2 in a fresh model/optimizer: bit-identical continuation
    model2 = _model(seed=1)
    model2.load_state_dict(saved[0])
    opt2 = LearnedOptTorch(model2.parameters(), w, kind=kind, lr=0.5, weight_decay=0.01, cfg=cfg)
    sched2 = torch.optim.lr_scheduler.StepLR(opt2, step_size=2, gamma=0.5)
    opt2.load_state_dict(saved[1])
    sched2.load_state_dict(saved[2])
    for t in range(3, 5):
        x, y = _batch(t)
        opt2.zero_grad()
        loss = torch.nn.functional.cross_entropy(model2(x), y)
        loss.backward()
        opt2.step(loss)
        sched2.step()
    for a, b in zip(final, model2.parameters()):
        assert torch.equal(a, b.detach())


def Hn_shape(p):
    from paper_2506_10315_amd.binding import flatten_shape
    _, r, c = flatten_shape(tuple(p.shape))
    return (r, c)


def test_parameters_without_gradients_are_skipped_and_the_loss_matters_for_velo():
    import torch
    from paper_2506_10315_amd.optim import LearnedOptTorch
    cfg = Hn.make_cfg("velo", lstm_hidden=32, n_bank=16)
    w = Hn.random_weights(cfg, 8)
    res = {}
    for loss_value in (0.7, 9.0):
        model = _model()
        frozen = model[2].bias
        opt = LearnedOptTorch(model.parameters(), w, kind="velo", lr=0.5, weight_decay=0.01, cfg=cfg)
        before = frozen.detach().clone()
        for t in range(3):
            x, y = _batch(t)
            opt.zero_grad(set_to_none=True)
            torch.nn.functional.cross_entropy(model(x), y).backward()
            frozen.grad = None                                  # e.g. an unused or frozen parameter
            opt.step(loss_value)
        torch.cuda.synchronize()
        assert torch.equal(frozen.detach(), before)             # no update, no weight decay
        assert bool((opt._engines[0].state[3] == 0).all())      # its accumulators never moved
        res[loss_value] = [p.detach().clone() for p in model.parameters()]
    assert any(not torch.equal(a, b) for a, b in zip(res[0.7], res[9.0]))   # the loss value reaches the update
