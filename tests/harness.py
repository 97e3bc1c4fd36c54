"""Shared plumbing of the GPU parity tests: runs the HIP path (through the C boundary) and the
CPU oracle on the same seeded inputs and compares them element by element."""
from __future__ import annotations

import numpy as np

import workloads as W
from oracle import lopt_oracle as O

TOL_PARAM = 1e-4      # max relative error on updated parameters (metric: oracle.rel_err)
TOL_ACC = 1e-5        # on accumulators
TOL_STATS = 2e-5      # on the feature statistics (fp32 sums over the tensor)


def oracle_config_from(cfg) -> O.OracleConfig:
    """The oracle takes the very float32 values the C boundary carries."""
    import paper_2506_10315_amd as P
    return O.OracleConfig(
        kind=O.KIND_SMALL_FC if cfg.kind == P.LOPT_SMALL_FC else O.KIND_VELO,
        hidden=int(cfg.hidden),
        mom_decay=tuple(float(x) for x in cfg.mom_decay), rms_decay=float(cfg.rms_decay),
        fac_decay=tuple(float(x) for x in cfg.fac_decay),
        eps_acc=float(cfg.eps_acc), eps_norm=float(cfg.eps_norm),
        exp_mult=float(cfg.exp_mult), step_mult=float(cfg.step_mult),
        lstm_hidden=int(cfg.lstm_hidden), n_bank=int(cfg.n_bank))


def make_cfg(kind: str, hidden=None, lstm_hidden=None, n_bank=None):
    import paper_2506_10315_amd as P
    cfg = P.default_config(P.LOPT_SMALL_FC if kind == "small_fc_lopt" else P.LOPT_VELO)
    if hidden is not None:
        cfg.hidden = hidden
    if lstm_hidden is not None:
        cfg.lstm_hidden = lstm_hidden
    if n_bank is not None:
        cfg.n_bank = n_bank
    return cfg


def random_weights(cfg, seed=0) -> np.ndarray:
    """Seeded optimizer weights of the right size for any (hidden, lstm_hidden, n_bank)."""
    import paper_2506_10315_amd as P
    if cfg.kind == P.LOPT_SMALL_FC:
        return W.small_fc_weights(seed, int(cfg.hidden))
    return W.velo_weights(seed, int(cfg.hidden), int(cfg.lstm_hidden), int(cfg.n_bank))


class Case:
    """A list of tensors with its own seeded parameter/gradient streams."""

    def __init__(self, config_id, specs, grad_kind="gauss_fixed", indices=None):
        self.config_id = config_id
        self.specs = list(specs)
        self.grad_kind = grad_kind
        self.indices = list(indices) if indices is not None else list(range(len(self.specs)))

    def p0(self, i):
        return W.init_param(self.config_id, self.indices[i], self.specs[i])

    def grad(self, i, step):
        return W.grad(self.config_id, self.indices[i], step, self.specs[i], self.grad_kind)


def gpu_state_to_numpy(opt, i):
    v = opt.state_views(i)
    out = {"M": np.stack([x.cpu().numpy() for x in v["M"]]), "V": v["V"].cpu().numpy(),
           "r": np.stack([x.cpu().numpy() for x in v["r"]]), "c": np.stack([x.cpu().numpy() for x in v["c"]])}
    if "h" in v:
        out["h"] = v["h"].cpu().numpy()
        out["cl"] = v["cl"].cpu().numpy()
    return out


def compare_state(gs, st, tag, tol=TOL_ACC):
    worst = 0.0
    for key in ("M", "V", "r", "c") + (("h", "cl") if "h" in st else ()):
        e = O.rel_err(gs[key], st[key])
        worst = max(worst, e)
        assert e <= (tol if key not in ("h", "cl") else 1e-4), f"{tag}: accumulator {key} rel err {e:.3e}"
    return worst


def run_free(case: Case, cfg, weights, steps, lr_fn=lambda t: 1.0, wd=0.0, check_every=1, device="cuda:0",
             check_stats=True, verbose=False):
    """Free-running parity: GPU and oracle both start from (p0, zero state) and take `steps` steps on the
    same gradients; parameters, accumulators and statistics are compared after every `check_every` steps."""
    import torch
    import paper_2506_10315_amd as P
    ocfg = oracle_config_from(cfg)
    n = len(case.specs)
    shapes = [s.shape for s in case.specs]
    opt = P.LearnedOptimizer(cfg, weights, shapes, device=device)
    p_gpu = [torch.from_numpy(case.p0(i)).to(device) for i in range(n)]
    p_ora = [case.p0(i).astype(np.float64) for i in range(n)]
    st_ora = [O.init_state(*p.shape, ocfg) for p in p_ora]
    worst = {"param": 0.0, "acc": 0.0, "stats": 0.0}
    for t in range(steps):
        gs = [case.grad(i, t) for i in range(n)]
        g_gpu = [torch.from_numpy(g).to(device) for g in gs]
        lr = float(np.float32(lr_fn(t)))
        opt.step(p_gpu, g_gpu, lr=lr, weight_decay=float(np.float32(wd)), step=t)
        infos = []
        for i in range(n):
            info = {}
            p_ora[i] = O.tensor_step(p_ora[i], gs[i], st_ora[i], weights, ocfg, t, lr, float(np.float32(wd)),
                                     ndim=case.specs[i].as_2d()[0], out=info)
            infos.append(info)
        if (t + 1) % check_every == 0 or t == steps - 1:
            torch.cuda.synchronize()
            stats = opt.stats() if check_stats else None
            for i in range(n):
                tag = f"step {t} tensor {i} {case.specs[i].shape}"
                e = O.rel_err(p_gpu[i].cpu().numpy(), p_ora[i])
                worst["param"] = max(worst["param"], e)
                assert e <= TOL_PARAM, f"{tag}: parameter rel err {e:.3e}"
                worst["acc"] = max(worst["acc"], compare_state(gpu_state_to_numpy(opt, i), st_ora[i], tag))
                if check_stats:
                    k = ocfg.n_normalized
                    s_g = stats[i].cpu().numpy()[:k].astype(np.float64)
                    s_o = infos[i]["stats"][:k]
                    # a statistic acts only through s + eps_norm (fp32 cannot hold s below ~1e-45 anyway)
                    en = ocfg.eps_norm
                    rel = np.abs(s_g - s_o) / (np.abs(s_o) + en)
                    es = float(np.max(rel))
                    worst["stats"] = max(worst["stats"], es)
                    assert es <= TOL_STATS, f"{tag}: statistics rel err {es:.3e} (feature {int(np.argmax(rel))})"
        if verbose:
            print(f"  step {t}: worst so far {worst}", flush=True)
    opt.close()
    return worst


def _device_grad(case: Case, i: int, step: int, device):
    """Seeded on-device draw for tensors the oracle does not look at (same distribution family as
    workloads.grad; avoids minutes of host generation at the 355M / 1.3B sizes)."""
    import torch
    _, rows, cols = case.specs[i].as_2d()
    gen = torch.Generator(device=device)
    gen.manual_seed((W.BASE_SEED * 1000003 + case.config_id * 10007 + case.indices[i] * 101 + step) % (2 ** 63))
    scale = W.grad_scale(case.config_id, case.indices[i], case.grad_kind)
    z = torch.randn(rows, cols, generator=gen, device=device, dtype=torch.float32)
    if case.grad_kind == "student_t3":
        chi = sum(torch.randn(rows, cols, generator=gen, device=device, dtype=torch.float32) ** 2 for _ in range(3))
        z = z / torch.sqrt(chi / 3.0)
    return z * scale


def run_forced(case: Case, cfg, weights, steps, checks, lr_fn=lambda t: 1.0, wd=0.0, device="cuda:0",
               progress=print, closed_form_all_at_step0=True):
    """Teacher-forced parity at full size. The GPU free-runs `steps` steps over ALL tensors of the case in
    one lopt_step per step (the launch configuration bench.py times). `checks` maps a step index to the list
    of tensor indices the oracle verifies at that step: it takes ONE step from the GPU's own state before
    that step (widened to float64) and parameters and accumulators are compared element by element.
    Tensors that appear in no check get seeded on-device gradients. At step 0 every tensor is also checked
    against the closed forms M_i = (1-beta_i) g, V = (1-beta_4) g^2 that hold after one step from zero state."""
    import torch
    import paper_2506_10315_amd as P
    ocfg = oracle_config_from(cfg)
    n = len(case.specs)
    shapes = [s.shape for s in case.specs]
    checked = sorted({i for v in checks.values() for i in v})
    opt = P.LearnedOptimizer(cfg, weights, shapes, device=device)
    p_gpu = []
    for i in range(n):
        if i in checked:
            p_gpu.append(torch.from_numpy(case.p0(i)).to(device))
        else:
            gen = torch.Generator(device=device)
            gen.manual_seed(W.BASE_SEED + 7919 * case.indices[i])
            _, rows, cols = case.specs[i].as_2d()
            p_gpu.append(torch.randn(rows, cols, generator=gen, device=device, dtype=torch.float32) * 0.02)
    worst = {"param": 0.0, "acc": 0.0, "closed_form": 0.0}
    for t in range(steps):
        gs = {i: case.grad(i, t) for i in checked}
        g_gpu = [torch.from_numpy(gs[i]).to(device) if i in gs else _device_grad(case, i, t, device) for i in range(n)]
        lr = float(np.float32(lr_fn(t)))
        subset = checks.get(t, [])
        torch.cuda.synchronize()
        before = {i: (p_gpu[i].cpu().numpy().astype(np.float64),
                      {k: v.astype(np.float64) for k, v in gpu_state_to_numpy(opt, i).items()}) for i in subset}
        opt.step(p_gpu, g_gpu, lr=lr, weight_decay=float(np.float32(wd)), step=t)
        torch.cuda.synchronize()
        if t == 0 and closed_form_all_at_step0:
            for i in range(n):
                v = opt.state_views(i)
                g = g_gpu[i].double()
                for k in range(3):
                    ref = (1.0 - float(cfg.mom_decay[k])) * g
                    e = float(((v["M"][k].double() - ref).abs().max() / (ref.abs().max() + 1e-300)).item())
                    worst["closed_form"] = max(worst["closed_form"], e)
                    assert e <= 1e-6, f"tensor {i}: M_{k+1} after one step deviates from (1-beta) g by {e:.2e}"
                ref = (1.0 - float(cfg.rms_decay)) * g * g
                e = float(((v["V"].double() - ref).abs().max() / (ref.abs().max() + 1e-300)).item())
                assert e <= 1e-6, f"tensor {i}: V after one step deviates from (1-beta) g^2 by {e:.2e}"
                for k in range(3):
                    b = float(cfg.fac_decay[k])
                    rr = (1.0 - b) * (g * g).mean(dim=1)
                    cc = (1.0 - b) * (g * g).mean(dim=0)
                    er = float(((v["r"][k].double() - rr).abs().max() / (rr.abs().max() + 1e-300)).item())
                    ec = float(((v["c"][k].double() - cc).abs().max() / (cc.abs().max() + 1e-300)).item())
                    assert er <= TOL_ACC and ec <= TOL_ACC, f"tensor {i}: r/c after one step off by {er:.2e}/{ec:.2e}"
                assert bool(torch.isfinite(p_gpu[i]).all()), f"tensor {i}: non-finite parameter"
            progress(f"  step 0: closed forms hold on all {n} tensors (worst {worst['closed_form']:.2e})")
        for i in subset:
            p_b, st = before[i]
            p_o = O.tensor_step(p_b, gs[i], st, weights, ocfg, t, lr, float(np.float32(wd)),
                                ndim=case.specs[i].as_2d()[0])
            tag = f"step {t} tensor {i} {case.specs[i].name} {case.specs[i].shape}"
            e = O.rel_err(p_gpu[i].cpu().numpy(), p_o)
            worst["param"] = max(worst["param"], e)
            assert e <= TOL_PARAM, f"{tag}: parameter rel err {e:.3e}"
            worst["acc"] = max(worst["acc"], compare_state(gpu_state_to_numpy(opt, i), st, tag))
            if case.specs[i].numel > 200000:
                progress(f"  {tag}: ok, worst so far {worst}")
        progress(f"  step {t} done: worst so far {worst}")
        del g_gpu
    for i in range(n):
        assert bool(torch.isfinite(p_gpu[i]).all()), f"tensor {i}: non-finite parameter at the end"
    opt.close()
    return worst


def run_free_subset(case: Case, cfg, weights, steps, subset, check_steps, lr_fn=lambda t: 1.0, wd=0.0,
                    device="cuda:0", progress=print):
    """Free-running parity over many steps at full size. The GPU takes `steps` steps over ALL tensors of the case
    (one lopt_step per step); the oracle free-runs the tensors in `subset` from the same start (every tensor's step
    depends on that tensor alone) and parameters and accumulators are compared after the steps in `check_steps`.
    Tensors outside the subset get seeded on-device parameters and gradients."""
    import torch
    import paper_2506_10315_amd as P
    ocfg = oracle_config_from(cfg)
    n = len(case.specs)
    sub = sorted(subset)
    opt = P.LearnedOptimizer(cfg, weights, [s.shape for s in case.specs], device=device)
    p_gpu = []
    for i in range(n):
        if i in sub:
            p_gpu.append(torch.from_numpy(case.p0(i)).to(device))
        else:
            gen = torch.Generator(device=device)
            gen.manual_seed(W.BASE_SEED + 7919 * case.indices[i])
            _, rows, cols = case.specs[i].as_2d()
            p_gpu.append(torch.randn(rows, cols, generator=gen, device=device, dtype=torch.float32) * 0.02)
    p_ora = {i: case.p0(i).astype(np.float64) for i in sub}
    st_ora = {i: O.init_state(*p_ora[i].shape, ocfg) for i in sub}
    worst = {"param": 0.0, "acc": 0.0}
    for t in range(steps):
        gs = {i: case.grad(i, t) for i in sub}
        g_gpu = [torch.from_numpy(gs[i]).to(device) if i in gs else _device_grad(case, i, t, device) for i in range(n)]
        lr, wdf = float(np.float32(lr_fn(t))), float(np.float32(wd))
        opt.step(p_gpu, g_gpu, lr=lr, weight_decay=wdf, step=t)
        for i in sub:
            p_ora[i] = O.tensor_step(p_ora[i], gs[i], st_ora[i], weights, ocfg, t, lr, wdf, ndim=case.specs[i].as_2d()[0])
        if t in check_steps:
            torch.cuda.synchronize()
            for i in sub:
                tag = f"step {t} tensor {i} {case.specs[i].name} {case.specs[i].shape}"
                e = O.rel_err(p_gpu[i].cpu().numpy(), p_ora[i])
                worst["param"] = max(worst["param"], e)
                assert e <= TOL_PARAM, f"{tag}: parameter rel err {e:.3e}"
                worst["acc"] = max(worst["acc"], compare_state(gpu_state_to_numpy(opt, i), st_ora[i], tag))
            progress(f"  step {t}: worst so far {worst}")
        del g_gpu
    torch.cuda.synchronize()
    for i in range(n):
        assert bool(torch.isfinite(p_gpu[i]).all()), f"tensor {i}: non-finite parameter at the end"
    opt.close()
    return worst
