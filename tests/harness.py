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
                    es = float(np.max(np.abs(s_g - s_o) / (np.abs(s_o) + 1e-300)))
                    worst["stats"] = max(worst["stats"], es)
                    assert es <= TOL_STATS, f"{tag}: statistics rel err {es:.3e} (feature {np.argmax(np.abs(s_g - s_o) / (np.abs(s_o) + 1e-300))})"
        if verbose:
            print(f"  step {t}: worst so far {worst}", flush=True)
    opt.close()
    return worst


def run_forced(case: Case, cfg, weights, steps, check_steps, lr_fn=lambda t: 1.0, wd=0.0, device="cuda:0",
               tensor_subset=None, verbose=False):
    """Teacher-forced parity at full size: the GPU free-runs; at each step in `check_steps` the oracle takes ONE
    step from the GPU's own state before that step (widened to float64) and the results are compared."""
    import torch
    import paper_2506_10315_amd as P
    ocfg = oracle_config_from(cfg)
    n = len(case.specs)
    shapes = [s.shape for s in case.specs]
    opt = P.LearnedOptimizer(cfg, weights, shapes, device=device)
    p_gpu = [torch.from_numpy(case.p0(i)).to(device) for i in range(n)]
    subset = list(range(n)) if tensor_subset is None else list(tensor_subset)
    worst = {"param": 0.0, "acc": 0.0}
    for t in range(steps):
        gs = [case.grad(i, t) for i in range(n)]
        g_gpu = [torch.from_numpy(g).to(device) for g in gs]
        lr = float(np.float32(lr_fn(t)))
        before = None
        if t in check_steps:
            torch.cuda.synchronize()
            before = {i: (p_gpu[i].cpu().numpy().astype(np.float64),
                          {k: v.astype(np.float64) for k, v in gpu_state_to_numpy(opt, i).items()}) for i in subset}
        opt.step(p_gpu, g_gpu, lr=lr, weight_decay=float(np.float32(wd)), step=t)
        if before is not None:
            torch.cuda.synchronize()
            for i in subset:
                p_b, st = before[i]
                p_o = O.tensor_step(p_b, gs[i], st, weights, ocfg, t, lr, float(np.float32(wd)),
                                    ndim=case.specs[i].as_2d()[0])
                tag = f"step {t} tensor {i} {case.specs[i].shape}"
                e = O.rel_err(p_gpu[i].cpu().numpy(), p_o)
                worst["param"] = max(worst["param"], e)
                assert e <= TOL_PARAM, f"{tag}: parameter rel err {e:.3e}"
                worst["acc"] = max(worst["acc"], compare_state(gpu_state_to_numpy(opt, i), st, tag))
            if verbose:
                print(f"  step {t}: worst so far {worst}", flush=True)
    opt.close()
    return worst
