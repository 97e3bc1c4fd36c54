"""Shared plumbing of the GPU parity tests: runs the HIP path (through the C boundary) and the
CPU oracle on the same seeded inputs and compares them element by element."""
from __future__ import annotations

import numpy as np

import workloads as W
from oracle import lopt_oracle as O

TOL_PARAM = 1e-4      # max relative error on updated parameters (metric: oracle.rel_err)
TOL_ACC = 1e-5        # on accumulators
TOL_STATS = 2e-5      # on the feature statistics (fp32 sums over the tensor)
TOL_DELTA = 1e-4      # on the update p_old - p_new itself, in the same metric, net of the fp32 rounding of p_new
TOL_LSTM = 1e-5       # on VeLO's LSTM state: the accumulator bar (worst seen over the whole GPU suite: 7e-7)
ORACLE_THREADS = 12   # independent tensors go through the oracle side by side (the oracle itself is untouched)


def pool_map(fn, items):
    """fn over items on a small thread pool (NumPy releases the GIL in its kernels). BLAS is held to ONE thread per
    call meanwhile: the pthreads OpenBLAS that NumPy ships returns wrong products when several Python threads each
    run a multi-threaded matmul (seen with 0.3.29; tests/test_harness_cpu.py holds the pooled results equal to the
    serial ones). Results in input order; the first exception propagates."""
    items = list(items)
    if len(items) <= 1:
        return [fn(x) for x in items]
    from concurrent.futures import ThreadPoolExecutor
    try:
        import threadpoolctl
        limit = threadpoolctl.threadpool_limits(limits=1, user_api="blas")
    except Exception:
        return [fn(x) for x in items]     # no way to hold BLAS to one thread: stay serial
    try:
        with ThreadPoolExecutor(max_workers=ORACLE_THREADS) as ex:
            return list(ex.map(fn, items))
    finally:
        if limit is not None:
            limit.restore_original_limits()


def delta_err(p_old_gpu, p_new_gpu, p_old_ora, p_new_ora) -> float:
    """Error of the update itself: max |d_gpu - d_ora| / (|d_ora| + rms(d_ora)) with d = p_old - p_new on each side's
    own trajectory. p_new is stored in fp32 on the GPU, so |p_new| * 2^-23 of the difference is rounding of the
    parameter, not of the update, and is taken off first."""
    dg = np.asarray(p_old_gpu, np.float64) - np.asarray(p_new_gpu, np.float64)
    do = np.asarray(p_old_ora, np.float64) - np.asarray(p_new_ora, np.float64)
    err = np.maximum(np.abs(dg - do) - np.abs(np.asarray(p_new_ora, np.float64)) * 2.0 ** -23, 0.0)
    rms = float(np.sqrt(np.mean(do * do)))
    den = np.abs(do) + rms
    den[den == 0.0] = 1.0
    return float(np.max(err / den))


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


def make_cfg(kind: str, hidden=None, lstm_hidden=None, n_bank=None, apply_kernel=None, groups=None, state_pass=None):
    import paper_2506_10315_amd as P
    from paper_2506_10315_amd.binding import APPLY_KERNELS, STATE_PASSES
    cfg = P.default_config(P.LOPT_SMALL_FC if kind == "small_fc_lopt" else P.LOPT_VELO)
    if apply_kernel is not None:
        cfg.apply_kernel = APPLY_KERNELS[apply_kernel]
    if state_pass is not None:
        cfg.state_pass = STATE_PASSES[state_pass]
    if groups is not None:
        cfg.groups = groups
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


WORST_LSTM = [0.0]    # largest LSTM-state error seen by compare_state in this process (reported by the long runs)


def compare_state(gs, st, tag, tol=TOL_ACC):
    """Accumulators to `tol`, VeLO's LSTM state (h, c) to TOL_LSTM (the same bar: it is a function of the logarithms of
    the fp32 statistics through ~1100-term fp32 gate sums and feeds back into itself over the steps, and still stays
    an order of magnitude inside it)."""
    worst = 0.0
    for key in ("M", "V", "r", "c") + (("h", "cl") if "h" in st else ()):
        e = O.rel_err(gs[key], st[key])
        if key not in ("h", "cl"):
            worst = max(worst, e)
        else:
            WORST_LSTM[0] = max(WORST_LSTM[0], e)
        assert e <= (tol if key not in ("h", "cl") else TOL_LSTM), f"{tag}: accumulator {key} rel err {e:.3e}"
    return worst


def gpu_hidden_mean(opt):
    """mean_hidden over ALL tensors of the GPU's list, from the state blobs as they stand (before a step): what the
    oracle is given as the cross-tensor input when it follows only some of the tensors. None for small_fc_lopt."""
    import torch
    import paper_2506_10315_amd as P
    if opt.cfg.kind != P.LOPT_VELO:
        return None
    H = torch.stack([opt.state_views(i)["h"] for i in range(opt.n)]).cpu().numpy()
    return O.mean_hidden(list(H))


def run_free(case: Case, cfg, weights, steps, lr_fn=lambda t: 1.0, wd=0.0, check_every=1, device="cuda:0",
             check_stats=True, verbose=False, loss_fn=None, static=False):
    """Free-running parity: GPU and oracle both start from (p0, zero state) and take `steps` steps over the whole list
    on the same gradients (and loss values); parameters, the update itself, accumulators and statistics are compared
    after every `check_every` steps."""
    import torch
    import paper_2506_10315_amd as P
    ocfg = oracle_config_from(cfg)
    loss_fn = loss_fn or (lambda t: W.loss_at(case.config_id, t))   # VeLO takes a loss value with every step
    n = len(case.specs)
    shapes = [s.shape for s in case.specs]
    ndims = [s.as_2d()[0] for s in case.specs]
    opt = P.LearnedOptimizer(cfg, weights, shapes, device=device)
    p_gpu = [torch.from_numpy(case.p0(i)).to(device) for i in range(n)]
    p_ora = [case.p0(i).astype(np.float64) for i in range(n)]
    st_ora = [O.init_state(*p.shape, ocfg) for p in p_ora]
    worst = {"param": 0.0, "delta": 0.0, "acc": 0.0, "stats": 0.0}
    for t in range(steps):
        gs = [case.grad(i, t) for i in range(n)]
        g_gpu = [torch.from_numpy(g).to(device) for g in gs]
        lr = float(np.float32(lr_fn(t)))
        loss = float(np.float32(loss_fn(t)))
        checking = (t + 1) % check_every == 0 or t == steps - 1
        old_gpu = [p.cpu().numpy() for p in p_gpu] if checking else None
        old_ora = p_ora
        opt.step(p_gpu, g_gpu, lr=lr, weight_decay=float(np.float32(wd)), step=t, loss=loss, static=static)
        infos = [{} for _ in range(n)]
        p_ora = O.list_step(p_ora, gs, st_ora, weights, ocfg, t, lr, float(np.float32(wd)), ndims, loss=loss, outs=infos)
        if checking:
            torch.cuda.synchronize()
            stats = opt.stats() if check_stats else None
            for i in range(n):
                tag = f"step {t} tensor {i} {case.specs[i].shape}"
                new_gpu = p_gpu[i].cpu().numpy()
                e = O.rel_err(new_gpu, p_ora[i])
                worst["param"] = max(worst["param"], e)
                assert e <= TOL_PARAM, f"{tag}: parameter rel err {e:.3e}"
                e = delta_err(old_gpu[i], new_gpu, old_ora[i], p_ora[i])
                worst["delta"] = max(worst["delta"], e)
                assert e <= TOL_DELTA, f"{tag}: update rel err {e:.3e}"
                worst["acc"] = max(worst["acc"], compare_state(gpu_state_to_numpy(opt, i), st_ora[i], tag))
                if check_stats:
                    k = ocfg.n_normalized
                    s_g = stats[i].cpu().numpy()[:k].astype(np.float64)
                    s_o = infos[i]["stats"][:k].copy()
                    # feature 1 is the parameter itself: free-running, the two sides' parameters differ within
                    # TOL_PARAM, which alone moves mean(p^2) by up to twice that. The reduction is checked against the
                    # mean square of the GPU's own parameters before the step (the drift is the parameter check's job)
                    s_o[1] = O.compute_squared_average(old_gpu[i].astype(np.float64).reshape(-1, 1))[0]
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


def _seeded_device_param(case: Case, i: int, device):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(W.BASE_SEED + 7919 * case.indices[i])
    _, rows, cols = case.specs[i].as_2d()
    return torch.randn(rows, cols, generator=gen, device=device, dtype=torch.float32) * 0.02


def _row_slabs(m, rows=48):
    """First, middle and last row slabs of a tall tensor (the middle one straddles a tile boundary)."""
    if m <= 3 * rows:
        return [slice(0, m)]
    mid = (m // 2 // 64) * 64 - rows // 2
    return [slice(0, rows), slice(mid, mid + rows), slice(m - rows, m)]


def run_forced(case: Case, cfg, weights, steps, checks, lr_fn=lambda t: 1.0, wd=0.0, device="cuda:0",
               progress=print, closed_form_all_at_step0=True, loss_fn=None, slab_checks=None):
    """Teacher-forced parity at full size. The GPU free-runs `steps` steps over ALL tensors of the case in
    one lopt_step per step (the launch configuration bench.py times). `checks` maps a step index to the list
    of tensor indices the oracle verifies at that step: it takes ONE step from the GPU's own state before
    that step (widened to float64; VeLO's cross-tensor input is oracle.mean_hidden of the GPU's LSTM outputs of all
    tensors before the step) and parameters, the update and accumulators are compared element by element.
    `slab_checks` does the same for tensors too large to evaluate whole: accumulators in full, the statistics against
    oracle.tensor_statistics, parameters against oracle.apply_rows on the first, a middle and the last row slab.
    Tensors that appear in no check get seeded on-device gradients. At step 0 every tensor is also checked
    against the closed forms M_i = (1-beta_i) g, V = (1-beta_4) g^2 that hold after one step from zero state."""
    import torch
    import paper_2506_10315_amd as P
    ocfg = oracle_config_from(cfg)
    loss_fn = loss_fn or (lambda t: W.loss_at(case.config_id, t))   # VeLO takes a loss value with every step
    n = len(case.specs)
    shapes = [s.shape for s in case.specs]
    slab_checks = slab_checks or {}
    checked = sorted({i for v in checks.values() for i in v} | {i for v in slab_checks.values() for i in v})
    opt = P.LearnedOptimizer(cfg, weights, shapes, device=device)
    p_gpu = [torch.from_numpy(case.p0(i)).to(device) if i in checked else _seeded_device_param(case, i, device)
             for i in range(n)]
    worst = {"param": 0.0, "delta": 0.0, "acc": 0.0, "stats": 0.0, "closed_form": 0.0}
    k_norm = ocfg.n_normalized
    for t in range(steps):
        subset, big = checks.get(t, []), slab_checks.get(t, [])
        gs = dict(zip(checked, pool_map(lambda i: case.grad(i, t), checked)))
        g_gpu = [torch.from_numpy(gs[i]).to(device) if i in gs else _device_grad(case, i, t, device) for i in range(n)]
        lr, wdf, loss = float(np.float32(lr_fn(t))), float(np.float32(wd)), float(np.float32(loss_fn(t)))
        torch.cuda.synchronize()
        before = {i: (p_gpu[i].cpu().numpy().astype(np.float64),
                      {k: v.astype(np.float64) for k, v in gpu_state_to_numpy(opt, i).items()}) for i in subset + big}
        h_mix = gpu_hidden_mean(opt) if (subset or big) else None
        opt.step(p_gpu, g_gpu, lr=lr, weight_decay=wdf, step=t, loss=loss)
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

        def verify(i):
            p_b, st = before[i]
            info = {}
            p_o = O.tensor_step(p_b, gs[i], st, weights, ocfg, t, lr, wdf, ndim=case.specs[i].as_2d()[0], out=info,
                                loss=loss, h_mix=h_mix)
            return p_o, st, info

        stats_gpu = opt.stats() if subset or big else None
        for i, (p_o, st, info) in zip(subset, pool_map(verify, subset)):
            tag = f"step {t} tensor {i} {case.specs[i].name} {case.specs[i].shape}"
            new_gpu = p_gpu[i].cpu().numpy()
            e = O.rel_err(new_gpu, p_o)
            worst["param"] = max(worst["param"], e)
            assert e <= TOL_PARAM, f"{tag}: parameter rel err {e:.3e}"
            e = delta_err(before[i][0], new_gpu, before[i][0], p_o)
            worst["delta"] = max(worst["delta"], e)
            assert e <= TOL_DELTA, f"{tag}: update rel err {e:.3e}"
            worst["acc"] = max(worst["acc"], compare_state(gpu_state_to_numpy(opt, i), st, tag))
            s_g = stats_gpu[i].cpu().numpy()[:k_norm].astype(np.float64)
            es = float(np.max(np.abs(s_g - info["stats"][:k_norm]) / (np.abs(info["stats"][:k_norm]) + ocfg.eps_norm)))
            worst["stats"] = max(worst["stats"], es)
            assert es <= TOL_STATS, f"{tag}: statistics rel err {es:.3e}"

        def verify_big(i):
            # the steps of oracle.tensor_step, with the apply half on row slabs only
            p_b, st = before[i]
            O.update_accumulators(st, gs[i], ocfg)
            s_o = O.tensor_statistics(p_b, gs[i], st, ocfg, t)
            if ocfg.kind == O.KIND_SMALL_FC:
                theta, lam = weights, 1.0
            else:
                theta, lam = O.velo_hypernetwork(s_o, t, case.specs[i].as_2d()[0], st, weights, ocfg, loss, h_mix)
            slabs = _row_slabs(p_b.shape[0])
            return st, s_o, [(sl, O.apply_rows(p_b, gs[i], st, s_o, theta, ocfg, t, lr, wdf, sl, lam)) for sl in slabs]

        for i, (st, s_o, slabs) in zip(big, pool_map(verify_big, big)):
            tag = f"step {t} tensor {i} {case.specs[i].name} {case.specs[i].shape}"
            worst["acc"] = max(worst["acc"], compare_state(gpu_state_to_numpy(opt, i), st, tag))
            s_g = stats_gpu[i].cpu().numpy()[:k_norm].astype(np.float64)
            es = float(np.max(np.abs(s_g - s_o[:k_norm]) / (np.abs(s_o[:k_norm]) + ocfg.eps_norm)))
            worst["stats"] = max(worst["stats"], es)
            assert es <= TOL_STATS, f"{tag}: statistics rel err {es:.3e}"
            for sl, p_o in slabs:
                new_gpu = p_gpu[i][sl].cpu().numpy()
                e = O.rel_err(new_gpu, p_o)
                worst["param"] = max(worst["param"], e)
                assert e <= TOL_PARAM, f"{tag} rows {sl.start}:{sl.stop}: parameter rel err {e:.3e}"
                e = delta_err(before[i][0][sl], new_gpu, before[i][0][sl], p_o)
                worst["delta"] = max(worst["delta"], e)
                assert e <= TOL_DELTA, f"{tag} rows {sl.start}:{sl.stop}: update rel err {e:.3e}"
            progress(f"  {tag}: accumulators, statistics and {len(slabs)} row slabs ok")
        progress(f"  step {t} done ({len(subset)} tensors whole, {len(big)} by slabs): worst so far {worst}")
        del g_gpu, before
    for i in range(n):
        assert bool(torch.isfinite(p_gpu[i]).all()), f"tensor {i}: non-finite parameter at the end"
    opt.close()
    return worst


def run_free_subset(case: Case, cfg, weights, steps, subset, check_steps, lr_fn=lambda t: 1.0, wd=0.0,
                    device="cuda:0", progress=print, loss_fn=None, limits=None):
    """Free-running parity over many steps at full size. The GPU takes `steps` steps over ALL tensors of the case
    (one lopt_step per step); the oracle free-runs the tensors in `subset` from the same start and parameters, the
    update and accumulators are compared after the steps in `check_steps`. `limits` maps a tensor index to the number of
    steps the oracle follows it (default: all of them). Everything of a followed tensor free-runs on both sides; the
    one thing the oracle takes from the GPU is VeLO's cross-tensor input (oracle.mean_hidden of the LSTM outputs of
    ALL tensors, which the oracle cannot know without stepping every tensor). Tensors outside the subset get seeded
    on-device parameters and gradients."""
    import torch
    import paper_2506_10315_amd as P
    ocfg = oracle_config_from(cfg)
    loss_fn = loss_fn or (lambda t: W.loss_at(case.config_id, t))   # VeLO takes a loss value with every step
    n = len(case.specs)
    sub = sorted(subset)
    limits = limits or {}
    opt = P.LearnedOptimizer(cfg, weights, [s.shape for s in case.specs], device=device)
    p_gpu = [torch.from_numpy(case.p0(i)).to(device) if i in sub else _seeded_device_param(case, i, device)
             for i in range(n)]
    p_ora = {i: case.p0(i).astype(np.float64) for i in sub}
    st_ora = {i: O.init_state(*p_ora[i].shape, ocfg) for i in sub}
    worst = {"param": 0.0, "delta": 0.0, "acc": 0.0}
    velo = ocfg.kind == O.KIND_VELO
    for t in range(steps):
        live = [i for i in sub if t < limits.get(i, steps)]
        gs = dict(zip(live, pool_map(lambda i: case.grad(i, t), live)))
        g_gpu = [torch.from_numpy(gs[i]).to(device) if i in gs else _device_grad(case, i, t, device) for i in range(n)]
        lr, wdf, loss = float(np.float32(lr_fn(t))), float(np.float32(wd)), float(np.float32(loss_fn(t)))
        checking = t in check_steps or any(t == limits.get(i, steps) - 1 for i in live)
        h_mix = gpu_hidden_mean(opt) if velo and live else None
        old_gpu = {i: p_gpu[i].cpu().numpy() for i in live} if checking else None
        opt.step(p_gpu, g_gpu, lr=lr, weight_decay=wdf, step=t, loss=loss)
        old_ora = {i: p_ora[i] for i in live}
        new = pool_map(lambda i: O.tensor_step(p_ora[i], gs[i], st_ora[i], weights, ocfg, t, lr, wdf,
                                               ndim=case.specs[i].as_2d()[0], loss=loss, h_mix=h_mix), live)
        for i, pn in zip(live, new):
            p_ora[i] = pn
        if checking:
            torch.cuda.synchronize()
            for i in live:
                tag = f"step {t} tensor {i} {case.specs[i].name} {case.specs[i].shape}"
                new_gpu = p_gpu[i].cpu().numpy()
                e = O.rel_err(new_gpu, p_ora[i])
                worst["param"] = max(worst["param"], e)
                assert e <= TOL_PARAM, f"{tag}: parameter rel err {e:.3e}"
                e = delta_err(old_gpu[i], new_gpu, old_ora[i], p_ora[i])
                worst["delta"] = max(worst["delta"], e)
                assert e <= TOL_DELTA, f"{tag}: update rel err {e:.3e}"
                worst["acc"] = max(worst["acc"], compare_state(gpu_state_to_numpy(opt, i), st_ora[i], tag))
            progress(f"  step {t}: {len(live)} tensors followed, worst so far {worst}")
        del g_gpu
    torch.cuda.synchronize()
    for i in range(n):
        assert bool(torch.isfinite(p_gpu[i]).all()), f"tensor {i}: non-finite parameter at the end"
    opt.close()
    return worst
