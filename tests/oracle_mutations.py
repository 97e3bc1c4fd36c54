"""Deliberate mistakes planted in the CPU oracle (on the CPU only). tests/test_oracle_mutations.py runs the pin
suite once per mutation and expects it to fail: evidence that a plausible slip anywhere in the oracle (a
dropped term, a wrong sign or axis, a transposed operand) is caught by at least one pin."""
import numpy as np


def _wrap(O, name, fn):
    orig = getattr(O, name)
    setattr(O, name, lambda *a, **k: fn(orig, *a, **k))


def swap_row_col_axes(O):
    def f(orig, st, g, cfg):
        g = np.asarray(g, float)
        before_r, before_c = st["r"].copy(), st["c"].copy()
        orig(st, g, cfg)
        g2 = g * g
        if g.shape[0] == g.shape[1]:
            for k in range(3):
                b = cfg.fac_decay[k]
                st["r"][k] = b * before_r[k] + (1 - b) * g2.mean(axis=0)
                st["c"][k] = b * before_c[k] + (1 - b) * g2.mean(axis=1)
        else:   # non-square: use a sum over the wrong axis scaled to the right length
            for k in range(3):
                b = cfg.fac_decay[k]
                st["r"][k] = b * before_r[k] + (1 - b) * np.resize(g2.mean(axis=0), g.shape[0])
                st["c"][k] = b * before_c[k] + (1 - b) * np.resize(g2.mean(axis=1), g.shape[1])
    _wrap(O, "update_accumulators", f)


def momentum_without_one_minus_beta(O):
    def f(orig, st, g, cfg):
        M = st["M"].copy()
        orig(st, g, cfg)
        for i in range(3):
            st["M"][i] = cfg.mom_decay[i] * M[i] + np.asarray(g, float)
    _wrap(O, "update_accumulators", f)


def second_moment_uses_abs_instead_of_square(O):
    def f(orig, st, g, cfg):
        V = st["V"].copy()
        orig(st, g, cfg)
        st["V"] = cfg.rms_decay * V + (1 - cfg.rms_decay) * np.abs(np.asarray(g, float))
    _wrap(O, "update_accumulators", f)


def update_added_instead_of_subtracted(O):
    def f(orig, direction, magnitude, cfg):
        return -orig(direction, magnitude, cfg)
    _wrap(O, "delta_theta", f)


def exp_multiplier_dropped(O):
    def f(orig, direction, magnitude, cfg):
        return direction * np.exp(magnitude) * cfg.step_mult
    _wrap(O, "delta_theta", f)


def normalization_without_square_root(O):
    def f(orig, F, s, cfg):
        out = F.copy()
        k = cfg.n_normalized
        out[:, :k] = F[:, :k] / (s[:k] + cfg.eps_norm)
        return out
    _wrap(O, "feature_normalization", f)


def time_features_normalized_too(O):
    def f(orig, F, s, cfg):
        return F / np.sqrt(s + cfg.eps_norm + 1e-300)
    _wrap(O, "feature_normalization", f)


def statistics_are_mean_not_mean_square(O):
    def f(orig, F):
        return np.abs(F).mean(axis=0)
    _wrap(O, "compute_squared_average", f)


def outputs_swapped(O):
    def f(orig, Fn, theta, cfg):
        d, m = orig(Fn, theta, cfg)
        return m, d
    _wrap(O, "apply_lo", f)


def second_relu_missing(O):
    def f(orig, Fn, theta, cfg):
        W1, b1, W2, b2, W3, b3 = O.unpack_mlp(theta, cfg.d_feat, cfg.hidden)
        h = np.maximum(Fn @ W1 + b1, 0.0)
        h = h @ W2 + b2
        out = h @ W3 + b3
        return out[:, 0], out[:, 1]
    _wrap(O, "apply_lo", f)


def w2_transposed(O):
    def f(orig, Fn, theta, cfg):
        W1, b1, W2, b2, W3, b3 = O.unpack_mlp(theta, cfg.d_feat, cfg.hidden)
        h = np.maximum(Fn @ W1 + b1, 0.0)
        h = np.maximum(h @ W2.T + b2, 0.0)
        out = h @ W3 + b3
        return out[:, 0], out[:, 1]
    _wrap(O, "apply_lo", f)


def factored_feature_without_row_mean(O):
    def f(orig, p, g, st, cfg, t, rows=slice(None)):
        F = orig(p, g, st, cfg, t, rows)
        for k in range(3):
            rbar = st["r"][k].mean()
            F[:, 10 + k] /= np.sqrt(rbar + cfg.eps_acc)
        return F
    _wrap(O, "construct_features", f)


def momentum_factor_pairing_shifted(O):
    def f(orig, p, g, st, cfg, t, rows=slice(None)):
        F = orig(p, g, st, cfg, t, rows)
        F[:, 25:28] = F[:, [26, 27, 25]]
        return F
    _wrap(O, "construct_features", f)


def clip_bound_wrong(O):
    O.GRAD_CLIP = 1.0


def time_scale_wrong(O):
    O.TIME_SCALES = (1.0, 3.0, 10.0, 30.0, 100.0, 300.0, 1000.0, 3000.0, 1e4, 3e4, 1e6)


def lstm_gate_order_ifog(O):
    def f(orig, u, h, c, Wx, Wh, b):
        HL = h.shape[0]
        z = u @ Wx + h @ Wh + b
        i, fg, o, g = z[:HL], z[HL:2 * HL], z[2 * HL:3 * HL], z[3 * HL:]
        sg = lambda x: 1 / (1 + np.exp(-x))
        c_new = sg(fg) * c + sg(i) * np.tanh(g)
        return sg(o) * np.tanh(c_new), c_new
    _wrap(O, "lstm_cell", f)


def weight_decay_uses_new_parameter(O):
    def f(orig, p, g, st, weights, cfg, t, lr, wd, **kw):
        p_new = orig(p, g, st, weights, cfg, t, lr, 0.0, **kw)
        return p_new * (1 - lr * wd) - 1e-3 * wd * np.sign(p_new)
    _wrap(O, "tensor_step", f)


def loss_features_dropped(O):
    def f(orig, loss):
        return 0.0 * orig(loss)
    _wrap(O, "loss_features", f)


def loss_features_not_odd(O):
    def f(orig, loss):
        return orig(abs(loss))
    _wrap(O, "loss_features", f)


def cross_tensor_term_is_a_sum(O):
    def f(orig, hs):
        return orig(hs) * len(hs)
    _wrap(O, "mean_hidden", f)


def cross_tensor_term_ignored(O):
    def f(orig, s, t, ndim, st, weights, cfg, loss=0.0, h_mix=None):
        return orig(s, t, ndim, st, weights, cfg, loss, None)
    _wrap(O, "velo_hypernetwork", f)


def cross_tensor_term_taken_after_the_state_moved(O):
    def f(ps, gs, sts, weights, cfg, t, lr, wd, ndims, loss=0.0, outs=None):
        res = []
        for i in range(len(ps)):
            h_mix = O.mean_hidden([st["h"] for st in sts]) if cfg.kind == O.KIND_VELO else None
            res.append(O.tensor_step(ps[i], gs[i], sts[i], weights, cfg, t, lr, wd, ndim=ndims[i],
                                     out=None if outs is None else outs[i], loss=loss, h_mix=h_mix))
        return res
    O.list_step = f


def step_size_output_not_applied(O):
    def f(orig, s, t, ndim, st, weights, cfg, loss=0.0, h_mix=None):
        theta, lam = orig(s, t, ndim, st, weights, cfg, loss, h_mix)
        return theta, 1.0
    _wrap(O, "velo_hypernetwork", f)


def step_size_scales_the_decay_too(O):
    def f(orig, p, g, st, weights, cfg, t, lr, wd, **kw):
        out = kw.get("out")
        info = out if out is not None else {}
        kw["out"] = info
        p_new = orig(p, g, st, weights, cfg, t, lr, wd, **kw)
        lam = info.get("lam", 1.0)
        return p_new - lr * wd * (lam - 1.0) * np.asarray(p, float)
    _wrap(O, "tensor_step", f)


MUTATIONS = {f.__name__: f for f in [
    loss_features_dropped, loss_features_not_odd, cross_tensor_term_is_a_sum, cross_tensor_term_ignored,
    cross_tensor_term_taken_after_the_state_moved, step_size_output_not_applied, step_size_scales_the_decay_too,
    swap_row_col_axes, momentum_without_one_minus_beta, second_moment_uses_abs_instead_of_square,
    update_added_instead_of_subtracted, exp_multiplier_dropped, normalization_without_square_root,
    time_features_normalized_too, statistics_are_mean_not_mean_square, outputs_swapped, second_relu_missing,
    w2_transposed, factored_feature_without_row_mean, momentum_factor_pairing_shifted, clip_bound_wrong,
    time_scale_wrong, lstm_gate_order_ifog, weight_decay_uses_new_parameter]}
