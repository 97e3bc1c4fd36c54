"""Pins for the CPU oracle: closed forms, invariants, library routines, brute force.

None of these re-types the oracle's own vectorised formulae: each pin is either a
closed form that follows from the update rules of the paper's feature tables, a
value the paper prints (tests/golden/paper_constants.txt), a library routine
(numpy mean/matmul, torch LSTMCell), or a scalar-loop brute force on a tiny tensor.
"""
import math

import numpy as np
import pytest

from oracle import lopt_oracle as O


def cfg(kind=O.KIND_SMALL_FC, **kw):
    return O.OracleConfig(kind=kind, **kw)


def velo_size(H, HL, K):
    """Floats in a VeLO weight blob: Wx[48,4HL] Wh[HL,4HL] Wg[HL,4HL] b[4HL] Wa[HL,K] ba[K] ws[HL] bs[1] B[K,P]."""
    P = 29 * H + H + H * H + H + 2 * H + 2
    return 48 * 4 * HL + 2 * HL * 4 * HL + 4 * HL + HL * K + K + HL + 1 + K * P


def rand_state_after(steps, m, n, c, seed=0, scale=1e-3):
    rng = np.random.default_rng(seed)
    st = O.init_state(m, n, c)
    g = None
    for _ in range(steps):
        g = rng.standard_normal((m, n)) * scale
        O.update_accumulators(st, g, c)
    return st, g, rng


# ------------------------------------------------------------------ constants the paper prints

def test_constants_match_paper(paper_constants):
    pc = paper_constants
    c = cfg()
    assert c.exp_mult == pytest.approx(pc["alpha"], rel=1e-7)
    assert c.step_mult == pytest.approx(pc["beta"], rel=1e-7)
    assert list(O.TIME_SCALES) == pc["time_scales"]
    assert len(O.TIME_SCALES) == pc["n_time_features"]
    assert cfg(O.KIND_SMALL_FC).d_feat == pc["d_feat_small_fc"]
    assert cfg(O.KIND_VELO).d_feat == pc["d_feat_velo"]
    assert O.GRAD_CLIP == pc["grad_clip"]
    assert c.hidden == pc["hidden_small_fc"]
    st = O.init_state(5, 7, c)
    assert st["M"].shape[0] == pc["n_momentum"]
    assert st["r"].shape == (pc["n_row_acc"], 5)
    assert st["c"].shape == (pc["n_col_acc"], 7)


# ------------------------------------------------------------------ accumulators

@pytest.mark.parametrize("k", [1, 2, 7, 40])
def test_accumulators_constant_gradient_closed_form(k):
    c = cfg()
    rng = np.random.default_rng(1)
    g = rng.standard_normal((6, 5)) * 1e-2
    st = O.init_state(6, 5, c)
    for _ in range(k):
        O.update_accumulators(st, g, c)
    for i in range(3):
        np.testing.assert_allclose(st["M"][i], (1 - c.mom_decay[i] ** k) * g, rtol=1e-12)
    np.testing.assert_allclose(st["V"], (1 - c.rms_decay ** k) * g * g, rtol=1e-12)
    for j in range(3):
        b = c.fac_decay[j]
        np.testing.assert_allclose(st["r"][j], (1 - b ** k) * np.mean(g * g, axis=1), rtol=1e-12)
        np.testing.assert_allclose(st["c"][j], (1 - b ** k) * np.mean(g * g, axis=0), rtol=1e-12)


def test_row_is_mean_over_columns_col_is_mean_over_rows():
    # a gradient that is non-zero in one row only: r lights up in that row, c everywhere
    c = cfg()
    g = np.zeros((4, 3))
    g[2, :] = [1.0, 2.0, 3.0]
    st = O.init_state(4, 3, c)
    O.update_accumulators(st, g, c)
    b = c.fac_decay[0]
    np.testing.assert_allclose(st["r"][0], (1 - b) * np.array([0, 0, (1 + 4 + 9) / 3, 0]), rtol=1e-12)
    np.testing.assert_allclose(st["c"][0], (1 - b) * np.array([1, 4, 9]) / 4, rtol=1e-12)


def test_different_decays_are_used_per_accumulator():
    c = cfg(mom_decay=(0.5, 0.25, 0.125), rms_decay=0.75, fac_decay=(0.1, 0.2, 0.3))
    g = np.full((2, 2), 2.0)
    st = O.init_state(2, 2, c)
    O.update_accumulators(st, g, c)
    assert [st["M"][i][0, 0] for i in range(3)] == pytest.approx([1.0, 1.5, 1.75])
    assert st["V"][0, 0] == pytest.approx(1.0)
    assert [st["r"][k][0] for k in range(3)] == pytest.approx([3.6, 3.2, 2.8])
    assert [st["c"][k][0] for k in range(3)] == pytest.approx([3.6, 3.2, 2.8])


# ------------------------------------------------------------------ features

def test_factored_feature_rank_one_closed_form():
    # g_ij = u_i w_j  =>  r_i c_j / mean(r) = (1-beta^k) g_ij^2  =>  feature = sign(g)/sqrt(1-beta^k)
    c = cfg(eps_acc=0.0)
    rng = np.random.default_rng(2)
    u = rng.uniform(0.5, 2.0, 7) * rng.choice([-1, 1], 7)
    w = rng.uniform(0.5, 2.0, 5) * rng.choice([-1, 1], 5)
    g = np.outer(u, w)
    st = O.init_state(7, 5, c)
    for k in range(1, 4):
        O.update_accumulators(st, g, c)
        F = O.construct_features(np.zeros_like(g), g, st, c, 0)
        for j in range(3):
            expect = np.sign(g).ravel() / math.sqrt(1 - c.fac_decay[j] ** k)
            np.testing.assert_allclose(F[:, 10 + j], expect, rtol=1e-11)
            # momentum feature: M_j = (1-beta_j^k) g
            expect_m = (1 - c.mom_decay[j] ** k) * expect
            np.testing.assert_allclose(F[:, 25 + j], expect_m, rtol=1e-11)


def test_one_dimensional_tensor_reduces_to_rms_normalised_gradient():
    c = cfg(eps_acc=0.0)
    rng = np.random.default_rng(3)
    st = O.init_state(1, 9, c)
    for _ in range(3):
        g = rng.standard_normal((1, 9))
        O.update_accumulators(st, g, c)
    F = O.construct_features(np.zeros_like(g), g, st, c, 0)
    for k in range(3):
        # rows=1: mean(r)=r so a=1 and the factor is 1/sqrt(c_j)
        np.testing.assert_allclose(F[:, 10 + k], g.ravel() / np.sqrt(st["c"][k]), rtol=1e-12)


def test_plain_features_are_the_inputs_themselves():
    c = cfg(O.KIND_VELO)
    st, g, rng = rand_state_after(3, 4, 6, c, seed=4, scale=0.3)   # some |g| > 0.1
    p = rng.standard_normal((4, 6))
    F = O.construct_features(p, g, st, c, 5)
    np.testing.assert_array_equal(F[:, 0], g.ravel())
    np.testing.assert_array_equal(F[:, 1], p.ravel())
    for i in range(3):
        np.testing.assert_array_equal(F[:, 2 + i], st["M"][i].ravel())
    np.testing.assert_array_equal(F[:, 5], st["V"].ravel())
    # element (i, j) is at flat index i*n + j: broadcast features tell rows from columns
    F3 = F.reshape(4, 6, -1)
    for k in range(3):
        for i in range(4):
            assert np.all(F3[i, :, 13 + k] == st["r"][k][i])
        for j in range(6):
            assert np.all(F3[:, j, 16 + k] == st["c"][k][j])
    clipped = F[:, 28]
    assert clipped.max() == pytest.approx(0.1) and clipped.min() == pytest.approx(-0.1)
    inside = np.abs(g.ravel()) <= 0.1
    np.testing.assert_array_equal(clipped[inside], g.ravel()[inside])


def test_time_features():
    tf0 = O.time_features(0)
    assert np.all(tf0 == 0.0)
    tf = O.time_features(3)
    assert tf[1] == pytest.approx(0.7615941559557649, rel=1e-15)        # tanh(1), t = x = 3
    assert O.time_features(100000)[10] == pytest.approx(0.7615941559557649, rel=1e-15)
    assert np.all(np.diff(O.time_features(50)) < 0)                    # larger scale, smaller value
    c = cfg()
    st, g, _ = rand_state_after(1, 3, 3, c)
    F = O.construct_features(g, g, st, c, 30)
    np.testing.assert_allclose(F[:, 28:], np.tile(np.tanh(30 / np.array(O.TIME_SCALES)), (9, 1)))


def test_broadcast_feature_statistics_follow_from_r_and_c_alone():
    c = cfg()
    st, g, rng = rand_state_after(4, 5, 8, c, seed=5)
    F = O.construct_features(g, g, st, c, 1)
    s = O.compute_squared_average(F)
    e = c.eps_acc
    for k in range(3):
        assert s[13 + k] == pytest.approx(np.mean(st["r"][k] ** 2), rel=1e-12)
        assert s[16 + k] == pytest.approx(np.mean(st["c"][k] ** 2), rel=1e-12)
        assert s[19 + k] == pytest.approx(np.mean(1 / (st["r"][k] + e)), rel=1e-12)
        assert s[22 + k] == pytest.approx(np.mean(1 / (st["c"][k] + e)), rel=1e-12)


# ------------------------------------------------------------------ normalization

@pytest.mark.parametrize("kind", [O.KIND_SMALL_FC, O.KIND_VELO])
def test_normalized_features_have_unit_mean_square(kind):
    c = cfg(kind, eps_norm=0.0)
    st, g, rng = rand_state_after(3, 6, 7, c, seed=6)
    p = rng.standard_normal((6, 7)) * 0.02
    F = O.construct_features(p, g, st, c, 4)
    s = O.compute_squared_average(F)
    Fn = O.feature_normalization(F, s, c)
    k = c.n_normalized
    np.testing.assert_allclose(np.mean(Fn[:, :k] ** 2, axis=0), np.ones(k), rtol=1e-12)
    # time features pass through untouched
    if kind == O.KIND_SMALL_FC:
        np.testing.assert_array_equal(Fn[:, k:], F[:, k:])


def test_normalization_with_eps_closed_form():
    c = cfg(eps_norm=0.5)
    st, g, rng = rand_state_after(2, 3, 4, c, seed=7, scale=1.0)
    F = O.construct_features(g, g, st, c, 0)
    s = O.compute_squared_average(F)
    Fn = O.feature_normalization(F, s, c)
    np.testing.assert_allclose(np.mean(Fn[:, :28] ** 2, axis=0), s[:28] / (s[:28] + 0.5), rtol=1e-12)


def test_gradient_scale_invariance_of_normalized_features():
    c = cfg(eps_acc=0.0, eps_norm=0.0)
    rng = np.random.default_rng(8)
    p = rng.standard_normal((5, 4))
    outs = []
    for lam in (1.0, 37.5):
        r2 = np.random.default_rng(9)
        st = O.init_state(5, 4, c)
        for t in range(3):
            g = r2.standard_normal((5, 4)) * lam
            O.update_accumulators(st, g, c)
        F = O.construct_features(p, g, st, c, 3)
        outs.append(O.feature_normalization(F, O.compute_squared_average(F), c))
    np.testing.assert_allclose(outs[0], outs[1], rtol=1e-10)


@pytest.mark.parametrize("kind", [O.KIND_SMALL_FC, O.KIND_VELO])
def test_row_and_column_permutation_equivariance(kind):
    c = cfg(kind, hidden=5, lstm_hidden=6, n_bank=3)
    rng = np.random.default_rng(10)
    m, n = 5, 6
    pr, pc_ = rng.permutation(m), rng.permutation(n)
    if kind == O.KIND_SMALL_FC:
        theta = rng.standard_normal(39 * 5 + 5 + 25 + 5 + 10 + 2) * 0.3
    else:
        n_theta = 29 * 5 + 5 + 25 + 5 + 10 + 2
        theta = rng.standard_normal(velo_size(5, 6, 3)) * 0.3
    p0 = rng.standard_normal((m, n)) * 0.02
    gs = [rng.standard_normal((m, n)) * 1e-2 for _ in range(3)]

    def run(perm):
        p = p0[pr][:, pc_] if perm else p0.copy()
        st = O.init_state(m, n, c)
        for t, g in enumerate(gs):
            gg = g[pr][:, pc_] if perm else g
            p = O.tensor_step(p, gg, st, theta, c, t, 0.7, 0.01)
        return p

    np.testing.assert_allclose(run(True), run(False)[pr][:, pc_], rtol=1e-9, atol=1e-15)


# ------------------------------------------------------------------ MLP and update

def _theta(d, H, W1=None, b1=None, W2=None, b2=None, W3=None, b3=None):
    z = lambda *s: np.zeros(s)
    parts = [W1 if W1 is not None else z(d, H), b1 if b1 is not None else z(H),
             W2 if W2 is not None else z(H, H), b2 if b2 is not None else z(H),
             W3 if W3 is not None else z(H, 2), b3 if b3 is not None else z(2)]
    return np.concatenate([np.asarray(x, float).ravel() for x in parts])


def test_zero_weights_constant_output_update(paper_constants):
    # only b3 = (d0, m0) non-zero: delta = beta * d0 * exp(alpha * m0) for every element
    c = cfg(hidden=4)
    d0, m0 = 0.6, -3.0
    theta = _theta(39, 4, b3=[d0, m0])
    rng = np.random.default_rng(11)
    p = rng.standard_normal((3, 5))
    g = rng.standard_normal((3, 5))
    st = O.init_state(3, 5, c)
    p1 = O.tensor_step(p, g, st, theta, c, 0, 1.0, 0.0)
    expect = paper_constants["beta"] * d0 * math.exp(paper_constants["alpha"] * m0)
    np.testing.assert_allclose(p - p1, np.full_like(p, expect), rtol=1e-6)   # update is subtracted
    # lr scales the update
    st = O.init_state(3, 5, c)
    p2 = O.tensor_step(p, g, st, theta, c, 0, 0.25, 0.0)
    np.testing.assert_allclose(p - p2, np.full_like(p, 0.25 * expect), rtol=1e-6)


def test_direction_is_output_zero_magnitude_is_output_one():
    c = cfg(hidden=2)
    Fn = np.zeros((1, 39))
    dirn, mag = O.apply_lo(Fn, _theta(39, 2, b3=[2.0, 5.0]), c)
    assert dirn[0] == 2.0 and mag[0] == 5.0


def test_mlp_is_affine_when_relus_are_inactive():
    c = cfg(hidden=6)
    rng = np.random.default_rng(12)
    W1 = rng.standard_normal((39, 6)) * 0.1
    W2 = rng.standard_normal((6, 6)) * 0.1
    W3 = rng.standard_normal((6, 2))
    b1 = np.full(6, 100.0)
    b2 = np.full(6, 100.0)
    b3 = rng.standard_normal(2)
    X = rng.standard_normal((17, 39))
    dirn, mag = O.apply_lo(X, _theta(39, 6, W1, b1, W2, b2, W3, b3), c)
    A = W1 @ W2 @ W3
    off = (b1 @ W2 + b2) @ W3 + b3
    np.testing.assert_allclose(np.stack([dirn, mag], 1), X @ A + off, rtol=1e-10)


def test_relu_clamps_negative_preactivations():
    c = cfg(hidden=1)
    # x0 -> h1 = relu(x0), h2 = relu(h1), direction = h2
    W1 = np.zeros((39, 1)); W1[0, 0] = 1.0
    theta = _theta(39, 1, W1, None, [[1.0]], None, [[1.0, 0.0]], None)
    X = np.zeros((3, 39)); X[:, 0] = [-2.0, 0.0, 3.0]
    dirn, _ = O.apply_lo(X, theta, c)
    np.testing.assert_array_equal(dirn, [0.0, 0.0, 3.0])
    # second ReLU: h1 = relu(x0) >= 0, W2 = -1 makes h2's pre-activation negative
    theta = _theta(39, 1, W1, None, [[-1.0]], None, [[1.0, 0.0]], None)
    dirn, _ = O.apply_lo(X, theta, c)
    np.testing.assert_array_equal(dirn, [0.0, 0.0, 0.0])


def test_weight_decay_closed_form():
    c = cfg(hidden=3)
    theta = _theta(39, 3)                 # MLP outputs exactly zero
    rng = np.random.default_rng(13)
    p0 = rng.standard_normal((4, 4))
    p = p0.copy()
    st = O.init_state(4, 4, c)
    lr, wd = 0.5, 0.1
    for t in range(6):
        p = O.tensor_step(p, rng.standard_normal((4, 4)), st, theta, c, t, lr, wd)
    np.testing.assert_allclose(p, p0 * (1 - lr * wd) ** 6, rtol=1e-12)


# ------------------------------------------------------------------ brute force, 4 x 3

def _brute_force_step(p, g, M, V, r, c, theta, C, kind, t, lr, wd, lam=1.0):
    """Scalar-loop implementation straight from the feature tables; lists only."""
    m, n = len(p), len(p[0])
    H = C.hidden
    bm, b4, bf, e = C.mom_decay, C.rms_decay, C.fac_decay, C.eps_acc
    for i in range(m):
        for j in range(n):
            for a in range(3):
                M[a][i][j] = bm[a] * M[a][i][j] + (1 - bm[a]) * g[i][j]
            V[i][j] = b4 * V[i][j] + (1 - b4) * g[i][j] ** 2
    for k in range(3):
        for i in range(m):
            r[k][i] = bf[k] * r[k][i] + (1 - bf[k]) * sum(g[i][j] ** 2 for j in range(n)) / n
        for j in range(n):
            c[k][j] = bf[k] * c[k][j] + (1 - bf[k]) * sum(g[i][j] ** 2 for i in range(m)) / m
    d = 39 if kind == O.KIND_SMALL_FC else 29
    feats = {}
    for i in range(m):
        for j in range(n):
            f = [g[i][j], p[i][j], M[0][i][j], M[1][i][j], M[2][i][j], V[i][j]]
            f += [M[a][i][j] / math.sqrt(V[i][j] + e) for a in range(3)]
            f += [1 / math.sqrt(V[i][j] + e)]
            fac = [math.sqrt((sum(r[k]) / m + e) / ((r[k][i] + e) * (c[k][j] + e))) for k in range(3)]
            f += [g[i][j] * fac[k] for k in range(3)]
            f += [r[k][i] for k in range(3)]
            f += [c[k][j] for k in range(3)]
            f += [1 / math.sqrt(r[k][i] + e) for k in range(3)]
            f += [1 / math.sqrt(c[k][j] + e) for k in range(3)]
            f += [M[k][i][j] * fac[k] for k in range(3)]
            if kind == O.KIND_SMALL_FC:
                f += [math.tanh(t / x) for x in (1, 3, 10, 30, 100, 300, 1000, 3000, 10000, 30000, 100000)]
            else:
                f += [max(-0.1, min(0.1, g[i][j]))]
            assert len(f) == d
            feats[(i, j)] = f
    n_norm = 28 if kind == O.KIND_SMALL_FC else 29
    s = [sum(feats[(i, j)][q] ** 2 for i in range(m) for j in range(n)) / (m * n) for q in range(d)]
    th = list(theta)
    W1 = [[th[q * H + u] for u in range(H)] for q in range(d)]; o = d * H
    b1 = th[o:o + H]; o += H
    W2 = [[th[o + q * H + u] for u in range(H)] for q in range(H)]; o += H * H
    b2 = th[o:o + H]; o += H
    W3 = [[th[o + q * 2 + u] for u in range(2)] for q in range(H)]; o += 2 * H
    b3 = th[o:o + 2]
    out = [[0.0] * n for _ in range(m)]
    for i in range(m):
        for j in range(n):
            x = [feats[(i, j)][q] / math.sqrt(s[q] + C.eps_norm) if q < n_norm else feats[(i, j)][q]
                 for q in range(d)]
            h1 = [max(0.0, b1[u] + sum(x[q] * W1[q][u] for q in range(d))) for u in range(H)]
            h2 = [max(0.0, b2[u] + sum(h1[q] * W2[q][u] for q in range(H))) for u in range(H)]
            o2 = [b3[u] + sum(h2[q] * W3[q][u] for q in range(H)) for u in range(2)]
            delta = lam * o2[0] * math.exp(o2[1] * C.exp_mult) * C.step_mult
            out[i][j] = p[i][j] - lr * (delta + wd * p[i][j])
    return out, s


def test_small_fc_4x3_against_scalar_brute_force():
    C = cfg(hidden=3)
    rng = np.random.default_rng(14)
    m, n = 4, 3
    theta = rng.uniform(-0.8, 0.8, 39 * 3 + 3 + 9 + 3 + 6 + 2)
    p = rng.standard_normal((m, n)) * 0.05
    st = O.init_state(m, n, C)
    M = [[[0.0] * n for _ in range(m)] for _ in range(3)]
    V = [[0.0] * n for _ in range(m)]
    r = [[0.0] * m for _ in range(3)]
    c = [[0.0] * n for _ in range(3)]
    pb = p.tolist()
    for t in range(4):
        g = rng.standard_normal((m, n)) * 1e-2
        info = {}
        p = O.tensor_step(p, g, st, theta, C, t, 0.9, 0.05, out=info)
        pb, s = _brute_force_step(pb, g.tolist(), M, V, r, c, theta, C, O.KIND_SMALL_FC, t, 0.9, 0.05)
        np.testing.assert_allclose(info["stats"], s, rtol=1e-11)
        np.testing.assert_allclose(p, np.array(pb), rtol=1e-10, atol=1e-16)
    np.testing.assert_allclose(st["M"], np.array(M), rtol=1e-12)
    np.testing.assert_allclose(st["V"], np.array(V), rtol=1e-12)
    np.testing.assert_allclose(st["r"], np.array(r), rtol=1e-12)
    np.testing.assert_allclose(st["c"], np.array(c), rtol=1e-12)


def test_velo_mlp_part_4x3_against_scalar_brute_force():
    # the per-element part of VeLO with the hypernetwork's output taken as given
    C = cfg(O.KIND_VELO, hidden=2, lstm_hidden=3, n_bank=2)
    rng = np.random.default_rng(15)
    m, n = 4, 3
    n_theta = 29 * 2 + 2 + 4 + 2 + 4 + 2
    weights = rng.uniform(-0.7, 0.7, velo_size(2, 3, 2))
    p = rng.standard_normal((m, n)) * 0.05
    st = O.init_state(m, n, C)
    M = [[[0.0] * n for _ in range(m)] for _ in range(3)]
    V = [[0.0] * n for _ in range(m)]
    r = [[0.0] * m for _ in range(3)]
    c = [[0.0] * n for _ in range(3)]
    for t in range(3):
        g = rng.standard_normal((m, n)) * 0.2          # exercises the clip
        info = {}
        p_prev = p.tolist()
        p = O.tensor_step(p, g, st, weights, C, t, 0.9, 0.05, ndim=2, out=info)
        pb, s = _brute_force_step(p_prev, g.tolist(), M, V, r, c, info["theta"], C, O.KIND_VELO, t, 0.9, 0.05,
                                  lam=info["lam"])
        np.testing.assert_allclose(info["stats"], s, rtol=1e-11)
        np.testing.assert_allclose(p, np.array(pb), rtol=1e-10, atol=1e-16)


# ------------------------------------------------------------------ VeLO hypernetwork

def test_lstm_cell_matches_torch_lstmcell():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(16)
    n_in, HL = 45, 7
    Wx = rng.standard_normal((n_in, 4 * HL)) * 0.3
    Wh = rng.standard_normal((HL, 4 * HL)) * 0.3
    b = rng.standard_normal(4 * HL) * 0.3
    u = rng.standard_normal(n_in)
    h = rng.standard_normal(HL)
    c = rng.standard_normal(HL)
    cell = torch.nn.LSTMCell(n_in, HL).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(Wx.T.copy()))
        cell.weight_hh.copy_(torch.from_numpy(Wh.T.copy()))
        cell.bias_ih.copy_(torch.from_numpy(b))
        cell.bias_hh.zero_()
        h1, c1 = cell(torch.from_numpy(u)[None], (torch.from_numpy(h)[None], torch.from_numpy(c)[None]))
    h2, c2 = O.lstm_cell(u, h, c, Wx, Wh, b)
    np.testing.assert_allclose(h2, h1[0].numpy(), rtol=1e-12)
    np.testing.assert_allclose(c2, c1[0].numpy(), rtol=1e-12)


def _split_velo(weights, H, HL, K):
    n_theta = 29 * H + H + H * H + H + 2 * H + 2
    o = 0
    out = []
    for shape in ((48, 4 * HL), (HL, 4 * HL), (HL, 4 * HL), (4 * HL,), (HL, K), (K,), (HL,), (1,), (K, n_theta)):
        n = int(np.prod(shape))
        out.append(weights[o:o + n].reshape(shape))
        o += n
    assert o == weights.size
    return out


def test_velo_hypernetwork_brute_force_and_state_carry():
    # scalar loops over the whole hypernetwork: input assembly (statistics, time, rank one-hot, loss), LSTM cell with
    # the cross-tensor input term, bank mixing, step-size output; the state carries from call to call
    C = cfg(O.KIND_VELO, hidden=2, lstm_hidden=3, n_bank=2)
    rng = np.random.default_rng(17)
    n_theta = 29 * 2 + 2 + 4 + 2 + 4 + 2
    weights = rng.uniform(-0.7, 0.7, velo_size(2, 3, 2))
    Wx, Wh, Wg, b, Wa, ba, ws, bs, B = _split_velo(weights, 2, 3, 2)
    st = O.init_state(2, 2, C)
    h = [0.0] * 3
    cl = [0.0] * 3
    sg = lambda x: 1 / (1 + math.exp(-x))
    for t, ndim, loss in [(0, 1, 2.5), (5, 2, 0.0), (9, 4, -0.75), (12, 7, 1e4)]:
        s = rng.uniform(1e-9, 10.0, 29)
        hm = rng.uniform(-1, 1, 3)
        theta, lam = O.velo_hypernetwork(s, t, ndim, st, weights, C, loss=loss, h_mix=hm)
        u = [0.05 * math.log(v + float(np.float32(1e-30))) for v in s]
        u += [math.tanh(t / x) for x in O.TIME_SCALES]
        u += [1.0 if q == min(ndim, 4) else 0.0 for q in range(5)]
        psi = math.copysign(math.log(1.0 + abs(loss)), loss) if loss != 0 else 0.0
        u += [math.tanh(psi / x) for x in (1.0, 3.0, 10.0)]
        assert len(u) == 48
        z = [b[q] + sum(u[a] * Wx[a][q] for a in range(48)) + sum(h[a] * Wh[a][q] for a in range(3))
             + sum(hm[a] * Wg[a][q] for a in range(3)) for q in range(12)]
        cl = [sg(z[3 + q]) * cl[q] + sg(z[q]) * math.tanh(z[6 + q]) for q in range(3)]
        h = [sg(z[9 + q]) * math.tanh(cl[q]) for q in range(3)]
        alpha = [ba[q] + sum(h[a] * Wa[a][q] for a in range(3)) for q in range(2)]
        expect = [sum(alpha[q] * B[q][w] for q in range(2)) for w in range(n_theta)]
        np.testing.assert_allclose(theta, expect, rtol=1e-11)
        np.testing.assert_allclose(st["h"], h, rtol=1e-12)
        assert lam == pytest.approx(math.exp(bs[0] + sum(h[a] * ws[a] for a in range(3))), rel=1e-12)


def test_loss_features_closed_forms():
    # zero loss (or no loss given) contributes nothing; psi = ln(1 + loss) = 1 at loss = e - 1; odd; bounded; monotone
    assert np.all(O.loss_features(0.0) == 0.0)
    np.testing.assert_allclose(O.loss_features(math.e - 1.0), [math.tanh(1.0), math.tanh(1 / 3), math.tanh(0.1)], rtol=1e-13)
    np.testing.assert_allclose(O.loss_features(-3.7), -O.loss_features(3.7), rtol=0, atol=0)
    big = O.loss_features(1e30)
    assert np.all(big <= 1.0) and big[0] == pytest.approx(1.0) and big[2] == pytest.approx(math.tanh(math.log(1e30) / 10), rel=1e-12)
    xs = np.array([-50.0, -1.0, -1e-3, 0.0, 1e-3, 0.2, 3.0, 700.0])
    f = np.stack([O.loss_features(x) for x in xs])
    assert np.all(np.diff(f, axis=0) > 0)
    assert len(O.LOSS_SCALES) == 3 and O.velo_input_size() == 48


def _velo_list_case(seed, Wg_zero=False, loss_rows_zero=False):
    C = cfg(O.KIND_VELO, hidden=3, lstm_hidden=4, n_bank=2)
    rng = np.random.default_rng(seed)
    w = rng.uniform(-0.6, 0.6, velo_size(3, 4, 2))
    if Wg_zero:
        o = 48 * 16 + 4 * 16
        w[o:o + 4 * 16] = 0.0
    if loss_rows_zero:
        w[45 * 16:48 * 16] = 0.0
    shapes = [(3, 4), (1, 5), (6, 2)]
    ps = [rng.standard_normal(sh) * 0.03 for sh in shapes]
    gss = [[rng.standard_normal(sh) * 0.01 for sh in shapes] for _ in range(3)]
    return C, w, shapes, ps, gss


def _run_list(C, w, shapes, ps, gss, order=None, losses=(0.3, 1.7, 0.9)):
    order = list(range(len(shapes))) if order is None else order
    ps = [ps[i].copy() for i in order]
    sts = [O.init_state(*shapes[i], C) for i in order]
    for t, gs in enumerate(gss):
        ps = O.list_step(ps, [gs[i] for i in order], sts, w, C, t, 0.8, 0.01, [[2, 1, 2][i] for i in order],
                         loss=losses[t])
    return ps, sts


def test_cross_tensor_term_is_the_mean_of_previous_outputs_over_the_list():
    C, w, shapes, ps, gss = _velo_list_case(31)
    # brute force of the mean, step by step: every tensor's LSTM sees the same vector, taken BEFORE any state moves
    sts = [O.init_state(*sh, C) for sh in shapes]
    cur = [p.copy() for p in ps]
    for t, gs in enumerate(gss):
        hbar = [sum(float(st["h"][j]) for st in sts) / len(sts) for j in range(4)]
        np.testing.assert_allclose(O.mean_hidden([st["h"] for st in sts]), hbar, rtol=1e-14, atol=0)
        if t == 0:
            assert hbar == [0.0] * 4
        ref_sts = [{k: v.copy() for k, v in st.items()} for st in sts]
        ref = [O.tensor_step(cur[i], gs[i], ref_sts[i], w, C, t, 0.8, 0.01, ndim=[2, 1, 2][i], loss=0.4, h_mix=hbar)
               for i in range(3)]
        cur = O.list_step(cur, gs, sts, w, C, t, 0.8, 0.01, [2, 1, 2], loss=0.4)
        for a, b_ in zip(cur, ref):
            np.testing.assert_allclose(a, b_, rtol=1e-13)
        for a, b_ in zip(sts, ref_sts):
            np.testing.assert_allclose(a["h"], b_["h"], rtol=1e-13)


def test_cross_tensor_term_order_invariance_and_decoupling():
    C, w, shapes, ps, gss = _velo_list_case(32)
    base, _ = _run_list(C, w, shapes, ps, gss)
    # the order of the list does not matter (a mean), each tensor's own result does not move with its position
    perm, _ = _run_list(C, w, shapes, ps, gss, order=[2, 0, 1])
    for k, i in enumerate([2, 0, 1]):
        np.testing.assert_allclose(perm[k], base[i], rtol=1e-12)
    # with non-zero mixing weights the tensors are coupled: a tensor stepped alone ends elsewhere ...
    alone = []
    for i in range(3):
        st = O.init_state(*shapes[i], C)
        p = ps[i].copy()
        for t, gs in enumerate(gss):
            p = O.tensor_step(p, gs[i], st, w, C, t, 0.8, 0.01, ndim=[2, 1, 2][i], loss=(0.3, 1.7, 0.9)[t])
        alone.append(p)
    assert max(np.abs(a - b_).max() for a, b_ in zip(alone, base)) > 1e-6
    # ... and with zero mixing weights exactly where the list run ends (the term is the only coupling)
    C0, w0, _, _, _ = _velo_list_case(32, Wg_zero=True)
    base0, _ = _run_list(C0, w0, shapes, ps, gss)
    for i in range(3):
        st = O.init_state(*shapes[i], C0)
        p = ps[i].copy()
        for t, gs in enumerate(gss):
            p = O.tensor_step(p, gs[i], st, w0, C0, t, 0.8, 0.01, ndim=[2, 1, 2][i], loss=(0.3, 1.7, 0.9)[t])
        np.testing.assert_allclose(p, base0[i], rtol=1e-13)


def test_cross_tensor_term_is_an_extra_lstm_input_like_torch_lstmcell():
    # h_mix @ Wg enters the gates like any other input: LSTMCell on [u | h_mix] with [Wx ; Wg] gives the same state
    torch = pytest.importorskip("torch")
    C = cfg(O.KIND_VELO, hidden=2, lstm_hidden=5, n_bank=2)
    rng = np.random.default_rng(33)
    w = rng.uniform(-0.5, 0.5, velo_size(2, 5, 2))
    Wx, Wh, Wg, b, Wa, ba, ws, bs, B = _split_velo(w, 2, 5, 2)
    st = O.init_state(2, 2, C)
    st["h"] = rng.uniform(-1, 1, 5)
    st["cl"] = rng.uniform(-1, 1, 5)
    h0, c0 = st["h"].copy(), st["cl"].copy()
    s = rng.uniform(1e-6, 3.0, 29)
    hm = rng.uniform(-1, 1, 5)
    O.velo_hypernetwork(s, 7, 2, st, w, C, loss=1.25, h_mix=hm)
    onehot = np.zeros(5); onehot[2] = 1.0
    u = np.concatenate([0.05 * np.log(s + float(np.float32(1e-30))), np.tanh(7.0 / np.array(O.TIME_SCALES)), onehot,
                        np.tanh(math.log(2.25) / np.array([1.0, 3.0, 10.0])), hm])
    cell = torch.nn.LSTMCell(53, 5).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.from_numpy(np.concatenate([Wx, Wg]).T.copy()))
        cell.weight_hh.copy_(torch.from_numpy(Wh.T.copy()))
        cell.bias_ih.copy_(torch.from_numpy(b))
        cell.bias_hh.zero_()
        h1, c1 = cell(torch.from_numpy(u)[None], (torch.from_numpy(h0)[None], torch.from_numpy(c0)[None]))
    np.testing.assert_allclose(st["h"], h1[0].numpy(), rtol=1e-12)
    np.testing.assert_allclose(st["cl"], c1[0].numpy(), rtol=1e-12)


def test_loss_reaches_the_update_only_through_its_input_weights():
    C, w, shapes, ps, gss = _velo_list_case(34)
    a, _ = _run_list(C, w, shapes, ps, gss, losses=(0.3, 1.7, 0.9))
    b_, _ = _run_list(C, w, shapes, ps, gss, losses=(5.0, 0.01, 40.0))
    assert max(np.abs(x - y).max() for x, y in zip(a, b_)) > 1e-7        # the loss matters ...
    C0, w0, _, _, _ = _velo_list_case(34, loss_rows_zero=True)
    a0, _ = _run_list(C0, w0, shapes, ps, gss, losses=(0.3, 1.7, 0.9))
    b0, _ = _run_list(C0, w0, shapes, ps, gss, losses=(5.0, 0.01, 40.0))
    for x, y in zip(a0, b0):                                              # ... through rows 45..47 of Wx and nothing else
        assert np.array_equal(x, y)


def test_step_size_output_scales_the_update_and_nothing_else():
    # w_s = 0: lam = exp(b_s) for every tensor and step. b_s = ln 2 doubles the update p_old - p_new (no weight decay);
    # with weight decay only the learned part doubles.
    C = cfg(O.KIND_VELO, hidden=3, lstm_hidden=4, n_bank=2)
    rng = np.random.default_rng(35)
    w = rng.uniform(-0.6, 0.6, velo_size(3, 4, 2))
    o_ws = 48 * 16 + 2 * 4 * 16 + 16 + 4 * 2 + 2
    w[o_ws:o_ws + 4] = 0.0
    p = rng.standard_normal((5, 4)) * 0.03
    g = rng.standard_normal((5, 4)) * 0.01
    res = {}
    for bs, wd in ((0.0, 0.0), (math.log(2.0), 0.0), (0.0, 0.1), (math.log(2.0), 0.1)):
        w[o_ws + 4] = bs
        info = {}
        res[(bs > 0, wd)] = O.tensor_step(p, g, O.init_state(5, 4, C), w, C, 3, 0.7, wd, out=info)
        assert info["lam"] == pytest.approx(math.exp(bs), rel=1e-14)
    d1, d2 = p - res[(False, 0.0)], p - res[(True, 0.0)]
    np.testing.assert_allclose(d2, 2.0 * d1, rtol=1e-12)
    e1, e2 = p - res[(False, 0.1)], p - res[(True, 0.1)]
    np.testing.assert_allclose(e1 - d1, 0.7 * 0.1 * p, rtol=1e-9, atol=1e-18)   # decay term: lr * wd * p, not scaled by lam
    np.testing.assert_allclose(e2 - d2, 0.7 * 0.1 * p, rtol=1e-9, atol=1e-18)


# ------------------------------------------------------------------ chunked evaluation

@pytest.mark.parametrize("kind", [O.KIND_SMALL_FC, O.KIND_VELO])
def test_row_slab_evaluation_equals_whole_tensor(kind):
    C = cfg(kind, hidden=4, lstm_hidden=5, n_bank=3)
    rng = np.random.default_rng(18)
    m, n = 13, 9
    if kind == O.KIND_SMALL_FC:
        w = rng.standard_normal(39 * 4 + 4 + 16 + 4 + 8 + 2) * 0.3
    else:
        n_theta = 29 * 4 + 4 + 16 + 4 + 8 + 2
        w = rng.standard_normal(velo_size(4, 5, 3)) * 0.3
    p0 = rng.standard_normal((m, n)) * 0.02
    gs = [rng.standard_normal((m, n)) * 1e-2 for _ in range(3)]
    res = []
    for chunk in (1 << 19, 20):
        p = p0.copy()
        st = O.init_state(m, n, C)
        for t, g in enumerate(gs):
            p = O.tensor_step(p, g, st, w, C, t, 1.0, 0.0, max_chunk_elems=chunk)
        res.append(p)
    np.testing.assert_allclose(res[0], res[1], rtol=1e-11, atol=1e-16)


def test_rel_err_metric():
    b = np.array([1.0, -1.0, 0.0, 2.0])
    a = b + np.array([0.0, 0.0, 1e-3, 0.0])
    rms = math.sqrt(6 / 4)
    assert O.rel_err(a, b) == pytest.approx(1e-3 / rms)
    assert O.rel_err(b, b) == 0.0


def test_apply_rows_equals_the_same_rows_of_a_full_step():
    C = cfg(hidden=4)
    rng = np.random.default_rng(19)
    m, n = 11, 6
    w = rng.standard_normal(39 * 4 + 4 + 16 + 4 + 8 + 2) * 0.3
    p = rng.standard_normal((m, n)) * 0.02
    g = rng.standard_normal((m, n)) * 1e-2
    st = O.init_state(m, n, C)
    info = {}
    full = O.tensor_step(p, g, st, w, C, 2, 0.8, 0.02, out=info)
    part = O.apply_rows(p, g, st, info["stats"], w, C, 2, 0.8, 0.02, slice(3, 7))
    np.testing.assert_allclose(part, full[3:7], rtol=1e-13)
