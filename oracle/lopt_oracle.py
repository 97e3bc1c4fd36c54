"""CPU oracle for the learned-optimizer step (small_fc_lopt and VeLO).

TEST INFRASTRUCTURE ONLY. This is a plain, slow float64 NumPy implementation of
the *naive* pipeline the paper describes (section "Analysis of Naive
Implementation" and the figure "Overview of the Learned Optimizer update
mechanism"): accumulator update -> construct_features() -> compute_squared_average()
-> feature_normalization() -> apply_lo() -> parameter update. It shares no code
with the HIP path and must never be imported by the product package.

Notation follows the paper's feature tables (appendix "Features for learned
optimizer input"): tensor W in R^{m x n}, gradient g, momentum accumulators
M_1..M_3 (decays beta_1..3), second moment V (beta_4), Adafactor row/column
accumulators r_k in R^m, c_k in R^n (beta_5..7), t = step index.

Readings taken where the paper is silent (each is a documented choice):
  * the ten accumulators are themselves MLP inputs (3 M, V, 3 r, 3 c), which is
    what makes the feature tables' totals 39 (small_fc_lopt) and 29 (VeLO);
  * only per-element features are normalized; the 11 time features tanh(t/x)
    are appended un-normalized;
  * r_k = mean over columns (one value per row), c_k = mean over rows;
  * eps_acc sits inside every reciprocal square root of an accumulator, eps_norm
    inside the normalization square root;
  * the update is subtracted (pseudocode of Kernel 2), lr multiplies it, and
    weight decay is decoupled: p <- p - lr * (delta + wd * p_old);
  * 1-D tensors are 1 x n matrices.
  * the VeLO per-tensor LSTM hypernetwork is not described by the paper at all;
    `velo_hypernetwork` below is this project's definition of it. What the paper
    does fix is that VeLO's step takes the current loss value (artifact appendix,
    "Basic Usage"): the loss enters the hypernetwork's input through
    `loss_features`. The definition also has a cross-tensor term (the mean of the
    tensors' previous LSTM outputs is an input of every tensor's LSTM) and a
    per-tensor step-size output.
    Fidelity of that part to the original VeLO: PARITY UNPINNED (no weights, no
    worked example); it is pinned only against torch.nn.LSTMCell, closed forms
    and brute force.
  * End-to-end agreement with the paper's released optimizers: PARITY UNPINNED
    (the paper prints no worked numeric example).

For memory, features are built for a slab of rows at a time when a tensor is
larger than `max_chunk_elems`; the arithmetic per element and the order of the
pipeline stages are unchanged (statistics over the whole tensor are finished
before any feature is normalized). Small tensors are processed as one slab,
i.e. exactly the naive [mn x d_feat] materialisation.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import numpy as np

F64 = np.float64

# Time-feature scales: feature table, row "Time Features".
TIME_SCALES = (1.0, 3.0, 10.0, 30.0, 100.0, 300.0, 1000.0, 3000.0, 1e4, 3e4, 1e5)
# Clip bound of VeLO's clipped-gradient feature: VeLO feature table, row "Clipped gradient value".
GRAD_CLIP = 0.1
# Scales of the loss features tanh(psi(loss)/x) (project-defined, see loss_features).
LOSS_SCALES = (1.0, 3.0, 10.0)
N_ELEM = 28           # per-element features shared by both optimizers
KIND_SMALL_FC = "small_fc_lopt"
KIND_VELO = "velo"


def _f32(x) -> float:
    """Scalars cross the C boundary as float32; the oracle takes the same value."""
    return float(np.float32(x))


@dataclass
class OracleConfig:
    kind: str = KIND_SMALL_FC
    hidden: int = 32                                   # MLP width (benchmarking section: 32)
    mom_decay: Sequence[float] = (_f32(0.9), _f32(0.99), _f32(0.999))      # beta_1..3
    rms_decay: float = _f32(0.999)                                        # beta_4
    fac_decay: Sequence[float] = (_f32(0.9), _f32(0.99), _f32(0.999))      # beta_5..7
    eps_acc: float = _f32(1e-16)
    eps_norm: float = _f32(1e-30)
    exp_mult: float = _f32(0.01)                       # alpha, section "Apply Learned Optimizer"
    step_mult: float = _f32(0.01)                      # beta, same place
    lstm_hidden: int = 512
    n_bank: int = 256

    @property
    def d_feat(self) -> int:
        return N_ELEM + (len(TIME_SCALES) if self.kind == KIND_SMALL_FC else 1)

    @property
    def n_normalized(self) -> int:
        """Number of leading features that get normalized."""
        return N_ELEM if self.kind == KIND_SMALL_FC else N_ELEM + 1


# --------------------------------------------------------------------------- state

def init_state(rows: int, cols: int, cfg: OracleConfig) -> Dict[str, np.ndarray]:
    """Zero accumulators (no bias correction anywhere in the feature tables)."""
    st = {
        "M": np.zeros((3, rows, cols), F64),
        "V": np.zeros((rows, cols), F64),
        "r": np.zeros((3, rows), F64),
        "c": np.zeros((3, cols), F64),
    }
    if cfg.kind == KIND_VELO:
        st["h"] = np.zeros(cfg.lstm_hidden, F64)
        st["cl"] = np.zeros(cfg.lstm_hidden, F64)
    return st


# --------------------------------------------------------------------------- accumulators

def update_accumulators(st: Dict[str, np.ndarray], g: np.ndarray, cfg: OracleConfig) -> None:
    """Feature tables, block "Accumulators" (identical for both optimizers)."""
    g = np.asarray(g, F64)
    g2 = g * g
    for i in range(3):
        b = cfg.mom_decay[i]
        st["M"][i] = b * st["M"][i] + (1.0 - b) * g
    b4 = cfg.rms_decay
    st["V"] = b4 * st["V"] + (1.0 - b4) * g2
    row_mean = g2.mean(axis=1)        # one value per row i
    col_mean = g2.mean(axis=0)        # one value per column j
    for k in range(3):
        b = cfg.fac_decay[k]
        st["r"][k] = b * st["r"][k] + (1.0 - b) * row_mean
        st["c"][k] = b * st["c"][k] + (1.0 - b) * col_mean


# --------------------------------------------------------------------------- features

def time_features(t: int) -> np.ndarray:
    return np.tanh(F64(t) / np.asarray(TIME_SCALES, F64))


def construct_features(p, g, st, cfg: OracleConfig, t: int, rows: slice = slice(None)) -> np.ndarray:
    """construct_features(): the [mn x d_feat] matrix for the given slab of rows.

    Column order (fixed by this project; the paper lists the features, not an order):
      0 g | 1 p | 2-4 M_1..3 | 5 V | 6-8 M_i/sqrt(V) | 9 1/sqrt(V) |
      10-12 g*sqrt(mean(r_k)/(r_k c_k^T)) | 13-15 r_k | 16-18 c_k |
      19-21 1/sqrt(r_k) | 22-24 1/sqrt(c_k) | 25-27 M_k*sqrt(mean(r_k)/(r_k c_k^T)) |
      small_fc_lopt: 28-38 tanh(t/x);  VeLO: 28 clip(g, -0.1, 0.1)
    """
    e = cfg.eps_acc
    p = np.asarray(p, F64)[rows]
    g = np.asarray(g, F64)[rows]
    M = st["M"][:, rows]
    V = st["V"][rows]
    r = st["r"]
    c = st["c"]
    mr, n = g.shape
    F = np.empty((mr, n, cfg.d_feat), F64)
    F[..., 0] = g
    F[..., 1] = p
    rs = 1.0 / np.sqrt(V + e)
    for i in range(3):
        F[..., 2 + i] = M[i]
        F[..., 6 + i] = M[i] * rs
    F[..., 5] = V
    F[..., 9] = rs
    for k in range(3):
        rbar = r[k].mean()                                    # (1/m) sum_h r_h, all rows
        a = np.sqrt(rbar + e) / np.sqrt(r[k, rows] + e)       # per row
        b = 1.0 / np.sqrt(c[k] + e)                           # per column
        fac = a[:, None] * b[None, :]
        F[..., 10 + k] = g * fac
        F[..., 13 + k] = r[k, rows][:, None]
        F[..., 16 + k] = c[k][None, :]
        F[..., 19 + k] = (1.0 / np.sqrt(r[k, rows] + e))[:, None]
        F[..., 22 + k] = b[None, :]
        F[..., 25 + k] = M[k] * fac
    if cfg.kind == KIND_SMALL_FC:
        F[..., 28:39] = time_features(t)
    else:
        F[..., 28] = np.clip(g, -GRAD_CLIP, GRAD_CLIP)
    return F.reshape(mr * n, cfg.d_feat)


def compute_squared_average(F: np.ndarray) -> np.ndarray:
    """compute_squared_average(): E[feature^2] over the rows of F."""
    return (F * F).mean(axis=0)


def feature_normalization(F: np.ndarray, s: np.ndarray, cfg: OracleConfig) -> np.ndarray:
    """feature_normalization(): feature / sqrt(E[feature^2] + eps) on the normalized columns."""
    out = F.copy()
    k = cfg.n_normalized
    out[:, :k] = F[:, :k] / np.sqrt(s[:k] + cfg.eps_norm)
    return out


# --------------------------------------------------------------------------- MLP

def unpack_mlp(theta: np.ndarray, d_in: int, hidden: int):
    """theta = W1[d,H] | b1[H] | W2[H,H] | b2[H] | W3[H,2] | b3[2], row-major."""
    theta = np.asarray(theta, F64).ravel()
    o = 0

    def take(*shape):
        nonlocal o
        n = int(np.prod(shape))
        v = theta[o:o + n].reshape(shape)
        o += n
        return v

    W1 = take(d_in, hidden); b1 = take(hidden)
    W2 = take(hidden, hidden); b2 = take(hidden)
    W3 = take(hidden, 2); b3 = take(2)
    assert o == theta.size, (o, theta.size)
    return W1, b1, W2, b2, W3, b3


def apply_lo(Fn: np.ndarray, theta: np.ndarray, cfg: OracleConfig):
    """apply_lo(): three linear layers with two ReLUs (pseudocode of Kernel 2);
    output 0 is the direction, output 1 the magnitude."""
    W1, b1, W2, b2, W3, b3 = unpack_mlp(theta, cfg.d_feat, cfg.hidden)
    h = np.maximum(Fn @ W1 + b1, 0.0)
    h = np.maximum(h @ W2 + b2, 0.0)
    out = h @ W3 + b3
    return out[:, 0], out[:, 1]


def delta_theta(direction, magnitude, cfg: OracleConfig):
    """delta = direction * exp(magnitude * alpha) * beta (section "Apply Learned Optimizer")."""
    return direction * np.exp(magnitude * cfg.exp_mult) * cfg.step_mult


# --------------------------------------------------------------------------- VeLO hypernetwork

def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def velo_input_size() -> int:
    """29 log-statistics + 11 time features + one-hot(min(ndim, 4)) + 3 loss features."""
    return (N_ELEM + 1) + len(TIME_SCALES) + 5 + len(LOSS_SCALES)


def unpack_velo(weights: np.ndarray, cfg: OracleConfig):
    """weights = Wx[48,4HL] | Wh[HL,4HL] | Wg[HL,4HL] | b[4HL] | Wa[HL,K] | ba[K] | ws[HL] | bs[1] | B[K,P]."""
    w = np.asarray(weights, F64).ravel()
    HL, K, H = cfg.lstm_hidden, cfg.n_bank, cfg.hidden
    n_in = velo_input_size()
    n_theta = (N_ELEM + 1) * H + H + H * H + H + 2 * H + 2
    o = 0

    def take(*shape):
        nonlocal o
        n = int(np.prod(shape))
        v = w[o:o + n].reshape(shape)
        o += n
        return v

    Wx = take(n_in, 4 * HL); Wh = take(HL, 4 * HL); Wg = take(HL, 4 * HL); b = take(4 * HL)
    Wa = take(HL, K); ba = take(K); ws = take(HL); bs = take(1); B = take(K, n_theta)
    assert o == w.size, (o, w.size)
    return Wx, Wh, Wg, b, Wa, ba, ws, bs, B


def lstm_cell(u, h, c, Wx, Wh, b):
    """One standard LSTM-cell step, gate order i, f, g, o."""
    HL = h.shape[0]
    z = u @ Wx + h @ Wh + b
    i, f, g, o = z[:HL], z[HL:2 * HL], z[2 * HL:3 * HL], z[3 * HL:]
    c_new = _sigmoid(f) * c + _sigmoid(i) * np.tanh(g)
    h_new = _sigmoid(o) * np.tanh(c_new)
    return h_new, c_new


def loss_features(loss: float) -> np.ndarray:
    """The loss value handed to VeLO's step (artifact appendix, "Basic Usage") as hypernetwork inputs:
    tanh(psi / x) for x in LOSS_SCALES with psi = sign(loss) * ln(1 + |loss|). Bounded, odd in the loss,
    zero for a loss of zero (which is also what a step without a loss value means)."""
    psi = np.sign(F64(loss)) * np.log1p(abs(F64(loss)))
    return np.tanh(psi / np.asarray(LOSS_SCALES, F64))


def mean_hidden(hs) -> np.ndarray:
    """Cross-tensor term: mean over the tensors of the step's list of their LSTM outputs h from the
    previous step (zeros before the first step)."""
    hs = [np.asarray(h, F64) for h in hs]
    return np.sum(hs, axis=0) / len(hs)


def velo_hypernetwork(s: np.ndarray, t: int, ndim: int, st, weights, cfg: OracleConfig,
                      loss: float = 0.0, h_mix=None):
    """Per-tensor MLP weights and step-size multiplier for this step (project-defined; see module header).

    input u = [0.05*ln(s_f + 1e-30) for the 29 statistics] ++ [11 time features]
              ++ one_hot(min(ndim, 4), 5) ++ loss_features(loss);
    (h, c) <- LSTMCell(u, (h, c)) with the extra input term h_mix @ Wg, h_mix = mean_hidden over the list
    (None: a list of this tensor alone, so h_mix is its own previous h);
    alpha = h W_a + b_a; theta = alpha @ B; lam = exp(h . w_s + b_s).
    Returns (theta, lam)."""
    Wx, Wh, Wg, b, Wa, ba, ws, bs, B = unpack_velo(weights, cfg)
    onehot = np.zeros(5, F64)
    onehot[min(int(ndim), 4)] = 1.0
    u = np.concatenate([0.05 * np.log(s[:N_ELEM + 1] + _f32(1e-30)), time_features(t), onehot, loss_features(loss)])
    hm = st["h"] if h_mix is None else np.asarray(h_mix, F64)
    h, c = lstm_cell(u, st["h"], st["cl"], Wx, Wh, b + hm @ Wg)
    st["h"], st["cl"] = h, c
    alpha = h @ Wa + ba
    lam = float(np.exp(h @ ws + bs[0]))
    return alpha @ B, lam


# --------------------------------------------------------------------------- one step of one tensor

def tensor_statistics(p, g, st, cfg: OracleConfig, t: int, max_chunk_elems: int = 1 << 19) -> np.ndarray:
    m, n = np.shape(g)
    rows_per = max(1, max_chunk_elems // max(n, 1))
    acc = np.zeros(cfg.d_feat, F64)
    for r0 in range(0, m, rows_per):
        F = construct_features(p, g, st, cfg, t, slice(r0, min(m, r0 + rows_per)))
        acc += (F * F).sum(axis=0)
    return acc / (m * n)


def tensor_step(p, g, st, weights, cfg: OracleConfig, t: int, lr: float, wd: float,
                ndim: int = 2, max_chunk_elems: int = 1 << 19, out: Optional[dict] = None,
                loss: float = 0.0, h_mix=None) -> np.ndarray:
    """One optimizer step of one tensor; returns the new parameters (float64) and
    updates `st` in place. `out`, if given, receives intermediate results. VeLO: `loss` is the loss value
    passed to the step, `h_mix` the mean_hidden of the step's tensor list (None: this tensor alone)."""
    p = np.asarray(p, F64)
    g = np.asarray(g, F64)
    m, n = g.shape
    update_accumulators(st, g, cfg)
    if m * n <= max_chunk_elems:
        F = construct_features(p, g, st, cfg, t)
        s = compute_squared_average(F)
    else:
        F = None
        s = tensor_statistics(p, g, st, cfg, t, max_chunk_elems)
    if cfg.kind == KIND_SMALL_FC:
        theta, lam = weights, 1.0
    else:
        theta, lam = velo_hypernetwork(s, t, ndim, st, weights, cfg, loss, h_mix)
    if out is not None:
        out["stats"] = s.copy()
        out["theta"] = np.array(theta, F64)
        out["lam"] = lam
    p_new = np.empty_like(p)
    rows_per = m if F is not None else max(1, max_chunk_elems // max(n, 1))
    for r0 in range(0, m, rows_per):
        sl = slice(r0, min(m, r0 + rows_per))
        Fc = F if F is not None else construct_features(p, g, st, cfg, t, sl)
        Fn = feature_normalization(Fc, s, cfg)
        direction, magnitude = apply_lo(Fn, theta, cfg)
        delta = lam * delta_theta(direction, magnitude, cfg).reshape(-1, n)
        p_new[sl] = p[sl] - lr * (delta + wd * p[sl])
    return p_new


def list_step(ps, gs, sts, weights, cfg: OracleConfig, t: int, lr: float, wd: float, ndims,
              loss: float = 0.0, outs=None):
    """One optimizer step over a list of tensors (what one call of the optimizer's step covers): for VeLO the
    cross-tensor term is taken over this list, before any tensor's LSTM state moves."""
    h_mix = mean_hidden([st["h"] for st in sts]) if cfg.kind == KIND_VELO and len(sts) else None
    return [tensor_step(ps[i], gs[i], sts[i], weights, cfg, t, lr, wd, ndim=ndims[i],
                        out=None if outs is None else outs[i], loss=loss, h_mix=h_mix)
            for i in range(len(ps))]


def apply_rows(p, g, st, s, theta, cfg: OracleConfig, t: int, lr: float, wd: float, rows: slice,
               lam: float = 1.0) -> np.ndarray:
    """New parameters of a slab of rows only, given the whole tensor's statistics `s`, the MLP
    weights `theta` and the step-size multiplier `lam` (accumulators in `st` already updated): the
    second half of tensor_step, for spot checks on tensors too large to evaluate in full."""
    p = np.asarray(p, F64)
    n = p.shape[1]
    Fc = construct_features(p, g, st, cfg, t, rows)
    Fn = feature_normalization(Fc, s, cfg)
    direction, magnitude = apply_lo(Fn, theta, cfg)
    delta = lam * delta_theta(direction, magnitude, cfg).reshape(-1, n)
    return p[rows] - lr * (delta + wd * p[rows])


def rel_err(a, b) -> float:
    """max_i |a_i - b_i| / (|b_i| + rms(b)): the error metric of the parity tests."""
    a = np.asarray(a, F64).ravel()
    b = np.asarray(b, F64).ravel()
    if b.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(b * b)))
    den = np.abs(b) + rms
    den[den == 0.0] = 1.0
    return float(np.max(np.abs(a - b) / den))
