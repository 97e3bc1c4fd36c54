"""Seeded synthetic workloads: parameter-set shapes and input generators.

This module serves both the CPU oracle's tests and the HIP path's tests/bench.
It holds no arithmetic of the optimizer itself: only shapes of the model
families the paper times (ViT-B/16, GPT-2 medium: timing tables of the
benchmarking section and the full-timing appendix table), a Llama-style 1.3B
set, and seeded random draws for parameters, gradients and optimizer weights.

Every array is float32 and is regenerated from (config, tensor, step) alone,
so a single tensor's stream can be produced without touching the others.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

BASE_SEED = 20250610

# stream ids inside a (config, tensor) seed
_STREAM_PARAM = 1
_STREAM_GRAD = 2
_STREAM_SCALE = 3
_STREAM_WEIGHTS = 4
_STREAM_TINY = 5


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: Tuple[int, ...]

    @property
    def numel(self) -> int:
        return int(np.prod(self.shape, dtype=np.int64))

    @property
    def ndim(self) -> int:
        return len(self.shape)

    def as_2d(self) -> Tuple[int, int, int]:
        """(ndim, rows, cols) as the C boundary wants it: leading size-1 dims
        squeezed, 1-D -> 1 x n, ndim > 2 -> (dim0, product of the rest)."""
        shp = list(self.shape)
        while len(shp) > 1 and shp[0] == 1:
            shp = shp[1:]
        if len(shp) == 1:
            return (1, 1, int(shp[0]))
        rows = int(shp[0])
        cols = int(np.prod(shp[1:], dtype=np.int64))
        return (len(shp), rows, cols)


@dataclass
class Workload:
    config_id: int
    name: str
    optimizer: str            # "small_fc_lopt" | "velo"
    tensors: List[TensorSpec]
    steps: int
    grad_kind: str            # "gauss_fixed" | "gauss_logscale" | "student_t3"
    lr: float = 1.0
    lr_schedule: str = "constant"   # "constant" | "cosine"
    weight_decay: float = 0.0
    notes: str = ""

    @property
    def numel(self) -> int:
        return sum(t.numel for t in self.tensors)


# --------------------------------------------------------------------------- shapes

def config1_shapes() -> List[TensorSpec]:
    return [TensorSpec("w0", (256, 256)), TensorSpec("b0", (256,)), TensorSpec("w1", (64, 256))]


def vit_b16_shapes() -> List[TensorSpec]:
    """timm-style ViT-B/16, 1000 classes: 152 tensors, 86,567,656 elements."""
    d, ff, depth = 768, 3072, 12
    t = [TensorSpec("cls_token", (1, 1, d)), TensorSpec("pos_embed", (1, 197, d)),
         TensorSpec("patch_embed.weight", (d, 3, 16, 16)), TensorSpec("patch_embed.bias", (d,))]
    for i in range(depth):
        b = f"blocks.{i}."
        t += [TensorSpec(b + "norm1.weight", (d,)), TensorSpec(b + "norm1.bias", (d,)),
              TensorSpec(b + "attn.qkv.weight", (3 * d, d)), TensorSpec(b + "attn.qkv.bias", (3 * d,)),
              TensorSpec(b + "attn.proj.weight", (d, d)), TensorSpec(b + "attn.proj.bias", (d,)),
              TensorSpec(b + "norm2.weight", (d,)), TensorSpec(b + "norm2.bias", (d,)),
              TensorSpec(b + "mlp.fc1.weight", (ff, d)), TensorSpec(b + "mlp.fc1.bias", (ff,)),
              TensorSpec(b + "mlp.fc2.weight", (d, ff)), TensorSpec(b + "mlp.fc2.bias", (d,))]
    t += [TensorSpec("norm.weight", (d,)), TensorSpec("norm.bias", (d,)),
          TensorSpec("head.weight", (1000, d)), TensorSpec("head.bias", (1000,))]
    return t


def gpt2_medium_shapes() -> List[TensorSpec]:
    """GPT-2 medium with separate q/k/v projections and a tied head: 388 tensors."""
    d, ff, depth, vocab, ctx = 1024, 4096, 24, 50257, 1024
    t = [TensorSpec("wte", (vocab, d)), TensorSpec("wpe", (ctx, d))]
    for i in range(depth):
        b = f"h.{i}."
        t += [TensorSpec(b + "ln_1.weight", (d,)), TensorSpec(b + "ln_1.bias", (d,))]
        for nm in ("q", "k", "v"):
            t += [TensorSpec(b + f"attn.{nm}.weight", (d, d)), TensorSpec(b + f"attn.{nm}.bias", (d,))]
        t += [TensorSpec(b + "attn.proj.weight", (d, d)), TensorSpec(b + "attn.proj.bias", (d,)),
              TensorSpec(b + "ln_2.weight", (d,)), TensorSpec(b + "ln_2.bias", (d,)),
              TensorSpec(b + "mlp.fc.weight", (ff, d)), TensorSpec(b + "mlp.fc.bias", (ff,)),
              TensorSpec(b + "mlp.proj.weight", (d, ff)), TensorSpec(b + "mlp.proj.bias", (d,))]
    t += [TensorSpec("ln_f.weight", (d,)), TensorSpec("ln_f.bias", (d,))]
    return t


def llama_1p3b_shapes(n_tiny: int = 2000) -> List[TensorSpec]:
    """Llama-style 1.3B (24 layers, d 2048, SwiGLU 5504, vocab 32000, untied head)
    plus n_tiny 1-D tensors of length uniform in [1, 512]."""
    d, ff, depth, vocab = 2048, 5504, 24, 32000
    t = [TensorSpec("embed", (vocab, d))]
    for i in range(depth):
        b = f"layers.{i}."
        t += [TensorSpec(b + "attn_norm", (d,))]
        for nm in ("q", "k", "v", "o"):
            t += [TensorSpec(b + f"attn.{nm}", (d, d))]
        t += [TensorSpec(b + "ffn_norm", (d,)),
              TensorSpec(b + "ffn.gate", (ff, d)), TensorSpec(b + "ffn.up", (ff, d)),
              TensorSpec(b + "ffn.down", (d, ff))]
    t += [TensorSpec("norm", (d,)), TensorSpec("lm_head", (vocab, d))]
    rng = np.random.default_rng(np.random.SeedSequence([BASE_SEED, 5, _STREAM_TINY]))
    sizes = rng.integers(1, 513, size=n_tiny)
    t += [TensorSpec(f"tiny.{i}", (int(s),)) for i, s in enumerate(sizes)]
    return t


def mlp_shapes(width: int, depth: int, in_dim: int = 1024, out_dim: int = 10) -> List[TensorSpec]:
    """Optimizee MLP with `depth` hidden layers of `width` units (the paper's controlled width/depth
    sweeps; it does not state input/output sizes, 1024 and 10 are this project's choice)."""
    dims = [in_dim] + [width] * depth + [out_dim]
    t = []
    for i in range(len(dims) - 1):
        t += [TensorSpec(f"fc{i}.weight", (dims[i + 1], dims[i])), TensorSpec(f"fc{i}.bias", (dims[i + 1],))]
    return t


def micro_workload(name: str, optimizer: str = "small_fc_lopt") -> Workload:
    """The paper's micro-workloads as shapes: 'layer1000' = one 1000x1000 weight without bias (its profiler
    figure); 'layer8192' = one 8192x8192 matrix (the step-time figure of its H100 appendix); 'mlp_w<W>_d<D>' = MLP of
    width W and depth D (its scaling figure)."""
    if name == "layer1000":
        tensors = [TensorSpec("fc.weight", (1000, 1000))]
    elif name == "layer8192":
        tensors = [TensorSpec("fc.weight", (8192, 8192))]
    elif name.startswith("mlp_w"):
        w, d = name[5:].split("_d")
        tensors = mlp_shapes(int(w), int(d))
    else:
        raise ValueError(name)
    return Workload(100, name, optimizer, tensors, 40, "gauss_logscale")


def get_workload(config_id: int, optimizer: str | None = None) -> Workload:
    """The five benchmark configurations (configs 4 and 5 take either optimizer; 5 defaults to VeLO)."""
    if config_id == 1:
        return Workload(1, "toy3", "small_fc_lopt", config1_shapes(), 10, "gauss_fixed")
    if config_id == 2:
        return Workload(2, "vit_b16", "small_fc_lopt", vit_b16_shapes(), 100, "gauss_logscale")
    if config_id == 3:
        return Workload(3, "vit_b16", "velo", vit_b16_shapes(), 100, "gauss_logscale",
                        lr_schedule="cosine", weight_decay=0.01)
    if config_id == 4:
        return Workload(4, "gpt2_medium", optimizer or "small_fc_lopt", gpt2_medium_shapes(), 50,
                        "student_t3")
    if config_id == 5:
        return Workload(5, "llama_1p3b_plus_tiny", optimizer or "velo", llama_1p3b_shapes(), 20, "gauss_logscale")
    raise ValueError(f"unknown config {config_id}")


# --------------------------------------------------------------------------- draws

def _rng(config_id: int, tensor_idx: int, stream: int, step: int = 0) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED, config_id, tensor_idx, stream, step]))


def init_param(config_id: int, tensor_idx: int, spec: TensorSpec) -> np.ndarray:
    """p0 ~ N(0, 0.02^2), float32, shape (rows, cols) of spec.as_2d()."""
    _, rows, cols = spec.as_2d()
    r = _rng(config_id, tensor_idx, _STREAM_PARAM)
    return (r.standard_normal(rows * cols, dtype=np.float32) * np.float32(0.02)).reshape(rows, cols)


def grad_scale(config_id: int, tensor_idx: int, grad_kind: str) -> float:
    if grad_kind == "gauss_fixed":
        return 1e-3
    if grad_kind == "gauss_logscale":
        u = _rng(config_id, tensor_idx, _STREAM_SCALE).uniform(-5.0, -2.0)
        return float(10.0 ** u)
    if grad_kind == "student_t3":
        return 1e-3
    raise ValueError(grad_kind)


def grad(config_id: int, tensor_idx: int, step: int, spec: TensorSpec, grad_kind: str) -> np.ndarray:
    """Gradient of one tensor at one step, float32, shape (rows, cols)."""
    _, rows, cols = spec.as_2d()
    n = rows * cols
    r = _rng(config_id, tensor_idx, _STREAM_GRAD, step)
    s = np.float32(grad_scale(config_id, tensor_idx, grad_kind))
    if grad_kind == "student_t3":
        g = r.standard_t(3.0, size=n).astype(np.float32) * s
    else:
        g = r.standard_normal(n, dtype=np.float32) * s
    return g.reshape(rows, cols)


def lr_at(w: Workload, step: int) -> float:
    """Learning rate handed to the step call (float32-representable)."""
    if w.lr_schedule == "cosine":
        v = w.lr * 0.5 * (1.0 + math.cos(math.pi * step / w.steps))
    else:
        v = w.lr
    return float(np.float32(v))


def loss_at(config_id: int, step: int) -> float:
    """Synthetic training-loss value handed to the step beside the gradients (VeLO takes it): a decaying curve with a
    ripple, float32-representable, the same for both sides of a parity test."""
    v = 0.5 + 6.0 * math.exp(-step / 25.0) + 0.3 * math.sin(1.7 * step + 0.1 * config_id)
    return float(np.float32(v))


# --------------------------------------------------------------------------- optimizer weights

N_TIME = 11
N_ELEM_FEATS = 28


def feature_dim(optimizer: str) -> int:
    return N_ELEM_FEATS + (N_TIME if optimizer == "small_fc_lopt" else 1)


def mlp_theta_size(d_in: int, hidden: int) -> int:
    return d_in * hidden + hidden + hidden * hidden + hidden + hidden * 2 + 2


def small_fc_weights(seed: int, hidden: int = 32) -> np.ndarray:
    """Glorot-uniform MLP weights, zero biases except small uniform ones so every
    bias path is exercised. Flat float32: W1[d,H] b1[H] W2[H,H] b2[H] W3[H,2] b3[2]."""
    d = feature_dim("small_fc_lopt")
    r = np.random.default_rng(np.random.SeedSequence([BASE_SEED, _STREAM_WEIGHTS, seed]))

    def glorot(fi, fo):
        lim = math.sqrt(6.0 / (fi + fo))
        return r.uniform(-lim, lim, size=(fi, fo)).astype(np.float32)

    parts = [glorot(d, hidden), r.uniform(-0.1, 0.1, hidden).astype(np.float32),
             glorot(hidden, hidden), r.uniform(-0.1, 0.1, hidden).astype(np.float32),
             glorot(hidden, 2), r.uniform(-0.1, 0.1, 2).astype(np.float32)]
    return np.concatenate([p.ravel() for p in parts])


def small_fc_weights_badly_scaled(seed: int) -> np.ndarray:
    """Legal but far from Glorot: some input rows of the first two layers 200x / 50x larger, some 10^4x smaller, hidden
    biases of order 10, a small last layer (so that the update stays of the order of the parameters). Hidden
    pre-activations reach several 10^4 on an outlier element. Hidden width 32."""
    w = small_fc_weights(seed, 32).copy()
    H, d = 32, feature_dim("small_fc_lopt")
    o = 0
    W1 = w[o:o + d * H].reshape(d, H); o += d * H
    b1 = w[o:o + H]; o += H
    W2 = w[o:o + H * H].reshape(H, H); o += H * H
    b2 = w[o:o + H]; o += H
    W3 = w[o:o + 2 * H].reshape(H, 2)
    r = np.random.default_rng(np.random.SeedSequence([BASE_SEED, _STREAM_WEIGHTS, 5000 + seed]))
    W1[[0, 10, 3, 7]] *= np.float32(200.0)
    W1[[5, 11, 20]] *= np.float32(1e-4)
    W2[[2, 9]] *= np.float32(50.0)
    W2[[4, 20]] *= np.float32(1e-4)
    b1[:] = r.uniform(-10, 10, H).astype(np.float32)
    b2[:] = r.uniform(-10, 10, H).astype(np.float32)
    W3 *= np.float32(2e-4)
    return w


VELO_N_STAT = 29
N_LOSS = 3
VELO_LSTM_IN = VELO_N_STAT + N_TIME + 5 + N_LOSS


def velo_weight_sizes(hidden: int, lstm_hidden: int, n_bank: int):
    theta = mlp_theta_size(VELO_N_STAT, hidden)
    return {
        "Wx": (VELO_LSTM_IN, 4 * lstm_hidden), "Wh": (lstm_hidden, 4 * lstm_hidden),
        "Wg": (lstm_hidden, 4 * lstm_hidden), "b": (4 * lstm_hidden,),
        "Wa": (lstm_hidden, n_bank), "ba": (n_bank,), "ws": (lstm_hidden,), "bs": (1,),
        "B": (n_bank, theta),
    }


def velo_weights(seed: int, hidden: int = 4, lstm_hidden: int = 512, n_bank: int = 256) -> np.ndarray:
    """Seeded random hypernetwork weights, flat float32 in the order
    Wx | Wh | Wg | b | Wa | ba | ws | bs | B (all row-major)."""
    r = np.random.default_rng(np.random.SeedSequence([BASE_SEED, _STREAM_WEIGHTS, 1000 + seed]))
    sz = velo_weight_sizes(hidden, lstm_hidden, n_bank)
    k = 1.0 / math.sqrt(lstm_hidden)
    out = []
    for nm in ("Wx", "Wh", "Wg", "b", "Wa", "ba"):
        out.append(r.uniform(-k, k, size=sz[nm]).astype(np.float32).ravel())
    # step-size head: wide enough that the per-tensor multiplier exp(h . ws + bs) spans about 0.5 .. 2
    out.append(r.uniform(-4 * k, 4 * k, size=sz["ws"]).astype(np.float32).ravel())
    out.append(r.uniform(-0.3, 0.3, size=sz["bs"]).astype(np.float32).ravel())
    # bank scaled so that the mixed per-tensor MLP produces updates of a size comparable to the parameters
    # (a few per cent to a few tens of per cent of rms(p) per step), like the small_fc_lopt test weights do
    lim = 12.0 / math.sqrt(n_bank)
    out.append(r.uniform(-lim, lim, size=sz["B"]).astype(np.float32).ravel())
    return np.concatenate(out)
