"""torch.optim.Optimizer veneer over the C boundary (paper: section "Library design", "Optimization Module":
a standard Optimizer with state dictionaries, composable with LR schedulers and decoupled weight decay).

Nothing numerical happens here: `step()` hands parameter, gradient and state pointers of each parameter group
to lopt_step, with the group's current `lr` and `weight_decay`."""
from __future__ import annotations

from typing import Iterable, Optional

import torch

from .binding import LOPT_SMALL_FC, LOPT_VELO, LearnedOptimizer, default_config, lopt_config


class LearnedOptTorch(torch.optim.Optimizer):
    """small_fc_lopt / VeLO as a torch optimizer.

    params: iterable of parameters or parameter-group dicts (fp32, CUDA, contiguous).
    weights: flat float32 array of the optimizer's own weights (layout: include/lopt.h, lopt_weights_count).
    kind: "small_fc_lopt" or "velo"; cfg overrides the default configuration of that kind.
    """

    def __init__(self, params: Iterable, weights, kind: str = "small_fc_lopt", lr: float = 1.0,
                 weight_decay: float = 0.0, cfg: Optional[lopt_config] = None):
        if kind not in ("small_fc_lopt", "velo"):
            raise ValueError(f"unknown kind {kind!r}")
        super().__init__(params, dict(lr=lr, weight_decay=weight_decay))
        self._cfg = cfg if cfg is not None else default_config(LOPT_SMALL_FC if kind == "small_fc_lopt" else LOPT_VELO)
        self._weights = weights
        self._engines = []
        for group in self.param_groups:
            ps = group["params"]
            for p in ps:
                if not (p.is_cuda and p.dtype == torch.float32 and p.is_contiguous()):
                    raise ValueError("parameters must be contiguous fp32 CUDA tensors")
            dev = ps[0].device if ps else torch.device("cuda:0")
            self._engines.append(LearnedOptimizer(self._cfg, weights, [tuple(p.shape) or (1,) for p in ps], device=dev))

    @torch.no_grad()
    def step(self, loss=None, closure=None):
        """One optimizer step. `loss` (a Python number or a one-element tensor) is the current loss value, the paper's
        call form `optimizer.step(loss)` for VeLO: it feeds the loss features of VeLO's hypernetwork
        (lopt_set_loss); small_fc_lopt ignores it. A callable in its place is taken as torch's closure. Without it (and without a closure's return value) the loss
        features are those of a zero loss. Parameters whose .grad is None are skipped, as torch optimizers do:
        neither they nor their accumulators move, and they do not count in VeLO's cross-tensor mean of that step."""
        out = None
        if callable(loss) and closure is None:
            loss, closure = None, loss
        if closure is not None:
            with torch.enable_grad():
                out = closure()
        if loss is None:
            loss = out
        loss_value = 0.0 if loss is None else float(loss)
        for group, eng in zip(self.param_groups, self._engines):
            ps = group["params"]
            idx = [i for i, p in enumerate(ps) if p.grad is not None]
            if not idx:
                continue
            gs = []
            for i in idx:
                g = ps[i].grad
                if not (g.is_contiguous() and g.dtype == torch.float32):
                    g = g.contiguous().float()
                gs.append(g)
            eng.step([ps[i] for i in idx], gs, lr=float(group["lr"]), weight_decay=float(group["weight_decay"]),
                     loss=loss_value, indices=None if len(idx) == len(ps) else idx)
        return out

    def state_dict(self):
        sd = super().state_dict()
        sd["lopt"] = [{"step": eng.step_count, "blobs": [b.clone() for b in eng.state]} for eng in self._engines]
        return sd

    def load_state_dict(self, state_dict):
        lopt = state_dict.get("lopt")
        super().load_state_dict({k: v for k, v in state_dict.items() if k != "lopt"})
        if lopt is not None:
            for eng, rec in zip(self._engines, lopt):
                if len(rec["blobs"]) != len(eng.state):
                    raise ValueError("state dict does not match this optimizer's parameter list")
                for dst, src in zip(eng.state, rec["blobs"]):
                    dst.copy_(src)
                eng.step_count = int(rec["step"])
