"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (every tensor of the model in one lopt_step). The oracle verifies sampled tensors element by
element (one tensor of every shape class; the oracle needs ~2.6 s per million elements), every tensor is
checked against the closed forms that hold after the first step, and all outputs must stay finite.
Tensors too large for the oracle in a test (the 51M / 65M-element embeddings) are covered by the closed
forms here and by tests/test_gpu_parity.py::test_tall_and_wide_tensors for the tall-tile code path."""
import numpy as np
import pytest

import workloads as W
from tests import harness as Hn

pytestmark = pytest.mark.gpu


def _idx(wl, names):
    by = {t.name: i for i, t in enumerate(wl.tensors)}
    return [by[nm] for nm in names]


def _progress(capsys):
    def p(msg):
        with capsys.disabled():
            print(msg, flush=True)
    return p


VIT_SAMPLE = ["cls_token", "pos_embed", "patch_embed.weight", "patch_embed.bias", "blocks.5.norm1.weight",
              "blocks.5.attn.qkv.weight", "blocks.5.attn.qkv.bias", "blocks.5.attn.proj.weight",
              "blocks.11.mlp.fc1.weight", "blocks.11.mlp.fc1.bias", "blocks.0.mlp.fc2.weight",
              "head.weight", "head.bias"]
VIT_SAMPLE_LATE = ["blocks.5.attn.proj.weight", "blocks.5.attn.qkv.bias", "head.weight", "pos_embed", "norm.bias"]


def test_config2_vit_b16_small_fc_full_size(capsys):
    wl = W.get_workload(2)
    cfg = Hn.make_cfg("small_fc_lopt")
    case = Hn.Case(2, wl.tensors, wl.grad_kind)
    worst = Hn.run_forced(case, cfg, W.small_fc_weights(0, 32), steps=3,
                          checks={0: _idx(wl, VIT_SAMPLE), 2: _idx(wl, VIT_SAMPLE_LATE)},
                          lr_fn=lambda t: W.lr_at(wl, t), wd=wl.weight_decay, progress=_progress(capsys))
    _progress(capsys)(f"config 2 worst: {worst}")


def test_config3_vit_b16_velo_full_size(capsys):
    wl = W.get_workload(3)
    cfg = Hn.make_cfg("velo")
    case = Hn.Case(3, wl.tensors, wl.grad_kind)
    worst = Hn.run_forced(case, cfg, W.velo_weights(0), steps=3,
                          checks={0: _idx(wl, VIT_SAMPLE), 2: _idx(wl, VIT_SAMPLE_LATE)},
                          lr_fn=lambda t: W.lr_at(wl, t), wd=wl.weight_decay, progress=_progress(capsys))
    _progress(capsys)(f"config 3 worst: {worst}")


GPT_SAMPLE = ["wpe", "h.3.ln_1.weight", "h.3.attn.q.weight", "h.3.attn.q.bias", "h.7.mlp.fc.weight",
              "h.7.mlp.fc.bias", "h.20.mlp.proj.weight", "ln_f.bias"]
GPT_SAMPLE_LATE = ["h.3.attn.q.weight", "h.7.mlp.fc.bias", "ln_f.bias"]


@pytest.mark.parametrize("optimizer", ["small_fc_lopt", "velo"])
def test_config4_gpt2_medium_full_size(optimizer, capsys):
    wl = W.get_workload(4, optimizer)
    cfg = Hn.make_cfg(optimizer)
    w = W.small_fc_weights(0, 32) if optimizer == "small_fc_lopt" else W.velo_weights(0)
    case = Hn.Case(4, wl.tensors, wl.grad_kind)
    worst = Hn.run_forced(case, cfg, w, steps=2, checks={0: _idx(wl, GPT_SAMPLE), 1: _idx(wl, GPT_SAMPLE_LATE)},
                          progress=_progress(capsys))
    _progress(capsys)(f"config 4 {optimizer} worst: {worst}")


def test_config5_llama_1p3b_velo_full_size(capsys):
    wl = W.get_workload(5)
    cfg = Hn.make_cfg("velo")
    case = Hn.Case(5, wl.tensors, wl.grad_kind)
    tiny = [i for i, t in enumerate(wl.tensors) if t.name.startswith("tiny.")]
    assert len(tiny) == 2000
    big = _idx(wl, ["layers.3.attn.q", "layers.10.attn_norm", "layers.20.ffn.gate", "norm"])
    worst = Hn.run_forced(case, cfg, W.velo_weights(0), steps=2,
                          checks={0: big + tiny, 1: tiny[::10] + _idx(wl, ["layers.10.attn_norm"])},
                          progress=_progress(capsys))
    _progress(capsys)(f"config 5 worst: {worst}")
