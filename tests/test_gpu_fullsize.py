"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (every tensor of the model in one lopt_step). Coverage:
  * ViT-B/16 shapes (both optimizers): EVERY tensor against the oracle at steps 0 and 1 (teacher-forced from the GPU's
    own state), a sample at step 2; free-running for the configuration's 100 steps on nine vectors and the 768 x 768
    projection, and for 20 steps on one matrix of every other shape class (qkv, fc1, fc2, patch embedding, head);
  * GPT-2-medium shapes (both optimizers): one tensor of every shape class at steps 0 and 1; the 50257 x 1024 embedding
    at both steps through oracle.tensor_statistics and oracle.apply_rows (accumulators in full, statistics, first /
    middle / last row slabs); free-running for 50 steps on eight vectors and for 20 steps on 1024 x 1024, 4096 x 1024,
    1024 x 4096 and the position embedding;
  * Llama-1.3B shapes + 2000 tiny tensors (VeLO): shape classes and every tiny tensor at step 0; both 32000 x 2048
    matrices by slabs at steps 0 and 1; free-running for 20 steps on 100 tiny tensors, three norm vectors and a
    2048 x 2048 matrix, 5 steps on a 5504 x 2048 and a 2048 x 5504 matrix;
  * every tensor of every set against the closed forms that hold after the first step; all outputs finite.
The oracle steps independent tensors on a thread pool (about 2.4 M elements/s per thread on the GPU machine's host).
Further down: tensors at the size limits (inputs that tile a small pattern, so that the oracle's result for the
pattern is the expected value of every element)."""
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


@pytest.mark.parametrize("config", [2, 3])
def test_vit_b16_every_tensor_for_two_steps(config, capsys):
    # all 152 tensors (86.6 M elements) go through the oracle at steps 0 and 1, a sample again at step 2
    wl = W.get_workload(config)
    cfg = Hn.make_cfg(wl.optimizer)
    w = W.small_fc_weights(0, 32) if wl.optimizer == "small_fc_lopt" else W.velo_weights(0)
    case = Hn.Case(config, wl.tensors, wl.grad_kind)
    everything = list(range(len(wl.tensors)))
    worst = Hn.run_forced(case, cfg, w, steps=3, checks={0: everything, 1: everything, 2: _idx(wl, VIT_SAMPLE_LATE)},
                          lr_fn=lambda t: W.lr_at(wl, t), wd=wl.weight_decay, progress=_progress(capsys))
    _progress(capsys)(f"config {config}: all {len(everything)} tensors at steps 0 and 1, worst: {worst}")


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
                          slab_checks={0: _idx(wl, ["wte"]), 1: _idx(wl, ["wte"])}, progress=_progress(capsys))
    _progress(capsys)(f"config 4 {optimizer} worst: {worst}")


def test_config5_llama_1p3b_velo_full_size(capsys):
    wl = W.get_workload(5)
    cfg = Hn.make_cfg("velo")
    case = Hn.Case(5, wl.tensors, wl.grad_kind)
    tiny = [i for i, t in enumerate(wl.tensors) if t.name.startswith("tiny.")]
    assert len(tiny) == 2000
    big = _idx(wl, ["layers.3.attn.q", "layers.10.attn_norm", "layers.20.ffn.gate", "norm"])
    emb = _idx(wl, ["embed", "lm_head"])
    worst = Hn.run_forced(case, cfg, W.velo_weights(0), steps=2,
                          checks={0: big + tiny, 1: tiny[::10] + _idx(wl, ["layers.10.attn_norm"])},
                          slab_checks={0: emb, 1: emb}, progress=_progress(capsys))
    _progress(capsys)(f"config 5 worst: {worst}")


def _periodic_tensor_case(kind, reps_r, reps_c, say, tag, pr=4, pc=4):
    """One tensor of (pr reps_r) x (pc reps_c) elements whose parameters and gradients tile a pr x pc base pattern: every
    row mean, column mean and whole-tensor mean is that of the base pattern, so the oracle's result for the pr x pc
    tensor, tiled, is the expected value of EVERY element (all of them are compared, on the device). Two steps: the
    second one runs on non-zero accumulators."""
    import torch
    import paper_2506_10315_amd as P
    from oracle import lopt_oracle as O
    dev = "cuda:0"
    rows, cols = pr * reps_r, pc * reps_c
    cfg = Hn.make_cfg(kind)
    ocfg = Hn.oracle_config_from(cfg)
    w = W.small_fc_weights(0, 32) if kind == "small_fc_lopt" else W.velo_weights(0)
    rng = np.random.default_rng([20250610, 900, 0 if kind == "small_fc_lopt" else 1])
    p_base = (rng.standard_normal((pr, pc)) * 0.02).astype(np.float32)
    g_base = [(rng.standard_normal((pr, pc)) * 1e-3).astype(np.float32) for _ in range(2)]

    def tile_into(dst2d, base):
        dst2d.view(reps_r, pr, reps_c, pc).copy_(torch.from_numpy(base).to(dev).view(1, pr, 1, pc))

    def tiled_err(t2d, base64):
        # oracle.rel_err of the tiled expectation, evaluated on the device in chunks of about 2^28 elements
        b = torch.from_numpy(np.asarray(base64, np.float64).astype(np.float32)).to(dev).view(1, pr, 1, pc)
        rms = float(np.sqrt(np.mean(np.asarray(base64, np.float64) ** 2)))
        den = b.abs() + rms
        v = t2d.view(reps_r, pr, reps_c, pc)
        worst = 0.0
        if reps_r > 1:
            step = max(1, (1 << 24) // reps_c)
            for a0 in range(0, reps_r, step):
                worst = max(worst, float(((v[a0:a0 + step] - b).abs_() / den).amax()))
        else:
            for c0 in range(0, reps_c, 1 << 24):
                worst = max(worst, float(((v[:, :, c0:c0 + (1 << 24)] - b).abs_() / den).amax()))
        return worst

    def vec_err(t1d, base64, reps):
        # a vector over rows or columns: compared on the device against the tiled base values
        k = len(base64)
        b = torch.from_numpy(np.asarray(base64, np.float64).astype(np.float32)).to(dev).view(1, k)
        rms = float(np.sqrt(np.mean(np.asarray(base64, np.float64) ** 2)))
        return float(((t1d.view(reps, k) - b).abs() / (b.abs() + rms)).amax())

    opt = P.LearnedOptimizer(cfg, w, [(rows, cols)], device=dev)
    p = torch.empty((rows, cols), dtype=torch.float32, device=dev)
    g = torch.empty((rows, cols), dtype=torch.float32, device=dev)
    tile_into(p, p_base)
    p_ora = p_base.astype(np.float64)
    st = O.init_state(pr, pc, ocfg)
    lr, wd = 1.0, float(np.float32(0.01))
    for t in range(2):
        tile_into(g, g_base[t])
        say(f"{tag} {kind}: step {t}")
        opt.step([p], [g], lr=lr, weight_decay=wd, step=t)
        torch.cuda.synchronize()
        p_ora = O.tensor_step(p_ora, g_base[t], st, w, ocfg, t, lr, wd, ndim=2)
        e = tiled_err(p, p_ora)
        assert e <= Hn.TOL_PARAM, f"step {t}: parameter rel err {e:.3e}"
        sv = opt.state_views(0)
        for k in range(3):
            assert tiled_err(sv["M"][k], st["M"][k]) <= Hn.TOL_ACC, f"step {t}: M{k + 1}"
            assert vec_err(sv["r"][k], st["r"][k], reps_r) <= Hn.TOL_ACC, f"step {t}: r{k + 1}"
            assert vec_err(sv["c"][k], st["c"][k], reps_c) <= Hn.TOL_ACC, f"step {t}: c{k + 1}"
        assert tiled_err(sv["V"], st["V"]) <= Hn.TOL_ACC, f"step {t}: V"
        say(f"{tag} {kind}: step {t} parameter rel err {e:.2e}")
    opt.close()
    del p, g
    torch.cuda.empty_cache()


@pytest.mark.parametrize("kind", ["small_fc_lopt", "velo"])
def test_maximum_size_tensor_matches_its_periodic_base_pattern(kind, capsys):
    # 46340 x 46340 = 2,147,395,600 elements (the boundary admits up to 2^31 - 1 per tensor): byte offsets beyond 2^32
    # in every streamed array
    _periodic_tensor_case(kind, 11585, 11585, _progress(capsys), "maximum size")


def test_widest_tensor_matches_its_periodic_base_pattern(capsys):
    # 4 x 2^28: a million column tiles per pass; the strip-form apply kernel's 32-bit lane offsets (relative to the
    # tile's first column) at 4 GiB per row
    _periodic_tensor_case("small_fc_lopt", 1, 1 << 26, _progress(capsys), "widest")


def test_two_row_tensor_with_lane_offsets_beyond_2_to_31(capsys):
    # 2 x 536,870,944: the upper half of every wavefront of the strip-form apply kernel addresses its row with a lane
    # offset of 4 n = 2^31 + 128 bytes and more, in the loads and in the (range-checked, unsigned) buffer stores
    _periodic_tensor_case("small_fc_lopt", 1, (1 << 27) + 8, _progress(capsys), "two rows, 2^29 + 32 columns", pr=2, pc=4)


def test_tallest_tensor_matches_its_periodic_base_pattern(capsys):
    # 2^28 x 4: the tallest statistics tiles (64 row tiles of 4,194,304 rows), a million row blocks in the row/column
    # pass, apply tiles with one of four column strips in use
    _periodic_tensor_case("small_fc_lopt", 1 << 26, 1, _progress(capsys), "tallest")


@pytest.mark.parametrize("kind", ["small_fc_lopt", "velo"])
def test_maximum_size_tensor_with_unaligned_rows(kind, capsys):
    # 32768 x 65535 = 2,147,450,880 elements, rows of 65535 floats (not a multiple of 4): the scalar-access
    # instantiations of every pass at byte offsets beyond 2^32; base pattern 4 x 3
    _periodic_tensor_case(kind, 8192, 21845, _progress(capsys), "maximum size, unaligned rows", pr=4, pc=3)


VIT_LONG_RUN = ["cls_token", "pos_embed", "patch_embed.bias", "blocks.5.norm1.weight", "blocks.5.attn.qkv.bias",
                "blocks.11.mlp.fc1.bias", "blocks.0.mlp.fc2.bias", "norm.bias", "head.bias", "blocks.5.attn.proj.weight"]
VIT_TWENTY = ["blocks.2.attn.qkv.weight", "blocks.11.mlp.fc1.weight", "blocks.0.mlp.fc2.weight", "patch_embed.weight",
              "head.weight"]


@pytest.mark.parametrize("config", [2, 3])
def test_vit_b16_hundred_steps_free_running(config, capsys):
    # the configurations' own step count (100), learning-rate schedule and weight decay: the GPU steps the whole
    # ViT-B/16 set; the oracle free-runs nine vectors and the 768 x 768 projection for all 100 steps and one matrix of
    # every other shape class (qkv, fc1, fc2, patch embedding, head) for the first 20
    wl = W.get_workload(config)
    cfg = Hn.make_cfg(wl.optimizer)
    w = W.small_fc_weights(0, 32) if wl.optimizer == "small_fc_lopt" else W.velo_weights(0)
    twenty = _idx(wl, VIT_TWENTY)
    worst = Hn.run_free_subset(Hn.Case(config, wl.tensors, wl.grad_kind), cfg, w, wl.steps,
                               _idx(wl, VIT_LONG_RUN) + twenty, check_steps={0, 9, 24, 49, 74, wl.steps - 1},
                               lr_fn=lambda t: W.lr_at(wl, t), wd=wl.weight_decay, progress=_progress(capsys),
                               limits={i: 20 for i in twenty})
    _progress(capsys)(f"config {config}, {wl.steps} steps free-running: worst {worst}")


@pytest.mark.parametrize("optimizer", ["small_fc_lopt", "velo"])
def test_gpt2_medium_fifty_steps_free_running(optimizer, capsys):
    # configuration 4 at its own step count (50, Student-t gradients): eight vectors for all 50 steps, one matrix of
    # every shape class but the token embedding for the first 20
    wl = W.get_workload(4, optimizer)
    cfg = Hn.make_cfg(optimizer)
    w = W.small_fc_weights(0, 32) if optimizer == "small_fc_lopt" else W.velo_weights(0)
    names = ["h.0.ln_1.weight", "h.3.attn.q.bias", "h.7.mlp.fc.bias", "h.12.ln_2.bias", "h.20.mlp.proj.bias",
             "h.23.attn.proj.bias", "ln_f.weight", "ln_f.bias"]
    twenty = _idx(wl, ["h.3.attn.q.weight", "h.7.mlp.fc.weight", "h.20.mlp.proj.weight", "wpe"])
    worst = Hn.run_free_subset(Hn.Case(4, wl.tensors, wl.grad_kind), cfg, w, wl.steps, _idx(wl, names) + twenty,
                               check_steps={0, 9, 24, wl.steps - 1}, progress=_progress(capsys),
                               limits={i: 20 for i in twenty})
    _progress(capsys)(f"config 4 {optimizer}, {wl.steps} steps free-running: worst {worst}")


def test_llama_1p3b_twenty_steps_free_running(capsys):
    # configuration 5 at its own step count (20): 100 of the 2000 tiny tensors, three norm vectors and a 2048 x 2048
    # projection for all 20 steps, a 5504 x 2048 and a 2048 x 5504 matrix for the first 5
    wl = W.get_workload(5)
    cfg = Hn.make_cfg("velo")
    tiny = [i for i, t in enumerate(wl.tensors) if t.name.startswith("tiny.")]
    five = _idx(wl, ["layers.20.ffn.gate", "layers.12.ffn.down"])
    sub = tiny[::20] + _idx(wl, ["layers.0.attn_norm", "layers.10.attn_norm", "norm", "layers.3.attn.q"]) + five
    worst = Hn.run_free_subset(Hn.Case(5, wl.tensors, wl.grad_kind), cfg, W.velo_weights(0), wl.steps, sub,
                               check_steps={0, 4, 9, wl.steps - 1}, progress=_progress(capsys),
                               limits={i: 5 for i in five})
    _progress(capsys)(f"config 5, {wl.steps} steps free-running: worst {worst}; LSTM state, whole session: {Hn.WORST_LSTM[0]:.2e}")


def test_config2_default_launch_plan_is_bit_identical_to_one_stream_at_full_size(monkeypatch):
    # ViT-B/16 shapes: the default plan (four tensor groups on two streams, tiles from a device counter) against every
    # pass over the whole list on one stream; three steps on seeded on-device inputs; parameters and state compared
    # bit by bit on the device
    import torch
    import paper_2506_10315_amd as P
    wl = W.get_workload(2)
    cfg = Hn.make_cfg("small_fc_lopt")
    w = W.small_fc_weights(0, 32)
    case = Hn.Case(2, wl.tensors, wl.grad_kind)
    dev = "cuda:0"

    def run():
        opt = P.LearnedOptimizer(cfg, w, [t.shape for t in wl.tensors], device=dev)
        ps = []
        for i, t in enumerate(wl.tensors):
            gen = torch.Generator(device=dev)
            gen.manual_seed(W.BASE_SEED + 7919 * i)
            _, rows, cols = t.as_2d()
            ps.append(torch.randn(rows, cols, generator=gen, device=dev, dtype=torch.float32) * 0.02)
        for s in range(3):
            gs = [Hn._device_grad(case, i, s, dev) for i in range(len(wl.tensors))]
            opt.step(ps, gs, lr=0.5, weight_decay=0.01, step=s)
        torch.cuda.synchronize()
        out = ps + [b.clone() for b in opt.state]
        opt.close()
        return out

    monkeypatch.setenv("LOPT_GROUPS", "1")
    ref = run()
    monkeypatch.delenv("LOPT_GROUPS")
    got = run()
    assert len(ref) == len(got)
    for a, b in zip(ref, got):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
