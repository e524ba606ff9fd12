"""Full-size checks in the launch configuration `bench.py --workload bert_base_qa` times (BERT-base span QA,
bf16, batch 32, sequence length 384, 12288 tokens): sampled outputs against the oracle, which can afford
single samples because the forward pass is independent per sample, and a property that ties the
full-batch gradient to the small-batch one that is checked against the oracle element by element."""
import numpy as np
import pytest

from oracle import encoder as orc
from paper_2102_03161_amd import binding, synth
from tests import gpu_harness as H
from tests.helpers import oracle_cfg, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


@pytest.fixture(scope="module")
def bertb(torch_mod):
    w = synth.workload("bert_base_qa")
    ctx = binding.Context(binding.make_config(w))
    vals = H.init_values(w, ctx, 4)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, 4, w["B"])
    yield w, ctx, vals, x, y
    ctx.close()


def forward_backward(torch, ctx, x, y):
    hk = ctx.frozen_forward(H.to_dev(torch, x))
    return ctx.active_fwd_bwd(hk, H.to_dev(torch, y))


def test_full_batch_forward_matches_oracle_on_sampled_samples(torch_mod, bertb):
    torch = torch_mod
    w, ctx, vals, x, y = bertb
    B, S, D = w["B"], w["S"], w["D"]
    print("full-size BERT-base B=32 S=384 k=0 forward, sampled against the oracle", flush=True)
    ctx.set_freeze_boundary(0)
    forward_backward(torch, ctx, x, y)
    logits = ctx.read_activation(binding.ACT_LOGITS, (B, S, 2))
    h0 = ctx.read_activation(binding.ACT_HK, (B, S, D))
    hL = ctx.read_activation(binding.ACT_HL, (B, S, D))
    cfg = oracle_cfg(w)
    p = {n: a.astype(np.float64) for n, a in vals.items()}
    for i in (1, B - 1):
        o_h0, _ = orc.frozen_forward(cfg, p, x[i:i + 1], 0)
        o_hL = orc.prefix_forward(cfg, p, o_h0, 0, cfg.L)
        _, o_z, _ = orc.head_loss_forward(cfg, p, o_hL, y[i:i + 1])
        assert rel_err(h0[i], o_h0[0]) < 2e-2
        assert rel_err(hL[i], o_hL[0]) < 2e-2      # the QA head reads every token: all rows are defined
        assert rel_err(logits[i], o_z[0]) < 2e-2, i


def test_full_batch_gradient_is_the_mean_of_sub_batch_gradients(torch_mod, bertb):
    """d(mean loss over 32)/dw = mean over four sub-batches of d(mean loss over 8)/dw."""
    torch = torch_mod
    w, ctx, vals, x, y = bertb
    print("full-size BERT-base B=32 S=384 k=0 gradient against four sub-batches", flush=True)
    tid = {name: t for t, name, *_ in ctx.tensors()}
    probe = ["front.E_p", "front.ln_g", "blk0.Wqkv", "blk0.ln1_g", "blk5.W1", "blk5.bo", "blk11.W2", "blk11.b1", "head.W"]
    ctx.set_freeze_boundary(0)
    forward_backward(torch, ctx, x, y)
    norms = ctx.layer_grad_norms()
    full = {n: ctx.read_tensor(tid[n], binding.KIND_GRAD) for n in probe}
    blk5 = [ctx.read_tensor(tid[f"blk5.{t}"], binding.KIND_GRAD).astype(np.float64) for t in orc.BLOCK_TENSORS]
    assert abs(norms[6] - np.sqrt(sum((a ** 2).sum() for a in blk5))) < 1e-5 * norms[6]
    acc = {n: np.zeros_like(full[n], dtype=np.float64) for n in probe}
    for c in range(4):
        sl = slice(8 * c, 8 * c + 8)
        forward_backward(torch, ctx, x[sl], y[sl])
        for n in probe:
            acc[n] += ctx.read_tensor(tid[n], binding.KIND_GRAD)
    gmax = max(float(np.max(np.abs(a))) for a in full.values())
    for n in probe:
        ref = acc[n] / 4
        err = float(np.max(np.abs(full[n] - ref))) / max(float(np.max(np.abs(ref))), 1e-2 * gmax)
        assert err < 2e-2, (n, err)


def test_sequence_classification_full_batch(torch_mod):
    """BERT-base with the first-token classification head (batch 64, sequence length 128), whose top block
    works on the first-token rows in both directions: sampled logits against the oracle, and the full-batch
    gradient against the mean of eight sub-batch gradients."""
    torch = torch_mod
    w = synth.workload("bert_base_cls")
    print("full-size BERT-base classification B=64 S=128 k=0", flush=True)
    ctx = binding.Context(binding.make_config(w))
    vals = H.init_values(w, ctx, 6)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, 6, w["B"])
    B, S, D = w["B"], w["S"], w["D"]
    forward_backward(torch, ctx, x, y)
    logits = ctx.read_activation(binding.ACT_LOGITS, (B, w["n_out"]))
    hL = ctx.read_activation(binding.ACT_HL, (B, S, D))
    cfg = oracle_cfg(w)
    p = {n: a.astype(np.float64) for n, a in vals.items()}
    for i in (0, 37, B - 1):
        o_h0, _ = orc.frozen_forward(cfg, p, x[i:i + 1], 0)
        o_hL = orc.prefix_forward(cfg, p, o_h0, 0, cfg.L)
        _, o_z, _ = orc.head_loss_forward(cfg, p, o_hL, y[i:i + 1])
        assert rel_err(hL[i][0], o_hL[0][0]) < 2e-2   # first-token row: the only one the top block computes
        # two logits that nearly cancel (|z| = 0.05 from 768 terms): held to the scale of the summands
        scale = np.abs(o_hL[0][0]) @ np.abs(p["head.W"]) + np.abs(p["head.b"])
        assert np.all(np.abs(logits[i] - o_z[0]) < 2e-2 * scale), i
    tid = {name: t for t, name, *_ in ctx.tensors()}
    probe = ["front.E_p", "blk0.Wqkv", "blk5.W1", "blk11.Wqkv", "blk11.Wo", "blk11.W1", "blk11.W2", "blk11.b2",
             "blk11.ln2_g", "head.W"]
    full = {n: ctx.read_tensor(tid[n], binding.KIND_GRAD) for n in probe}
    acc = {n: np.zeros_like(full[n], dtype=np.float64) for n in probe}
    for c in range(8):
        sl = slice(8 * c, 8 * c + 8)
        forward_backward(torch, ctx, x[sl], y[sl])
        for n in probe:
            acc[n] += ctx.read_tensor(tid[n], binding.KIND_GRAD)
    gmax = max(float(np.max(np.abs(a))) for a in full.values())
    for n in probe:
        ref = acc[n] / 8
        err = float(np.max(np.abs(full[n] - ref))) / max(float(np.max(np.abs(ref))), 1e-2 * gmax)
        assert err < 2e-2, (n, err)
    ctx.close()
