"""pt_layer_grad_norms_static (the entry point that allocates nothing: its per-chunk partial sums live in the
library's static device array) against pt_layer_grad_norms, through the C ABI, on two calls in a row, the
second over a smaller input.  Same kernels, same order of additions: the norms must agree bit for bit."""
import numpy as np
import pytest

from paper_2102_03161_amd import binding, synth
from tests import gpu_harness as H
from tests.test_gpu_parity import MID_BERT, MID_VIT

pytestmark = pytest.mark.gpu


def _norms_both_ways(torch, w, k, seed):
    ctx = binding.Context(binding.make_config(w))
    vals = H.init_values(w, ctx, seed)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, seed, w["B"])
    ctx.set_freeze_boundary(k)
    hk = ctx.frozen_forward(H.to_dev(torch, x), None)
    ctx.active_fwd_bwd(hk, H.to_dev(torch, y))
    ref = ctx.layer_grad_norms()
    got = ctx.layer_grad_norms_static()
    again = ctx.layer_grad_norms()
    ctx.close()
    return ref, got, again


def test_static_scratch_norms_equal_the_workspace_norms_twice_in_a_row():
    import torch
    assert torch.cuda.is_available()
    # first call: 3-block ViT, everything active; second call: a smaller model with a frozen prefix, which
    # leaves most of what the first call wrote into the shared array untouched and must not read it
    big = dict(MID_VIT, dtype="bf16")
    small = dict(MID_BERT, dtype="f32", L=2, D=128, H=2, F=256, S=9, B=3, vocab=50, max_pos=12)
    for w, k, seed in ((big, 0, 11), (small, 1, 12)):
        print(f"static norms: arch={w['arch']} L={w['L']} D={w['D']} k={k}", flush=True)
        ref, got, again = _norms_both_ways(torch, w, k, seed)
        assert np.array_equal(ref, again)
        assert np.array_equal(got, ref), (got, ref)
        assert np.all(ref[1:1 + k] == 0.0) and np.all(ref[1 + k:] > 0.0)
        if k > 0:
            assert ref[0] == 0.0
