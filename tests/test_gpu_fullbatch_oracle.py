"""The full batch of the benchmarked configurations against the oracle, element by element on every gradient
tensor: ViT-B/16 micro-batch 64 at k = 0 and 6 and micro-batch 128 at k = 9, BERT-base span QA batch 32 (S = 384) at
k = 0, 4 and 8 -- the
launch configurations bench.py times (192x256 and 256x256 two-group tiles, the grouped weight-gradient launch
with its split over the tokens, fused attention backward at full occupancy).  The oracle computes the same
batch in sub-batches (oracle.accumulated_fwd_bwd, fp64) to bound host memory; the loss and the gradient of the
mean loss are the sample-weighted means.  Tolerance: 2e-2 per tensor (max |a-b| / max |b|), loss and norms 2e-2."""
import time

import numpy as np
import pytest

from oracle import encoder as orc
from paper_2102_03161_amd import binding, synth
from tests import gpu_harness as H
from tests.helpers import oracle_cfg

pytestmark = pytest.mark.gpu

TOL = 2e-2


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def full_batch_case(torch, name, seed, ks, sub):
    w = synth.workload(name)
    B = w["B"]
    ctx = binding.Context(binding.make_config(w))
    vals = H.init_values(w, ctx, seed)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, seed, B)
    cfg = oracle_cfg(w)
    p = {n: a.astype(np.float64) for n, a in vals.items()}
    xx = x.astype(np.float64) if w["arch"] == "vit" else x
    dx, dy = H.to_dev(torch, x), H.to_dev(torch, y)
    for k in ks:
        print(f"full batch {name} B={B} k={k}: GPU step", flush=True)
        ctx.set_freeze_boundary(k)
        loss = ctx.active_fwd_bwd(ctx.frozen_forward(dx, None), dy)
        norms = ctx.layer_grad_norms()
        grads = H.gpu_read_all(ctx, binding.KIND_GRAD)
        t0 = time.time()
        o_loss, o_grads = orc.accumulated_fwd_bwd(cfg, p, xx, y, k, [sub] * (B // sub))
        o_norms = orc.layer_grad_norms(cfg, o_grads, k)
        print(f"  oracle: {time.time() - t0:.1f} s", flush=True)
        errs = H.grad_errors(w, grads, o_grads, cfg, k)
        errs["loss"] = abs(loss - o_loss) / abs(o_loss)
        for i, n in enumerate(o_norms):
            if n == 0.0:
                assert norms[i] == 0.0, i
            else:
                errs[f"norm{i}"] = abs(norms[i] - n) / n
        worst = sorted(errs.items(), key=lambda kv: -kv[1])[:4]
        # how many tensors sit below one-hundredth of the model's largest gradient (the floor that used to
        # apply to every tensor), and the worst error among them
        gmax = max(float(np.abs(a).max()) for a in o_grads.values())
        small = [n for n, a in o_grads.items() if float(np.abs(a).max()) < 1e-2 * gmax and n not in H.exactly_cancelling(w, k)]
        worst_small = max((errs["grad:" + n] for n in small), default=0.0)
        print(f"  {len(errs)} values compared; worst {[(n, f'{e:.2e}') for n, e in worst]}; "
              f"{len(small)} tensors below gmax/100, worst of them {worst_small:.2e}", flush=True)
        bad = {n: e for n, e in errs.items() if not (e <= TOL)}
        assert not bad, bad
    ctx.close()


# one case per test, so that a test never computes for more than about half a minute without reporting
@pytest.mark.parametrize("k", [0, 6])
def test_vit_b16_full_batch_against_the_oracle(torch_mod, k):
    full_batch_case(torch_mod, "vit_b16", 2, (k,), 8)


@pytest.mark.parametrize("k", [0, 4, 8])
def test_bert_base_full_batch_against_the_oracle(torch_mod, k):
    full_batch_case(torch_mod, "bert_base_qa", 4, (k,), 4)


def test_vit_b16_b128_full_batch_against_the_oracle(torch_mod):
    """Micro-batch 128 (the freeze-schedule configuration: 25216 tokens, other tile counts and split depths than
    at 64), at the last boundary of the schedule."""
    full_batch_case(torch_mod, "vit_b16_b128", 5, (9,), 8)
