"""A shape that takes the weight-gradient launch's riders off the benchmarked path: pre-LN blocks of width 1024
(the LayerNorm pass on board runs with four 256-column groups per lane instead of three), a narrow MLP, so that
a block's four matrices have 72 tiles and split three ways (the carried slab summation adds three slabs, and
the column-sum partials of two biases ride with it), 12608 tokens (a multiple of 64, which the grouped launch
needs).  Three blocks: the top one runs on the class-token rows, the two below hand their slabs on.  bf16 mode
against the exact oracle (or the bf16 storage model) at 2e-2, value by value."""
import pytest

from paper_2102_03161_amd import binding
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu

CASE = (dict(arch="vit", L=3, D=1024, H=16, F=256, S=197, n_out=10, img=224, patch=16, chans=3, vocab=0, max_pos=0,
             ln_eps=1e-6, B=64, optimizer="adamw", dtype="bf16"), 0, 64, 311)


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def test_riders_with_three_way_split_and_wide_rows(torch_mod):
    w, k, nb, seed = CASE
    print("weight-gradient riders, D=1024, three-way split", flush=True)
    ctx = binding.Context(binding.make_config(w, B=nb))
    vals = H.init_values(w, ctx, seed)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, seed, nb)
    g = H.gpu_step(torch_mod, ctx, w, x, y, k)
    ctx.close()
    o = H.oracle_step(w, vals, x, y, k)
    m = H.storage_model_step(w, vals, x, y, k)
    rss = H.summand_rss(w, vals, x, y, k)
    e = H.grad_errors(w, g["grads"], o["grads"], o["cfg"], k, rss)
    print(f"  bf16 vs exact: worst {max(e.values()):.2e}", flush=True)
    H.compare_step(w, g, o, k, 2e-2, check_params=False, model=m, rss=rss)
