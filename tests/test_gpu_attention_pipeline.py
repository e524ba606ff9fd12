"""Shapes that take the pipelined attention backward kernel (head size 64, 129 to 208 tokens, more heads than
the chip has compute units, so that workgroups walk over several heads) with everything ragged that can be:
a head count that is no multiple of the number of workgroups, a sequence that ends inside a 32-row tile, inside
a 16-row image block, or exactly on the image's last row.  One block, narrow MLP: the attention gradients carry
the step.  bf16 mode against the exact oracle (or the bf16 storage model) at 2e-2, value by value, as for every
other shape."""
import pytest

from paper_2102_03161_amd import binding
from tests import gpu_harness as H

pytestmark = pytest.mark.gpu

CASES = [
    # 53 x 5 = 265 heads, S = 161: six tiles, the last with one row; image of 176 rows
    (dict(arch="bert", L=1, D=320, H=5, F=64, S=161, n_out=2, img=0, patch=0, chans=0, vocab=50, max_pos=161,
          ln_eps=1e-12, B=53, optimizer="adamw", dtype="bf16"), 0, 53, 301),
    # 65 x 4 = 260 heads, S = 208: the image's last row is a real row, the last tile reads 16 rows past it
    (dict(arch="bert", L=1, D=256, H=4, F=64, S=208, n_out=2, img=0, patch=0, chans=0, vocab=50, max_pos=208,
          ln_eps=1e-12, B=65, optimizer="adamw", dtype="bf16", head="cls"), 0, 65, 302),
    # ViT-B/16's attention shape (12 heads of 197 tokens) at batch 23: 276 heads over 256 workgroups
    (dict(arch="vit", L=1, D=768, H=12, F=128, S=197, n_out=10, img=224, patch=16, chans=3, vocab=0, max_pos=0,
          ln_eps=1e-6, B=23, optimizer="adamw", dtype="bf16"), 0, 23, 303),
]


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


@pytest.mark.parametrize("case", CASES, ids=[f"{c[0]['arch']}_S{c[0]['S']}_H{c[0]['H']}_B{c[2]}" for c in CASES])
def test_pipelined_attention_backward(torch_mod, case):
    w, k, nb, seed = case
    print(f"attention pipeline case S={w['S']} H={w['H']} B={nb}", flush=True)
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
