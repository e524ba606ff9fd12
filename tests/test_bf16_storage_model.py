"""The bf16 storage model (tests/bf16_storage_model.py) pinned to the oracle, and what it says about the small
configurations on which the bf16 step exceeds the 2e-2 bar of the named workloads.  CPU only."""
import numpy as np
import pytest

from oracle import encoder as orc
from paper_2102_03161_amd import synth
from tests import bf16_storage_model as M
from tests.helpers import SMALL_BERT, SMALL_BERT_CLS, SMALL_VIT, oracle_cfg
from tests.small_shape_cases import CASES, case_id


def _setup(w, seed, nb):
    cfg = oracle_cfg(w)
    p = {n: synth.round_bf16(synth.gen_param(seed, n, s)).astype(np.float64) for n, s in orc.param_shapes(cfg).items()}
    x, y = synth.gen_inputs(w, seed, nb)
    if w["arch"] == "vit":
        x = synth.round_bf16(x).astype(np.float64)
    return cfg, p, x, y


@pytest.mark.parametrize("w", [SMALL_VIT, SMALL_BERT, SMALL_BERT_CLS], ids=["vit", "bert", "bert_cls"])
@pytest.mark.parametrize("k", [0, 1, 3])
def test_without_rounding_the_model_is_the_oracle(monkeypatch, w, k):
    """With the rounding switched off the model must give the oracle's loss, activations and gradients (up to
    the order of fp64 additions): it adds rounding points to the oracle's arithmetic and nothing else."""
    monkeypatch.setattr(M, "r", lambda a: np.asarray(a, dtype=np.float64))
    cfg, p, x, y = _setup(w, 5, w["B"])
    hk, fs = orc.frozen_forward(cfg, p, x, k)
    loss, grads, aux = orc.active_fwd_bwd(cfg, p, hk, y, k, fs)
    lm, gm, am = M.step(cfg, p, x, y, k)
    assert abs(lm - loss) <= 1e-13 * abs(loss)
    assert np.allclose(am["h_k"], hk, rtol=0, atol=1e-12) and np.allclose(am["h_L"], aux["h_L"], rtol=0, atol=1e-12)
    assert set(gm) == set(grads)
    for n in grads:
        assert np.allclose(gm[n], grads[n], rtol=0, atol=1e-13 * max(1.0, float(np.abs(grads[n]).max()))), n


def test_rounding_is_to_nearest_even_bf16():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.1], dtype=np.float64)
    assert np.array_equal(M.r(x), np.array([1.0, 1.0, 1.015625, -2.5, 0.10009765625]))


# (the D = 2048 case takes the oracle most of a minute: the GPU test covers it)
@pytest.mark.parametrize("case", CASES[:8], ids=[case_id(c) for c in CASES[:8]])
def test_storage_rounding_alone_leaves_the_bar_of_the_named_workloads(case):
    """On these shapes the exact arithmetic with nothing but bf16 storage of activations and matrix-core
    operands is already further than 1.5e-2 (most of them further than 2e-2) from the exact result on some
    gradient tensor or on the logits: no implementation that keeps those tensors in bf16 can meet 2e-2 against the exact oracle here, which
    is why the GPU test holds the library to this model on them (and to the exact oracle in fp32 mode)."""
    w, k, nb, seed = case
    cfg, p, x, y = _setup(w, seed, nb)
    hk, fs = orc.frozen_forward(cfg, p, x, k)
    _, grads, aux = orc.active_fwd_bwd(cfg, p, hk, y, k, fs)
    _, gm, am = M.step(cfg, p, x, y, k)
    gmax = max(float(np.abs(a).max()) for a in grads.values())
    dev = {n: float(np.abs(gm[n] - grads[n]).max() / np.abs(grads[n]).max()) for n in grads if np.abs(grads[n]).max() > 1e-9 * gmax}
    dev["logits"] = float(np.abs(am["logits"] - aux["logits"]).max() / np.abs(aux["logits"]).max())
    dev["h_L"] = float(np.abs(am["h_L"] - aux["h_L"]).max() / np.abs(aux["h_L"]).max())
    worst = max(dev, key=dev.get)
    print(f"{case_id(case)}: worst {worst} = {dev[worst]:.3e}; tensors above 2e-2: {sum(v > 2e-2 for v in dev.values())}")
    assert dev[worst] > 1.5e-2
