"""Shared test plumbing: build oracle configs / parameters from the seeded
generators.  Holds none of the method's arithmetic."""
import numpy as np

from oracle import encoder as orc
from paper_2102_03161_amd import synth


def oracle_cfg(w):
    return orc.Config(**synth.model_fields(w))


def oracle_params(w, seed, dtype=np.float64, bf16=False, scale=None):
    cfg = oracle_cfg(w)
    p = {}
    for name, shape in orc.param_shapes(cfg).items():
        a = synth.gen_param(seed, name, shape)
        if scale is not None and not synth.is_gain(name):
            a = a * np.float32(scale / 0.02)
        if bf16:
            a = synth.round_bf16(a)
        p[name] = a.astype(dtype)
    return cfg, p


def rel_err(a, b):
    """max |a-b| / max(max |b|, tiny): the per-tensor error metric."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.max(np.abs(a - b)) / max(float(np.max(np.abs(b))), 1e-30)) if b.size else 0.0


SMALL_VIT = dict(arch="vit", L=3, D=16, H=2, F=40, S=5, n_out=3, img=4, patch=2, chans=2,
                 vocab=0, max_pos=0, ln_eps=1e-6, B=3, dtype="f32", optimizer="sgdm")
SMALL_BERT = dict(arch="bert", L=3, D=16, H=2, F=40, S=6, n_out=2, img=0, patch=0, chans=0,
                  vocab=11, max_pos=8, ln_eps=1e-12, B=3, dtype="f32", optimizer="adamw")
SMALL_BERT_CLS = dict(SMALL_BERT, n_out=4, head="cls")
