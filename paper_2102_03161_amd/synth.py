"""Seeded synthetic workloads: shapes, inputs, labels and initial weights.

This module serves both the HIP path and the CPU checker.  It holds no
arithmetic of the training step itself: only named workload shapes, a
counter-based random generator keyed by (seed, tensor name), and the bf16
round-to-nearest-even helper used to hand both sides identical starting bytes.

The workloads stand in, by shape only, for the datasets the paper trains on
(Sec. 4.1: ImageNet / CIFAR-100 for ViT-B/16 at 224x224, SQuAD for BERT):
inputs are N(0,1) pixels or uniform token ids, weights N(0, 0.02), labels
uniform.  No dataset item is reproduced.
"""
from __future__ import annotations

import zlib

import numpy as np

# Named workloads.  "B" is the training micro-batch of the workload.
WORKLOADS = {
    # tiny ViT, fp32: 2 pre-LN blocks, 32x32x3 images, 8x8 patches -> S = 17
    "vit_tiny": dict(arch="vit", L=2, D=64, H=4, F=256, S=17, n_out=10, img=32, patch=8, chans=3,
                     vocab=0, max_pos=0, ln_eps=1e-6, B=4, dtype="f32", optimizer="sgdm"),
    # tiny BERT, fp32: 2 post-LN blocks
    "bert_tiny": dict(arch="bert", L=2, D=64, H=4, F=256, S=24, n_out=2, img=0, patch=0, chans=0,
                      vocab=97, max_pos=32, ln_eps=1e-12, B=4, dtype="f32", optimizer="adamw"),
    # ViT-B/16: 12 pre-LN blocks, 224x224x3, 16x16 patches -> S = 197
    "vit_b16": dict(arch="vit", L=12, D=768, H=12, F=3072, S=197, n_out=1000, img=224, patch=16, chans=3,
                    vocab=0, max_pos=0, ln_eps=1e-6, B=64, dtype="bf16", optimizer="adamw"),
    "vit_b16_b128": dict(arch="vit", L=12, D=768, H=12, F=3072, S=197, n_out=1000, img=224, patch=16,
                         chans=3, vocab=0, max_pos=0, ln_eps=1e-6, B=128, dtype="bf16", optimizer="adamw"),
    # BERT-base span QA: 12 post-LN blocks, S = 384
    "bert_base_qa": dict(arch="bert", L=12, D=768, H=12, F=3072, S=384, n_out=2, img=0, patch=0, chans=0,
                         vocab=30522, max_pos=512, ln_eps=1e-12, B=32, dtype="bf16", optimizer="adamw"),
    # BERT-large span QA (the paper's SQuAD model, App. A.1 / Sec. 4.1): 24 post-LN blocks, S = 512
    "bert_large_qa": dict(arch="bert", L=24, D=1024, H=16, F=4096, S=512, n_out=2, img=0, patch=0, chans=0,
                          vocab=30522, max_pos=512, ln_eps=1e-12, B=64, dtype="bf16", optimizer="adamw"),
    # BERT-base sequence classification (SST-2-shaped: 2 classes, S = 128)
    "bert_base_cls": dict(arch="bert", L=12, D=768, H=12, F=3072, S=128, n_out=2, img=0, patch=0, chans=0,
                          vocab=30522, max_pos=512, ln_eps=1e-12, B=64, dtype="bf16", optimizer="adamw", head="cls"),
    "bert_tiny_cls": dict(arch="bert", L=2, D=64, H=4, F=256, S=24, n_out=3, img=0, patch=0, chans=0,
                          vocab=97, max_pos=32, ln_eps=1e-12, B=4, dtype="f32", optimizer="adamw", head="cls"),
}

MODEL_KEYS = ("arch", "L", "D", "H", "F", "S", "n_out", "img", "patch", "chans", "vocab", "max_pos", "ln_eps")


def workload(name: str, **overrides) -> dict:
    w = dict(WORKLOADS[name])
    w.update(overrides)
    return w


def model_fields(w: dict) -> dict:
    f = {k: w[k] for k in MODEL_KEYS}
    f["head"] = w.get("head", "default")
    return f


def _rng(seed: int, name: str) -> np.random.Generator:
    # Philox is counter-based: the stream depends only on the key below.
    key = (int(seed) << 32) | (zlib.crc32(name.encode()) & 0xFFFFFFFF)
    return np.random.Generator(np.random.Philox(key=key))


def is_gain(name: str) -> bool:
    return name.endswith("_g")


def gen_param(seed: int, name: str, shape) -> np.ndarray:
    """fp32 initial value of a parameter tensor: N(0, 0.02); LayerNorm gains
    1 + N(0, 0.02) so that every term of the backward pass is exercised."""
    x = _rng(seed, "param:" + name).standard_normal(size=tuple(shape), dtype=np.float32) * np.float32(0.02)
    if is_gain(name):
        x = x + np.float32(1.0)
    return x.astype(np.float32)


def gen_inputs(w: dict, seed: int, B: int | None = None, tag: str = ""):
    """(inputs, labels) for one batch.  ViT: fp32 images [B,C,H,W] ~ N(0,1),
    labels int32 [B] uniform in [0, n_out).  BERT: int32 ids [B,S] uniform in
    [0, vocab), labels int32 [B,2] (start, end) uniform in [0, S), or for the
    classification head int32 [B] uniform in [0, n_out)."""
    B = w["B"] if B is None else B
    r = _rng(seed, "batch:" + tag)
    if w["arch"] == "vit":
        x = r.standard_normal(size=(B, w["chans"], w["img"], w["img"]), dtype=np.float32)
        y = r.integers(0, w["n_out"], size=(B,), dtype=np.int32)
    else:
        x = r.integers(0, w["vocab"], size=(B, w["S"]), dtype=np.int32)
        if w.get("head", "default") == "cls":
            y = r.integers(0, w["n_out"], size=(B,), dtype=np.int32)
        else:
            y = r.integers(0, w["S"], size=(B, 2), dtype=np.int32)
    return x, y


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16-representable fp32 value."""
    return bf16_to_f32(bf16_bits(x)).reshape(np.shape(x))
