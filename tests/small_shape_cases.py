"""Small configurations (widths of 8 to 320, a few tokens to a few thousand) drawn at random through the parity
harness, on which the bf16 step lands further than 2e-2 from the exact oracle on some gradient tensors.
Each entry: (workload fields, boundary k, batch, seed).  Shared by the CPU test that shows where the excess
comes from and the GPU test that holds the library to the bf16 storage model on them."""

CASES = [
    (dict(arch="vit", L=3, D=8, H=1, F=512, S=50, n_out=2, img=28, patch=4, chans=1, vocab=0, max_pos=0,
          ln_eps=1e-6, B=130, optimizer="sgdm", dtype="bf16"), 0, 130, 122),
    (dict(arch="bert", L=2, D=128, H=2, F=160, S=9, n_out=2, img=0, patch=0, chans=0, vocab=11, max_pos=12,
          ln_eps=1e-12, B=2, optimizer="adamw", dtype="bf16", head="cls"), 0, 2, 112),
    (dict(arch="vit", L=3, D=320, H=8, F=64, S=5, n_out=2, img=8, patch=4, chans=3, vocab=0, max_pos=0,
          ln_eps=1e-6, B=33, optimizer="adamw", dtype="bf16"), 0, 33, 130),
    (dict(arch="bert", L=2, D=96, H=4, F=64, S=64, n_out=2, img=0, patch=0, chans=0, vocab=60, max_pos=67,
          ln_eps=1e-12, B=33, optimizer="adamw", dtype="bf16", head="cls"), 0, 33, 106),
    (dict(arch="vit", L=2, D=64, H=2, F=64, S=26, n_out=2, img=20, patch=4, chans=3, vocab=0, max_pos=0,
          ln_eps=1e-6, B=64, optimizer="adamw", dtype="bf16"), 0, 64, 167),
    (dict(arch="bert", L=3, D=256, H=4, F=256, S=77, n_out=2, img=0, patch=0, chans=0, vocab=11, max_pos=80,
          ln_eps=1e-12, B=50, optimizer="adamw", dtype="bf16", head="cls"), 0, 50, 100),
    (dict(arch="vit", L=2, D=48, H=3, F=64, S=10, n_out=2, img=6, patch=2, chans=1, vocab=0, max_pos=0,
          ln_eps=1e-6, B=3, optimizer="sgdm", dtype="bf16"), 0, 3, 143),
    (dict(arch="vit", L=2, D=24, H=3, F=32, S=5, n_out=2, img=4, patch=2, chans=3, vocab=0, max_pos=0,
          ln_eps=1e-6, B=8, optimizer="adamw", dtype="bf16"), 1, 8, 140),
    (dict(arch="bert", L=3, D=2048, H=16, F=1040, S=31, n_out=2, img=0, patch=0, chans=0, vocab=11, max_pos=34,
          ln_eps=1e-12, B=5, optimizer="adamw", dtype="bf16"), 0, 5, 108),
    # two-class logits that nearly cancel (measured against the root-sum-square of their summands)
    (dict(arch="vit", L=2, D=64, H=2, F=100, S=10, n_out=2, img=12, patch=4, chans=1, vocab=0, max_pos=0,
          ln_eps=1e-6, B=130, optimizer="sgdm", dtype="bf16"), 1, 130, 123),
]

# Found by the same search and still outside the bar, by a hair: 52 tokens, one LayerNorm shift gradient whose
# sums cancel to 46 % of their root-sum-square; the storage model is 1.5e-2 from the exact value, the library
# 2.07e-2 from the exact value and 2.09e-2 from the model.  Tracked, not hidden: the GPU test runs it as an
# expected (non-strict) failure.
MARGINAL = [
    (dict(arch="vit", L=3, D=160, H=4, F=32, S=26, n_out=2, img=20, patch=4, chans=1, vocab=0, max_pos=0,
          ln_eps=1e-6, B=2, optimizer="adamw", dtype="bf16"), 0, 2, 102),
]


def case_id(c):
    w, k, nb, seed = c
    return f"{w['arch']}-D{w['D']}-S{w['S']}-B{nb}-k{k}-s{seed}"
