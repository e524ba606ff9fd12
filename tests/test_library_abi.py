"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host-only entry points behave."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import encoder as orc
from paper_2102_03161_amd import binding, synth
from tests.helpers import oracle_cfg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pt_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = declared_symbols()
    assert len(names) >= 20 and "pt_frozen_forward" in names and "pt_last_error" in names
    for n in names:
        assert hasattr(lib, n), n
    # ... and nothing else: helpers, kernels' host stubs and tuning hooks stay inside the library
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", binding.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = sorted(line.split()[-1] for line in out.splitlines() if line.strip())
    assert exported == names, sorted(set(exported) ^ set(names))


@pytest.mark.parametrize("name", list(synth.WORKLOADS))
def test_arena_sizes_and_parameter_count(name):
    w = synth.workload(name)
    cfg = binding.make_config(w, cache_slots=16)
    params, state, work, cache = binding.query_arena_bytes(cfg)
    n_params = sum(int(np.prod(s)) for s in orc.param_shapes(oracle_cfg(w)).values())
    esz = 2 if w["dtype"] == "bf16" else 4
    # masters (+ bf16 shadows) cover the parameters with less than 2% padding on the real models
    assert params >= n_params * (4 + (2 if esz == 2 else 0))
    if n_params > 10_000_000:
        assert params <= 1.02 * n_params * 6
    assert state >= n_params * 4 * (3 if w["optimizer"] == "adamw" else 2)
    assert cache == 16 * w["S"] * w["D"] * esz
    assert work > w["B"] * w["S"] * w["D"] * esz * (w["L"] + 1)
    if name == "vit_b16":
        assert n_params == 86_567_656


def test_bad_configurations_are_rejected():
    lib = binding.load_library()
    for field, value in [("H", 5), ("S", 198), ("L", 0), ("dtype", 7), ("cache_slots", -1), ("patch", 15)]:
        cfg = binding.make_config(synth.workload("vit_b16"))
        setattr(cfg, field, value)
        with pytest.raises(binding.PtError) as e:
            binding.query_arena_bytes(cfg)
        assert e.value.status == binding.PT_EINVAL
    cfg = binding.make_config(synth.workload("bert_base_qa"))
    cfg.max_pos = 100
    with pytest.raises(binding.PtError):
        binding.query_arena_bytes(cfg)
    z = ctypes.c_size_t()
    assert lib.pt_query_arena_bytes(None, z, z, z, z) == binding.PT_EINVAL


def test_next_boundary_matches_the_rule_on_random_norms():
    rng = np.random.default_rng(0)
    for L in (2, 12, 24):
        for alpha in (0.2, 1 / 3, 0.4, 0.5):
            for _ in range(40):
                norms = rng.random(L + 2).astype(np.float32)
                k_prev = int(rng.integers(0, L + 1))
                assert binding.next_boundary(norms, L, k_prev, alpha) == orc.next_boundary(norms, k_prev, L, alpha)
    n = np.ones(14, dtype=np.float32)
    n[12] = 0.1
    k, seq = 0, []
    for _ in range(6):
        k = binding.next_boundary(n, 12, k, 1 / 3)
        seq.append(k)
    assert seq == [4, 6, 8, 9, 10, 10]
    # decimal fractions whose product with the layer count is an integer: the bound is that integer (exact
    # rational arithmetic), not one less as it would be with alpha narrowed to single precision
    from fractions import Fraction
    flat = np.ones(34, dtype=np.float32)
    flat[-2] = 0.5                      # argmin at the top block: the bound decides
    for a_txt in ("0.7", "0.9", "0.3", "0.6", "0.1"):
        for L in (10, 20, 30):
            for k_prev in (0, 10):
                if k_prev >= L:
                    continue
                nn = np.ones(L + 2, dtype=np.float32)
                nn[L] = 0.5
                want = int(k_prev + Fraction(a_txt) * (L - k_prev))
                assert binding.next_boundary(nn, L, k_prev, float(a_txt)) == want, (a_txt, L, k_prev)
                assert orc.next_boundary(nn, k_prev, L, float(a_txt)) == want, (a_txt, L, k_prev)
    with pytest.raises(binding.PtError):
        binding.next_boundary(n, 12, 13, 0.5)
    with pytest.raises(binding.PtError):
        binding.next_boundary(n, 12, 0, 1.0)


def test_bf16_rounding_helper_is_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1e-40], dtype=np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    r = synth.round_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 and r[2] == np.float32(1.015625) and r[3] == -2.5
    import torch
    t = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, t)
    y = np.random.default_rng(1).standard_normal(10000).astype(np.float32)
    assert np.array_equal(synth.round_bf16(y), torch.tensor(y).to(torch.bfloat16).to(torch.float32).numpy())


def test_host_tier_accumulator_and_head_configuration():
    w = synth.workload("vit_b16")
    base = binding.query_arena_bytes(binding.make_config(w, cache_slots=16))
    row = w["S"] * w["D"] * 2
    # the window rows of a host tier are the last rows of the cache arena
    tiered = binding.query_arena_bytes(binding.make_config(w, cache_slots=16, host_slots=100, window_slots=2 * w["B"]))
    assert tiered[3] == (16 + 2 * w["B"]) * row and tiered[:3] == base[:3]
    # an accumulator adds one gradient-sized buffer to the state arena
    acc = binding.query_arena_bytes(binding.make_config(w, cache_slots=16, grad_accum=True))
    assert acc[1] * 3 == base[1] * 4 and acc[0] == base[0] and acc[2] == base[2]
    for kw in (dict(host_slots=10, window_slots=2 * w["B"] - 1), dict(host_slots=0, window_slots=8),
               dict(host_slots=-1, window_slots=0)):
        with pytest.raises(binding.PtError) as e:
            binding.query_arena_bytes(binding.make_config(w, cache_slots=16, **kw))
        assert e.value.status == binding.PT_EINVAL
    # heads: a BERT span head has two outputs, the classification head any number; unknown heads are refused
    b = synth.workload("bert_base_qa")
    cfg = binding.make_config(b)
    cfg.n_out = 3
    with pytest.raises(binding.PtError):
        binding.query_arena_bytes(cfg)
    cfg.head = binding.PT_HEAD_CLS
    binding.query_arena_bytes(cfg)
    cfg.head = 9
    with pytest.raises(binding.PtError):
        binding.query_arena_bytes(cfg)


def test_a_frozen_block_costs_a_fraction_of_an_active_one():
    """Sec. 3.2.1 item 2: a frozen layer keeps no backward activation maps, gradients or optimizer state.  A context
    created with k_min frozen blocks plans none of them: per block the state arena shrinks by the gradient and
    the two moments (12 bytes per parameter) and the work arena by the block's saved tensors, so that what a
    frozen block still occupies (its fp32 master and bf16 shadow) is well under a sixth of an active block."""
    w = synth.workload("vit_b16")
    block_params = 7_087_872
    sizes = {k: binding.query_arena_bytes(binding.make_config(w, k_min=k)) for k in range(w["L"] + 1)}
    for k in range(1, w["L"] + 1):
        assert sizes[k][0] == sizes[0][0]                                   # parameters stay
        assert sizes[k][1] < sizes[k - 1][1] and sizes[k][2] <= sizes[k - 1][2]
    for k in range(2, w["L"]):                                              # (k = 1 also drops the front end's state)
        d_state = sizes[k - 1][1] - sizes[k][1]
        d_work = sizes[k - 1][2] - sizes[k][2]
        assert abs(d_state - 12 * block_params) <= 12 * 12 * 1024           # padding of 12 tensors to 1024 values
        assert d_work >= 14 * w["B"] * w["S"] * w["D"] * 2                  # the saved activations of a block
        frozen = 6 * block_params
        active = frozen + d_state + d_work
        assert frozen / active < 1 / 6
    with pytest.raises(binding.PtError):
        binding.query_arena_bytes(binding.make_config(w, k_min=w["L"] + 1))


def test_sequences_too_long_for_the_lds_resident_attention_kernels_are_rejected_up_front():
    """Without matrix-core attention (fp32 mode, or a head size other than 64) a strip of score rows over the
    whole sequence lives in LDS, and the first-token kernels keep one score row: configurations that would not
    fit the 160 KB of a CU are refused by pt_query_arena_bytes / pt_create, before anything is enqueued."""
    base = dict(synth.workload("bert_base_qa"), max_pos=1 << 20, vocab=100)
    ok = binding.make_config(dict(base, dtype="f32", S=1024, B=1))
    binding.query_arena_bytes(ok)
    for bad in (dict(base, dtype="f32", S=1536, B=1),                    # fp32: generic kernels
                dict(base, dtype="bf16", S=1536, B=1, H=24),             # bf16 with head size 32
                dict(base, dtype="bf16", S=60000, B=1, head="cls", n_out=2)):   # first-token kernels
        with pytest.raises(binding.PtError) as e:
            binding.query_arena_bytes(binding.make_config(bad))
        assert e.value.status == binding.PT_EINVAL
    # the matrix-core path streams keys through LDS: long sequences are fine there
    binding.query_arena_bytes(binding.make_config(dict(base, dtype="bf16", S=4096, B=1)))
