"""GPU tests of the frozen-prefix activation cache (Sec. 3.4, App. D.1 item 2):
integer decisions match the oracle exactly; cached bytes are bit-identical to a
recompute; advancing a stale row equals a fresh forward; lookup is by sample id,
not by batch position."""
import numpy as np
import pytest

from oracle import encoder as orc
from paper_2102_03161_amd import binding, synth
from tests import gpu_harness as H
from tests.helpers import oracle_cfg, rel_err
from tests.test_gpu_parity import MID_BERT, MID_VIT

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


def raw_hk(ctx, w, nb):
    return ctx.read_activation(binding.ACT_HK, (nb, w["S"], w["D"]))


def row_as_f32(w, raw):
    return synth.bf16_to_f32(raw.view(np.uint16)) if w["dtype"] == "bf16" else raw.view(np.float32)


@pytest.mark.parametrize("w", [MID_VIT, MID_BERT, dict(MID_VIT, dtype="f32")], ids=["vit_bf16", "bert_bf16", "vit_f32"])
def test_cache_contract(torch_mod, w):
    torch = torch_mod
    L, S, D = w["L"], w["S"], w["D"]
    nb = w["B"]
    ctx = binding.Context(binding.make_config(w, cache_slots=64))
    vals = H.init_values(w, ctx, 21)
    H.load_params(ctx, vals)
    cfg = oracle_cfg(w)
    p64 = {n: a.astype(np.float64) for n, a in vals.items()}
    ocache = orc.ActivationCache()
    xa, _ = H.batch_for(w, 21, nb, "a")
    xb, _ = H.batch_for(w, 21, nb, "b")
    ids_a = [40 + 2 * i for i in range(nb)]
    ids_b = [3 + i for i in range(nb)]
    dxa, dxb = H.to_dev(torch, xa), H.to_dev(torch, xb)
    o_in = (lambda x: x.astype(np.float64)) if w["arch"] == "vit" else (lambda x: x)

    def decisions(batch_ids, k):
        return [ocache.decision(s, k) for s in batch_ids]

    # ---- k = 1: first epoch misses, second epoch hits ------------------------
    ctx.set_freeze_boundary(1)
    want = decisions(ids_a, 1)
    ctx.frozen_forward(dxa, ids_a)
    h_miss = raw_hk(ctx, w, nb)
    o_h, o_dec, o_runs = ocache.frozen_forward(cfg, p64, o_in(xa), ids_a, 1)
    assert o_dec == want and [d[0] for d in want] == ["miss"] * nb
    st = ctx.cache_stats()
    assert (st["misses"], st["hits"], st["advances"], st["block_runs"]) == (nb, 0, 0, o_runs)
    tol = 2e-2 if w["dtype"] == "bf16" else 1e-4
    assert rel_err(h_miss, o_h) < tol
    # cached bytes == what the forward produced; bypassing the cache gives the same bytes
    for i, sid in enumerate(ids_a):
        raw, kw = ctx.cache_row(sid)
        assert kw == 1 and np.array_equal(row_as_f32(w, raw).reshape(S, D), h_miss[i])
    ctx.frozen_forward(dxa, None)
    assert np.array_equal(raw_hk(ctx, w, nb), h_miss)
    ctx.frozen_forward(dxa, ids_a)
    assert np.array_equal(raw_hk(ctx, w, nb), h_miss)
    st2 = ctx.cache_stats()
    assert st2["hits"] == nb and st2["block_runs"] == st["block_runs"] + nb  # only the bypass call ran blocks
    ocache.frozen_forward(cfg, p64, o_in(xa), ids_a, 1)

    # ---- shuffled order: rows follow their sample id -------------------------
    perm = np.random.default_rng(0).permutation(nb)
    ctx.frozen_forward(H.to_dev(torch, xa[perm]), [ids_a[i] for i in perm])
    assert np.array_equal(raw_hk(ctx, w, nb), h_miss[perm])
    assert ctx.cache_stats()["hits"] == 2 * nb

    # ---- a batch mixing hits and misses, in interleaved positions ------------
    mix_x = np.concatenate([xa[:2], xb[:2], xa[2:3]])
    mix_ids = ids_a[:2] + ids_b[:2] + ids_a[2:3]
    order = [2, 0, 3, 1, 4]
    mix_x, mix_ids = mix_x[order], [mix_ids[i] for i in order]
    want = decisions(mix_ids, 1)
    before = ctx.cache_stats()
    ctx.frozen_forward(H.to_dev(torch, mix_x), mix_ids)
    h_mix = raw_hk(ctx, w, len(mix_ids))
    o_h, o_dec, o_runs = ocache.frozen_forward(cfg, p64, o_in(mix_x), mix_ids, 1)
    assert o_dec == want
    after = ctx.cache_stats()
    assert after["misses"] - before["misses"] == sum(d[0] == "miss" for d in want) == 2
    assert after["hits"] - before["hits"] == 3 and after["block_runs"] - before["block_runs"] == o_runs == 2
    ctx.frozen_forward(H.to_dev(torch, mix_x), None)
    assert np.array_equal(raw_hk(ctx, w, len(mix_ids)), h_mix)   # mixed path == plain recompute, bit for bit

    # ---- boundary moves 1 -> L: stale rows advance through blocks 1..L-1 only --
    ctx.set_freeze_boundary(L)
    want = decisions(ids_a, L)
    assert [d for d in want] == [("advance", 1)] * nb
    before = ctx.cache_stats()
    ctx.frozen_forward(dxa, ids_a)
    h_adv = raw_hk(ctx, w, nb)
    o_h, o_dec, o_runs = ocache.frozen_forward(cfg, p64, o_in(xa), ids_a, L)
    after = ctx.cache_stats()
    assert after["advances"] - before["advances"] == nb and after["block_runs"] - before["block_runs"] == o_runs == nb * (L - 1)
    ctx.frozen_forward(dxa, None)
    assert np.array_equal(raw_hk(ctx, w, nb), h_adv)             # advance == fresh forward through 0..L-1
    assert rel_err(h_adv, o_h) < tol
    # a batch with a hit (written at L), a stale row (written at 1) and a miss
    tri_x = np.concatenate([xb[1:2], xa[:1], xb[4:5]])
    tri_ids = [ids_b[1], ids_a[0], ids_b[4]]
    want = decisions(tri_ids, L)
    assert [d[0] for d in want] == ["advance", "hit", "miss"]
    before = ctx.cache_stats()
    ctx.frozen_forward(H.to_dev(torch, tri_x), tri_ids)
    h_tri = raw_hk(ctx, w, 3)
    o_h, o_dec, o_runs = ocache.frozen_forward(cfg, p64, o_in(tri_x), tri_ids, L)
    after = ctx.cache_stats()
    assert o_dec == want and after["block_runs"] - before["block_runs"] == o_runs == (L - 1) + L
    ctx.frozen_forward(H.to_dev(torch, tri_x), None)
    assert np.array_equal(raw_hk(ctx, w, 3), h_tri)
    for sid in tri_ids:
        assert ctx.cache_row(sid)[1] == L
    ctx.close()


def test_training_from_cache_equals_training_from_recompute(torch_mod):
    """A step whose boundary activation came from the cache gives the same gradients,
    bit for bit, as one that recomputed the frozen prefix."""
    torch = torch_mod
    w = MID_VIT
    nb = w["B"]
    res = []
    for use_cache in (False, True):
        ctx = binding.Context(binding.make_config(w, cache_slots=16))
        vals = H.init_values(w, ctx, 23)
        H.load_params(ctx, vals)
        x, y = H.batch_for(w, 23, nb)
        ids = list(range(nb))
        ctx.set_freeze_boundary(2)
        if use_cache:
            ctx.frozen_forward(H.to_dev(torch, x), ids)     # warm the cache
        res.append(H.gpu_step(torch, ctx, w, x, y, 2, sample_ids=ids if use_cache else None))
        if use_cache:
            assert ctx.cache_stats()["hits"] == nb
        ctx.close()
    a, b = res
    assert a["loss"] == b["loss"]
    for n in a["grads"]:
        assert np.array_equal(a["grads"][n], b["grads"][n]), n


@pytest.mark.parametrize("w", [MID_VIT, MID_BERT], ids=["vit_bf16", "bert_bf16"])
def test_host_tier_is_invisible_to_the_result(torch_mod, w):
    """A context whose cache is mostly in pinned host memory (ids >= cache_slots pass through a window of
    2 B device rows) against an all-HBM context and the oracle's cache on the same call sequence: the same
    decisions, bit-identical h_k and cached rows, with and without prefetching, across boundary moves."""
    torch = torch_mod
    S, D = w["S"], w["D"]
    nb = 4
    n_ids = 16
    tiered = binding.Context(binding.make_config(w, B=nb, cache_slots=3, host_slots=n_ids - 3, window_slots=2 * nb))
    plain = binding.Context(binding.make_config(w, B=nb, cache_slots=n_ids))
    vals = H.init_values(w, plain, 23)
    H.load_params(plain, vals)
    H.load_params(tiered, vals)
    cfg = oracle_cfg(w)
    p64 = {n: a.astype(np.float64) for n, a in vals.items()}
    ocache = orc.ActivationCache()
    xs, _ = H.batch_for(w, 23, n_ids, "pool")
    o_in = (lambda x: x.astype(np.float64)) if w["arch"] == "vit" else (lambda x: x)
    rng = np.random.default_rng(5)
    tally = {"hit": 0, "advance": 0, "miss": 0}

    def call(ids, k, prefetch_next=None):
        ids = [int(i) for i in ids]
        print(f"host tier call k={k} ids={ids}", flush=True)
        want = [ocache.decision(s, k) for s in ids]
        for d in want:
            tally[d[0]] += 1
        dx = H.to_dev(torch, xs[ids])
        tiered.frozen_forward(dx, ids)
        if prefetch_next is not None:
            tiered.cache_prefetch(prefetch_next)
        a = raw_hk(tiered, w, len(ids))
        plain.frozen_forward(dx, ids)
        b = raw_hk(plain, w, len(ids))
        assert np.array_equal(a, b)
        ocache.frozen_forward(cfg, p64, o_in(xs[ids]), ids, k)
        return want

    for c in (tiered, plain):
        c.set_freeze_boundary(1)
    order = rng.permutation(n_ids)
    batches = [order[i:i + nb] for i in range(0, n_ids, nb)]
    for i, ids in enumerate(batches):                       # epoch 1: misses, written through the window
        assert [d[0] for d in call(ids, 1)] == ["miss"] * nb
    assert tiered.cache_stats() == plain.cache_stats()
    for i, ids in enumerate(batches):                       # epoch 2: hits; the next batch is prefetched
        nxt = batches[i + 1] if i + 1 < len(batches) else None
        assert [d[0] for d in call(ids, 1, prefetch_next=nxt)] == ["hit"] * nb
    hs = tiered.host_tier_stats()
    assert hs["rows_to_host"] == n_ids - 3 and hs["prefetched"] > 0 and hs["prefetched_used"] == hs["prefetched"]
    for c in (tiered, plain):
        c.set_freeze_boundary(2)
    order2 = rng.permutation(n_ids)
    for i in range(0, n_ids - nb, nb):                      # epoch 3: advances (stale rows), no prefetch
        assert [d[0] for d in call(order2[i:i + nb], 2)] == ["advance"] * nb
    mixed = list(order2[n_ids - nb:n_ids - 2]) + list(order2[:2])   # two stale rows, two current ones
    got = call(mixed, 2, prefetch_next=order2[:nb])
    assert [d[0] for d in got] == ["advance", "advance", "hit", "hit"]
    call(order2[:nb], 2)                                    # prefetched hits again
    got = call(list(order2[n_ids - 2:]) + list(order2[4:6]), 2)
    assert [d[0] for d in got] == ["advance", "advance", "hit", "hit"]
    assert tiered.cache_stats() == plain.cache_stats()
    st = tiered.cache_stats()
    assert (st["hits"], st["advances"], st["misses"]) == (tally["hit"], tally["advance"], tally["miss"])
    for sid in range(n_ids):                                # every row, whichever tier holds it
        ra, ka = tiered.cache_row(sid)
        rb, kb = plain.cache_row(sid)
        assert ka == kb == 2 and np.array_equal(ra, rb), sid
    # the host tier moved rows both ways and the ids outside both tiers are refused
    hs = tiered.host_tier_stats()
    assert hs["rows_to_device"] > 0 and hs["rows_to_host"] >= 2 * (n_ids - 3)
    with pytest.raises(binding.PtError):
        tiered.frozen_forward(H.to_dev(torch, xs[:nb]), [0, 1, 2, n_ids])
    with pytest.raises(binding.PtError):
        tiered.cache_prefetch([n_ids])
    # prefetch is best effort: ids of the HBM tier need nothing, and the window (2 B rows) bounds the rest
    assert tiered.cache_prefetch([0, 1, 2]) == 0
    assert tiered.cache_prefetch(list(range(3, n_ids))) == 2 * nb
    assert tiered.cache_prefetch(list(range(3, n_ids))) == 0           # already staged / window full
    call(list(range(3, 3 + nb)), 2)                                     # staged rows are used ...
    call(list(range(n_ids - nb, n_ids)), 2)                             # ... and unstaged ones are fetched on demand
    assert tiered.cache_stats() == plain.cache_stats()
    tiered.close()
    plain.close()
    # a context without a host tier has nothing to prefetch; one configured for it refuses to run unattached
    plain = binding.Context(binding.make_config(w, B=nb, cache_slots=4))
    assert plain.cache_prefetch([0, 1]) == 0
    plain.close()


def test_cache_timing_profiler(torch_mod):
    """pt_time_frozen_forward: counts what it ran, leaves the batch's h_k in place, and refuses contexts with
    nothing to time."""
    torch = torch_mod
    w = MID_VIT
    nb, k, reps = w["B"], 2, 3
    ctx = binding.Context(binding.make_config(w, cache_slots=32))
    H.load_params(ctx, H.init_values(w, ctx, 29))
    x, _ = H.batch_for(w, 29, nb)
    dx = H.to_dev(torch, x)
    ids = list(range(5, 5 + nb))
    with pytest.raises(binding.PtError):          # k = 0: no prefix
        ctx.time_frozen_forward(dx, ids, reps)
    ctx.set_freeze_boundary(k)
    ms_re, ms_hit = ctx.time_frozen_forward(dx, ids, reps)
    assert ms_re > 0 and ms_hit > 0
    st = ctx.cache_stats()
    assert (st["misses"], st["hits"], st["advances"]) == (nb, reps * nb, 0)
    assert st["block_runs"] == (1 + reps) * nb * k
    h_after = raw_hk(ctx, w, nb)
    ctx.frozen_forward(dx, None)
    assert np.array_equal(raw_hk(ctx, w, nb), h_after)
    ctx.close()
    plain = binding.Context(binding.make_config(w))
    plain.set_freeze_boundary(1)
    with pytest.raises(binding.PtError):          # no cache configured
        plain.time_frozen_forward(dx, ids, reps)
    plain.close()
