"""Drives the HIP library and the oracle from the same seeded inputs (test plumbing)."""
import numpy as np

from oracle import encoder as orc
from paper_2102_03161_amd import binding, synth
from tests.helpers import oracle_cfg, rel_err

def f32_exact(**hp):
    """Hyper-parameters cross the C ABI as fp32: both sides get the fp32-representable values."""
    return {k: float(np.float32(v)) for k, v in hp.items()}


HP = f32_exact(lr=1e-3, momentum=0.9, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def init_values(w, ctx, seed):
    """fp32 initial parameter values by tensor name; bf16 workloads start from bf16-representable masters."""
    vals = {}
    for tid, name, shape, _, _ in ctx.tensors():
        a = synth.gen_param(seed, name, shape)
        vals[name] = synth.round_bf16(a) if w["dtype"] == "bf16" else a
    return vals


def load_params(ctx, vals):
    for tid, name, shape, _, _ in ctx.tensors():
        ctx.write_tensor(tid, binding.KIND_PARAM, vals[name])


def batch_for(w, seed, nb, tag=""):
    x, y = synth.gen_inputs(w, seed, nb, tag)
    if w["arch"] == "vit" and w["dtype"] == "bf16":
        x = synth.round_bf16(x)
    return x, y


def to_dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def gpu_read_all(ctx, kind):
    return {name: ctx.read_tensor(tid, kind) for tid, name, _, _, _ in ctx.tensors()}


def oracle_step(w, vals, x, y, k, hp=HP, state=None, compute_vals=None):
    """One oracle step in fp64.  compute_vals: parameter values the forward/backward reads
    (the bf16-rounded masters in bf16 mode); the update is applied to `vals`."""
    cfg = oracle_cfg(w)
    p = {n: a.astype(np.float64) for n, a in vals.items()}
    pc = p if compute_vals is None else {n: a.astype(np.float64) for n, a in compute_vals.items()}
    xx = x.astype(np.float64) if w["arch"] == "vit" else x
    hk, fs = orc.frozen_forward(cfg, pc, xx, k)
    loss, grads, aux = orc.active_fwd_bwd(cfg, pc, hk, y, k, fs)
    norms = orc.layer_grad_norms(cfg, grads, k)
    st = orc.new_opt_state(p) if state is None else state
    if w["optimizer"] == "adamw":
        orc.adamw_step(cfg, p, grads, st, k, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"])
    else:
        orc.sgdm_step(cfg, p, grads, st, k, hp["lr"], hp["momentum"], hp["weight_decay"])
    return dict(cfg=cfg, hk=hk, loss=loss, grads=grads, norms=norms, aux=aux, params=p, state=st)


def oracle_update(w, o, vals, gpu_grads, k, hp=HP, state=None):
    """Applies the oracle's update rule to gradients read back from the GPU."""
    cfg = o["cfg"]
    p = {n: a.astype(np.float64) for n, a in vals.items()}
    o["params_before"] = {n: a.copy() for n, a in p.items()}
    st = orc.new_opt_state(p) if state is None else state
    g64 = {n: a.astype(np.float64) for n, a in gpu_grads.items()}
    if w["optimizer"] == "adamw":
        orc.adamw_step(cfg, p, g64, st, k, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"])
    else:
        orc.sgdm_step(cfg, p, g64, st, k, hp["lr"], hp["momentum"], hp["weight_decay"])
    o["params_from_gpu_grads"] = p


def first_token_rows_only(w, k):
    """True when the step computes only each sample's first row of the top block's output: the head reads
    nothing else (ViT class token, BERT sequence classification), so an active top block works on those rows
    behind its attention and leaves the other rows of ACT_HL unspecified."""
    return (w["arch"] == "vit" or w.get("head") == "cls") and w["S"] >= 4 and k < w["L"]


def gpu_step(torch, ctx, w, x, y, k, hp=HP, sample_ids=None):
    ctx.set_freeze_boundary(k)
    dx = to_dev(torch, x)
    dy = to_dev(torch, y)
    nb = x.shape[0]
    hk_ptr = ctx.frozen_forward(dx, sample_ids)
    loss = ctx.active_fwd_bwd(hk_ptr, dy)
    S, D = w["S"], w["D"]
    out = dict(loss=loss)
    out["hk"] = ctx.read_activation(binding.ACT_HK, (nb, S, D))
    out["hL"] = ctx.read_activation(binding.ACT_HL, (nb, S, D))
    if first_token_rows_only(w, k):
        out["hL"] = out["hL"][:, :1, :]
    out["logits"] = ctx.read_activation(binding.ACT_LOGITS, (nb, w["n_out"]) if (w["arch"] == "vit" or w.get("head") == "cls") else (nb, S, 2))
    out["norms"] = ctx.layer_grad_norms()
    out["grads"] = gpu_read_all(ctx, binding.KIND_GRAD)
    ctx.optimizer_step(**hp)
    out["params"] = gpu_read_all(ctx, binding.KIND_PARAM)
    torch.cuda.synchronize()
    return out


def exactly_cancelling(w, k):
    """Gradient tensors whose true value is zero by exact cancellation, so that what any implementation
    computes for them is round-off of the summands.  Under the span head the loss of a sample depends on
    the logits only through softmaxes over the sequence axis, whose gradients sum to zero over the tokens:
    the head bias (the sum of dz over the tokens) and the shift of the last post-LN LayerNorm (the sum of
    dL/dh_L = dz W^T over the tokens) vanish identically.  The oracle returns ~1e-18 for them."""
    if w["arch"] == "bert" and w.get("head", "default") != "cls":
        names = {"head.b"}
        if w["L"] - 1 >= k:
            names.add(f"blk{w['L'] - 1}.ln2_b")
        return names
    return set()


def grad_errors(w, got, ref, cfg, k, rss=None):
    """Per-tensor max |a - b| / max |b| over the active gradient tensors.  Frozen tensors must hold exact zeros.
    A tensor whose elements are sums that cancel is measured against the root-sum-square of its summands when
    that is larger than the tensor's own peak (rss: per tensor, from the exact intermediates); without rss only
    the tensors that cancel to exactly zero get a floor (one-hundredth of the model's largest gradient)."""
    errs = {}
    gmax = max(float(np.max(np.abs(a))) for a in ref.values())
    zero = exactly_cancelling(w, k)
    for name, a in got.items():
        if orc.is_active(name, cfg, k):
            r = ref[name]
            peak = float(np.max(np.abs(r)))
            if rss is not None:
                scale = max(peak, float(np.max(rss[name])))
            elif name in zero:
                assert peak < 1e-9 * gmax, (name, peak)      # the oracle agrees that it cancels
                scale = 1e-2 * gmax
            else:
                scale = peak
            errs["grad:" + name] = float(np.max(np.abs(np.asarray(a, dtype=np.float64) - r))) / max(scale, 1e-300)
        else:
            assert not np.any(a), f"frozen tensor {name} has a gradient"
    return errs


def compare_step(w, g, o, k, tol, check_params=True, model=None, rss=None):
    """Per-tensor max-abs error relative to the tensor's largest magnitude, against the exact oracle `o`.
    model (bf16 mode, shapes other than the named workloads at their batch): the bf16 storage model's step; a
    value passes if it is within `tol` of the exact oracle or within `tol` of the model, i.e. if exact
    arithmetic, or exact arithmetic plus the rounding of what bf16 mode stores, explains it."""
    cfg = o["cfg"]
    errs = {}
    errs["loss"] = abs(g["loss"] - o["loss"]) / abs(o["loss"])
    errs["hk"] = rel_err(g["hk"], o["hk"])
    errs["hL"] = rel_err(g["hL"], o["aux"]["h_L"][:, :g["hL"].shape[1], :])
    errs["logits"] = rel_err(g["logits"], o["aux"]["logits"])
    lscale = 1.0
    if rss is not None and "act:logits" in rss:   # logits that cancel: against the root-sum-square of their summands
        peak = float(np.max(np.abs(o["aux"]["logits"])))
        lscale = peak / max(peak, float(np.max(rss["act:logits"])))
        errs["logits"] *= lscale
    errs.update(grad_errors(w, g["grads"], o["grads"], cfg, k, rss))
    if model is not None:
        alt = {"loss": abs(g["loss"] - model["loss"]) / abs(model["loss"]), "hk": rel_err(g["hk"], model["hk"]),
               "hL": rel_err(g["hL"], model["aux"]["h_L"][:, :g["hL"].shape[1], :]),
               "logits": rel_err(g["logits"], model["aux"]["logits"]) * lscale}
        alt.update(grad_errors(w, g["grads"], model["grads"], cfg, k, rss))
        by_model = sorted(n for n in errs if errs[n] > tol and alt[n] <= tol)
        if by_model:
            print(f"  within {tol} of the storage model but not of the exact oracle: "
                  + ", ".join(f"{n} ({errs[n]:.2e} / {alt[n]:.2e})" for n in by_model), flush=True)
        both = sorted(n for n in errs if errs[n] > tol and alt[n] > tol)
        if both:
            print("  outside both: " + ", ".join(f"{n} ({errs[n]:.2e} / {alt[n]:.2e})" for n in both), flush=True)
        errs = {n: min(e, alt[n]) for n, e in errs.items()}
    on = o["norms"]
    for i in range(len(on)):
        if on[i] == 0.0:
            assert g["norms"][i] == 0.0, f"norm slot {i} must be exactly zero"
        else:
            errs[f"norm{i}"] = abs(g["norms"][i] - on[i]) / on[i]
    if check_params:
        # The update is checked on the GPU's own gradients: an Adam step is sign-like
        # (|delta| ~ lr whatever |g| is), so comparing against an update computed from the
        # oracle's gradient would measure sign flips of near-zero gradient elements, not the
        # update rule.  Gradients are compared above; here the rule itself is held to fp32 round-off.
        for name, a in g["params"].items():
            d_ref = o["params_from_gpu_grads"][name] - o["params_before"][name]
            d_got = a.astype(np.float64) - o["params_before"][name]
            lim = 2e-5 * float(np.max(np.abs(d_ref))) + 2e-7 * float(np.max(np.abs(o["params_before"][name])))
            errs["update:" + name] = float(np.max(np.abs(d_got - d_ref))) / max(lim, 1e-300) * tol
    bad = {n: e for n, e in errs.items() if not (e <= tol)}
    assert not bad, f"tolerance {tol} exceeded: {bad}"
    return errs


def storage_model_step(w, vals, x, y, k):
    """The bf16 storage model's step in the shape compare_step takes for the oracle's."""
    from tests import bf16_storage_model as model
    cfg = oracle_cfg(w)
    p = {n: a.astype(np.float64) for n, a in vals.items()}
    xx = x.astype(np.float64) if w["arch"] == "vit" else x
    loss, grads, aux = model.step(cfg, p, xx, y, k)
    return dict(cfg=cfg, hk=aux["h_k"], loss=loss, grads=grads, norms=orc.layer_grad_norms(cfg, grads, k),
                aux={"h_L": aux["h_L"], "logits": aux["logits"]})


def summand_rss(w, vals, x, y, k):
    from tests import bf16_storage_model as model
    p = {n: a.astype(np.float64) for n, a in vals.items()}
    xx = x.astype(np.float64) if w["arch"] == "vit" else x
    return model.summand_rss(oracle_cfg(w), p, xx, y, k)
