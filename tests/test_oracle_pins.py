"""Pins for the CPU oracle: each checks it against something other than itself
(finite differences, closed forms, invariants, brute force, or a library's
textbook routine).  CPU only."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as tF

from oracle import encoder as orc
from paper_2102_03161_amd import synth
from tests.helpers import SMALL_BERT, SMALL_BERT_CLS, SMALL_VIT, oracle_cfg, oracle_params, rel_err

ARCHS = [SMALL_VIT, SMALL_BERT, SMALL_BERT_CLS]
ARCH_IDS = ["vit", "bert", "bert_cls"]


def full_loss(cfg, p, x, y):
    h, fs = orc.frozen_forward(cfg, p, x, 0)
    loss, _, _ = orc.active_fwd_bwd(cfg, p, h, y, 0, fs)
    return loss


def batch(w, seed=7):
    x, y = synth.gen_inputs(w, seed)
    if w["arch"] == "vit":
        x = x.astype(np.float64)
    return x, y


# ---------------------------------------------------------------- finite differences
@pytest.mark.parametrize("w", ARCHS, ids=ARCH_IDS)
@pytest.mark.parametrize("k", [0, 1, 2])
def test_backward_matches_central_differences(w, k):
    cfg, p = oracle_params(w, seed=11, scale=0.4)
    x, y = batch(w)
    h, fs = orc.frozen_forward(cfg, p, x, k)
    loss, grads, aux = orc.active_fwd_bwd(cfg, p, h, y, k, fs)
    rng = np.random.default_rng(3)
    eps = 1e-6

    def loss_at(pp):
        hh, f2 = orc.frozen_forward(cfg, pp, x, k)
        return orc.active_fwd_bwd(cfg, pp, hh, y, k, f2)[0]

    checked = 0
    for name in p:
        if not orc.is_active(name, cfg, k):
            assert name not in grads
            continue
        g = grads[name]
        assert g.shape == p[name].shape
        flat_idx = rng.choice(p[name].size, size=min(5, p[name].size), replace=False)
        if name == "front.E_w":      # make sure rows that occur in the batch are probed
            flat_idx = np.concatenate([flat_idx, np.unique(x)[:3] * cfg.D + 1])
        for fi in flat_idx:
            idx = np.unravel_index(int(fi), p[name].shape)
            q = {n: a for n, a in p.items()}
            q[name] = p[name].copy()
            q[name][idx] += eps
            lp = loss_at(q)
            q[name][idx] -= 2 * eps
            lm = loss_at(q)
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - g[idx]) <= 2e-6 * max(1.0, abs(fd)) + 1e-8, (name, idx, fd, g[idx])
            checked += 1
    assert checked > 40

    # gradient with respect to the boundary activation
    for _ in range(6):
        idx = tuple(rng.integers(0, s) for s in h.shape)
        hp = h.copy(); hp[idx] += eps
        hm = h.copy(); hm[idx] -= eps
        fd = (orc.active_fwd_bwd(cfg, p, hp, y, k, fs)[0] - orc.active_fwd_bwd(cfg, p, hm, y, k, fs)[0]) / (2 * eps)
        assert abs(fd - aux["dh_k"][idx]) <= 2e-6 * max(1.0, abs(fd)) + 1e-8


# ---------------------------------------------------------------- library routine: torch
def torch_model_loss(w, cfg, p, x, y):
    """The same network assembled from PyTorch's own modules (conv2d patch
    embedding, nn.TransformerEncoderLayer, F.layer_norm, F.cross_entropy) with
    autograd for the backward pass."""
    tp = {n: torch.tensor(a, dtype=torch.float64, requires_grad=True) for n, a in p.items()}
    D = cfg.D
    if cfg.arch == "vit":
        img = torch.tensor(x, dtype=torch.float64)
        wconv = tp["front.W_pe"].t().reshape(D, cfg.chans, cfg.patch, cfg.patch)
        e = tF.conv2d(img, wconv, tp["front.b_pe"], stride=cfg.patch).flatten(2).transpose(1, 2)
        h = torch.cat([tp["front.cls"].expand(e.shape[0], 1, D), e], dim=1) + tp["front.pos"]
    else:
        ids = torch.tensor(x, dtype=torch.long)
        emb = tF.embedding(ids, tp["front.E_w"]) + tp["front.E_p"][: cfg.S]
        h = tF.layer_norm(emb, (D,), tp["front.ln_g"], tp["front.ln_b"], cfg.ln_eps)
    for l in range(cfg.L):
        pre = f"blk{l}."
        lay = torch.nn.TransformerEncoderLayer(D, cfg.H, cfg.F, dropout=0.0, activation="gelu",
                                               layer_norm_eps=cfg.ln_eps, batch_first=True,
                                               norm_first=(cfg.arch == "vit"), dtype=torch.float64)
        # functional re-binding so that gradients flow to our leaf tensors
        binds = {
            "self_attn.in_proj_weight": tp[pre + "Wqkv"].t(), "self_attn.in_proj_bias": tp[pre + "bqkv"],
            "self_attn.out_proj.weight": tp[pre + "Wo"].t(), "self_attn.out_proj.bias": tp[pre + "bo"],
            "linear1.weight": tp[pre + "W1"].t(), "linear1.bias": tp[pre + "b1"],
            "linear2.weight": tp[pre + "W2"].t(), "linear2.bias": tp[pre + "b2"],
            "norm1.weight": tp[pre + "ln1_g"], "norm1.bias": tp[pre + "ln1_b"],
            "norm2.weight": tp[pre + "ln2_g"], "norm2.bias": tp[pre + "ln2_b"],
        }
        h = torch.func.functional_call(lay, binds, (h,))
    if cfg.arch == "vit":
        c = tF.layer_norm(h[:, 0], (D,), tp["head.ln_g"], tp["head.ln_b"], cfg.ln_eps)
        z = c @ tp["head.W"] + tp["head.b"]
        loss = tF.cross_entropy(z, torch.tensor(y, dtype=torch.long))
    elif cfg.head == "cls":
        z = h[:, 0] @ tp["head.W"] + tp["head.b"]
        loss = tF.cross_entropy(z, torch.tensor(y, dtype=torch.long))
    else:
        z = h @ tp["head.W"] + tp["head.b"]
        yy = torch.tensor(y, dtype=torch.long)
        loss = 0.5 * (tF.cross_entropy(z[:, :, 0], yy[:, 0]) + tF.cross_entropy(z[:, :, 1], yy[:, 1]))
    loss.backward()
    return float(loss.detach()), {n: t.grad.numpy() for n, t in tp.items()}, z.detach().numpy()


@pytest.mark.parametrize("w", ARCHS + [synth.workload("vit_tiny"), synth.workload("bert_tiny"),
                                       synth.workload("bert_tiny_cls")],
                         ids=["vit_s", "bert_s", "bert_cls_s", "vit_tiny", "bert_tiny", "bert_tiny_cls"])
def test_whole_step_matches_torch_modules(w):
    cfg, p = oracle_params(w, seed=5, scale=0.3)
    x, y = batch(w)
    tl, tg, tz = torch_model_loss(w, cfg, p, x, y)
    h, fs = orc.frozen_forward(cfg, p, x, 0)
    loss, grads, aux = orc.active_fwd_bwd(cfg, p, h, y, 0, fs)
    assert abs(loss - tl) < 1e-12 * max(1, abs(tl))
    assert rel_err(aux["logits"], tz) < 1e-12
    for n in p:
        # absolute floor: some gradients are exactly zero in exact arithmetic (the last
        # post-LN bias under a softmax over the sequence axis) and hold only round-off
        assert np.max(np.abs(grads[n] - tg[n])) <= 1e-10 * np.max(np.abs(tg[n])) + 1e-15, n


def test_patchify_matches_unfold_and_loops():
    w = SMALL_VIT
    cfg = oracle_cfg(w)
    x, _ = batch(w)
    got = orc.patchify(cfg, x)
    ref = tF.unfold(torch.tensor(x), kernel_size=cfg.patch, stride=cfg.patch).transpose(1, 2).numpy()
    assert np.array_equal(got, ref)
    g = cfg.img // cfg.patch
    for b in range(x.shape[0]):
        for gy in range(g):
            for gx in range(g):
                for c in range(cfg.chans):
                    for py in range(cfg.patch):
                        for px in range(cfg.patch):
                            j = (c * cfg.patch + py) * cfg.patch + px
                            assert got[b, gy * g + gx, j] == x[b, c, gy * cfg.patch + py, gx * cfg.patch + px]


# ---------------------------------------------------------------- softmax / attention
def test_attention_brute_force_loops():
    cfg, p = oracle_params(SMALL_VIT, seed=2, scale=0.5)
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, cfg.S, cfg.D))
    a, saved = orc.mhsa_forward(cfg, p, "blk0.", x)
    P = saved[4]
    assert np.allclose(P.sum(-1), 1.0, atol=1e-14)
    D, H = cfg.D, cfg.H
    dh = D // H
    W, bq = p["blk0.Wqkv"], p["blk0.bqkv"]
    for b in range(2):
        ctx = np.zeros((cfg.S, D))
        for hd in range(H):
            cols = slice(hd * dh, (hd + 1) * dh)
            for i in range(cfg.S):
                qi = x[b, i] @ W[:, 0:D][:, cols] + bq[0:D][cols]
                sc = []
                vs = []
                for j in range(cfg.S):
                    kj = x[b, j] @ W[:, D:2 * D][:, cols] + bq[D:2 * D][cols]
                    vs.append(x[b, j] @ W[:, 2 * D:][:, cols] + bq[2 * D:][cols])
                    sc.append(sum(qi[t] * kj[t] for t in range(dh)) / math.sqrt(dh))
                den = sum(math.exp(s) for s in sc)
                for j in range(cfg.S):
                    ctx[i, cols] += math.exp(sc[j]) / den * vs[j]
        ref = ctx @ p["blk0.Wo"] + p["blk0.bo"]
        assert np.allclose(a[b], ref, atol=1e-13)


def test_softmax_shift_invariance_and_uniform_case():
    rng = np.random.default_rng(1)
    s = rng.standard_normal((4, 7))
    assert np.allclose(orc.softmax_lastaxis(s), orc.softmax_lastaxis(s + 123.0), atol=1e-14)
    # zero query/key projections -> uniform attention -> context is the mean of V over the sequence
    cfg, p = oracle_params(SMALL_VIT, seed=2, scale=0.5)
    D = cfg.D
    p["blk0.Wqkv"][:, : 2 * D] = 0
    p["blk0.bqkv"][: 2 * D] = 0
    x = rng.standard_normal((2, cfg.S, D))
    _, saved = orc.mhsa_forward(cfg, p, "blk0.", x)
    v_full = x @ p["blk0.Wqkv"][:, 2 * D:] + p["blk0.bqkv"][2 * D:]
    assert np.allclose(saved[5], np.broadcast_to(v_full.mean(1, keepdims=True), v_full.shape), atol=1e-14)


def test_attention_backward_rows_of_dS_sum_to_zero_and_fd():
    cfg, p = oracle_params(SMALL_VIT, seed=2, scale=0.5)
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, cfg.S, cfg.D))
    da = rng.standard_normal((2, cfg.S, cfg.D))
    grads = {}
    a, saved = orc.mhsa_forward(cfg, p, "blk0.", x)
    dx = orc.mhsa_backward(cfg, p, "blk0.", da, saved, grads)
    # directional derivative of <a, da> along a random direction
    d = rng.standard_normal(x.shape)
    e = 1e-6
    fd = ((orc.mhsa_forward(cfg, p, "blk0.", x + e * d)[0] * da).sum()
          - (orc.mhsa_forward(cfg, p, "blk0.", x - e * d)[0] * da).sum()) / (2 * e)
    assert abs(fd - (dx * d).sum()) < 1e-7 * max(1, abs(fd))


def test_sequence_length_one_reduces_to_value_path():
    w = dict(SMALL_VIT)
    cfg, p = oracle_params(w, seed=9, scale=0.5)
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 1, cfg.D))
    D = cfg.D
    a, _ = orc.mhsa_forward(cfg, p, "blk1.", x)
    ref = (x @ p["blk1.Wqkv"][:, 2 * D:] + p["blk1.bqkv"][2 * D:]) @ p["blk1.Wo"] + p["blk1.bo"]
    assert np.allclose(a, ref, atol=1e-14)


@pytest.mark.parametrize("w", ARCHS, ids=ARCH_IDS)
def test_block_is_permutation_equivariant_over_tokens(w):
    cfg, p = oracle_params(w, seed=9, scale=0.5)
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, cfg.S, cfg.D))
    perm = rng.permutation(cfg.S)
    out, _ = orc.block_forward(cfg, p, 1, x)
    outp, _ = orc.block_forward(cfg, p, 1, x[:, perm])
    assert np.allclose(outp, out[:, perm], atol=1e-13)


# ---------------------------------------------------------------- LayerNorm / GELU
def test_layer_norm_invariants():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((5, 9, 32)) * 3 + 1.5
    eps = 1e-6
    y, saved = orc.layer_norm(x, np.ones(32), np.zeros(32), eps)
    assert np.allclose(y.mean(-1), 0, atol=1e-14)
    var = x.var(-1)
    assert np.allclose(y.var(-1), var / (var + eps), atol=1e-13)
    ref = tF.layer_norm(torch.tensor(x), (32,), eps=eps).numpy()
    assert np.allclose(y, ref, atol=1e-13)
    g = rng.standard_normal(32)
    dy = rng.standard_normal(x.shape)
    dx, dg, db = orc.layer_norm_bwd(dy, saved, g)
    assert np.allclose(dx.sum(-1), 0, atol=1e-12)
    # orthogonality to xhat is exact only for eps = 0 (sum xhat^2 = D var/(var+eps))
    _, saved0 = orc.layer_norm(x, np.ones(32), np.zeros(32), 0.0)
    dx0, _, _ = orc.layer_norm_bwd(dy, saved0, g)
    assert np.allclose((dx0 * saved0[0]).sum(-1), 0, atol=1e-12)
    assert np.allclose(dg, (dy * saved[0]).reshape(-1, 32).sum(0))
    assert np.allclose(db, dy.reshape(-1, 32).sum(0))


def test_gelu_values_identity_and_derivative():
    assert orc.gelu(np.array(0.0)) == 0.0
    # GELU(1) = Phi(1), GELU(-1) = -(1 - Phi(1)); Phi(1) = 0.841344746068543 (normal tables)
    assert abs(orc.gelu(np.array(1.0)) - 0.841344746068543) < 1e-14
    assert abs(orc.gelu(np.array(-1.0)) + 0.158655253931457) < 1e-14
    x = np.linspace(-6, 6, 241)
    assert np.allclose(orc.gelu(x) - orc.gelu(-x), x, atol=1e-14)
    e = 1e-6
    fd = (orc.gelu(x + e) - orc.gelu(x - e)) / (2 * e)
    assert np.allclose(orc.gelu_grad(x), fd, atol=1e-9)
    assert np.allclose(orc.gelu(x), tF.gelu(torch.tensor(x)).numpy(), atol=1e-15)


# ---------------------------------------------------------------- losses
@pytest.mark.parametrize("w,ln_c", [(SMALL_VIT, math.log(3)), (SMALL_BERT, math.log(6)),
                                    (synth.workload("vit_tiny"), 2.302585092994046)],
                         ids=["vit", "bert", "vit_tiny"])
def test_zero_head_gives_log_of_class_count(w, ln_c):
    cfg, p = oracle_params(w, seed=3)
    p["head.W"][:] = 0
    p["head.b"][:] = 0
    x, y = batch(w)
    h, fs = orc.frozen_forward(cfg, p, x, 0)
    loss, grads, aux = orc.active_fwd_bwd(cfg, p, h, y, 0, fs)
    assert abs(loss - ln_c) < 1e-14
    B = x.shape[0]
    if cfg.arch == "vit":
        dz = np.full((B, cfg.n_out), 1.0 / cfg.n_out)
        dz[np.arange(B), y] -= 1
        assert np.allclose(grads["head.b"], dz.sum(0) / B, atol=1e-15)
    else:
        # each logit column: (1/S - onehot) * 0.5 / B summed over tokens and batch = 0
        assert np.allclose(grads["head.b"], 0, atol=1e-15)
    # zero head weight: no gradient reaches the encoder
    assert all(np.all(grads[n] == 0) for n in grads if n.startswith("blk"))


@pytest.mark.parametrize("w", ARCHS, ids=ARCH_IDS)
def test_boundary_at_L_is_softmax_regression(w):
    cfg, p = oracle_params(w, seed=3, scale=0.5)
    x, y = batch(w)
    L = cfg.L
    h, fs = orc.frozen_forward(cfg, p, x, L)
    loss, grads, aux = orc.active_fwd_bwd(cfg, p, h, y, L)
    assert not any(n.startswith("blk") or n.startswith("front") for n in grads)
    B = x.shape[0]
    from scipy.special import softmax as sp_softmax
    if cfg.arch == "vit":
        feats = tF.layer_norm(torch.tensor(h[:, 0]), (cfg.D,), torch.tensor(p["head.ln_g"]),
                              torch.tensor(p["head.ln_b"]), cfg.ln_eps).numpy()
        prob = sp_softmax(feats @ p["head.W"] + p["head.b"], axis=-1)
        onehot = np.eye(cfg.n_out)[y]
        assert np.allclose(grads["head.W"], feats.T @ (prob - onehot) / B, atol=1e-14)
    elif cfg.head == "cls":
        prob = sp_softmax(h[:, 0] @ p["head.W"] + p["head.b"], axis=-1)
        onehot = np.eye(cfg.n_out)[y]
        assert np.allclose(grads["head.W"], h[:, 0].T @ (prob - onehot) / B, atol=1e-14)
        assert np.allclose(grads["head.b"], (prob - onehot).sum(0) / B, atol=1e-14)
    else:
        z = h @ p["head.W"] + p["head.b"]
        prob = sp_softmax(z, axis=1)
        onehot = np.zeros_like(prob)
        onehot[np.arange(B), y[:, 0], 0] = 1
        onehot[np.arange(B), y[:, 1], 1] = 1
        gw = np.einsum("bsd,bsc->dc", h, (prob - onehot) * 0.5 / B)
        assert np.allclose(grads["head.W"], gw, atol=1e-14)


# ---------------------------------------------------------------- freeze semantics
@pytest.mark.parametrize("w", ARCHS, ids=ARCH_IDS)
def test_freezing_is_structural(w):
    cfg, p = oracle_params(w, seed=8, scale=0.3)
    x, y = batch(w)
    h0, fs = orc.frozen_forward(cfg, p, x, 0)
    loss0, g0, _ = orc.active_fwd_bwd(cfg, p, h0, y, 0, fs)
    n0 = orc.layer_grad_norms(cfg, g0, 0)
    for k in range(1, cfg.L + 1):
        hk, fsk = orc.frozen_forward(cfg, p, x, k)
        lossk, gk, _ = orc.active_fwd_bwd(cfg, p, hk, y, k, fsk)
        assert lossk == loss0
        for n in p:
            if orc.is_active(n, cfg, k):
                assert np.array_equal(gk[n], g0[n]), n
            else:
                assert n not in gk
        nk = orc.layer_grad_norms(cfg, gk, k)
        assert np.all(nk[: k + 1] == 0.0)            # front end and blocks below k
        assert np.array_equal(nk[k + 1:], n0[k + 1:])
        # update leaves frozen bytes untouched
        q = {n: a.copy() for n, a in p.items()}
        st = orc.new_opt_state(q)
        orc.drop_frozen_state(cfg, st, k)
        orc.adamw_step(cfg, q, gk, st, k, 1e-3, 0.9, 0.999, 1e-8, 0.01)
        for n in p:
            if orc.is_active(n, cfg, k):
                assert not np.array_equal(q[n], p[n]), n
            else:
                assert np.array_equal(q[n], p[n])
                assert n not in st["m"] and n not in st["v"]


@pytest.mark.parametrize("w", ARCHS, ids=ARCH_IDS)
@pytest.mark.parametrize("k", [0, 1])
def test_micro_batch_accumulation_equals_the_full_batch(w, k):
    """The loss is a mean over samples, so the sample-weighted mean of micro-batch gradients is the
    full-batch gradient (pinned above by central differences), whatever the cut, ragged included."""
    cfg, p = oracle_params(w, seed=5, scale=0.3)
    x, y = batch(w)
    B = x.shape[0]
    hk, fs = orc.frozen_forward(cfg, p, x, k)
    loss, grads, _ = orc.active_fwd_bwd(cfg, p, hk, y, k, fs)
    for sizes in ([B], [1] * B, [B - 1, 1], [2, B - 2]):
        la, ga = orc.accumulated_fwd_bwd(cfg, p, x, y, k, sizes)
        assert abs(la - loss) < 1e-13 * abs(loss)
        assert set(ga) == set(grads)
        for n in grads:
            assert np.allclose(ga[n], grads[n], rtol=0, atol=1e-13 * max(1.0, np.abs(grads[n]).max())), (n, sizes)
    # a planted mistake would show: an unweighted mean of unequal micro-batches is a different vector
    hk1, fs1 = orc.frozen_forward(cfg, p, x[:B - 1], k)
    _, g1, _ = orc.active_fwd_bwd(cfg, p, hk1, y[:B - 1], k, fs1)
    hk2, fs2 = orc.frozen_forward(cfg, p, x[B - 1:], k)
    _, g2, _ = orc.active_fwd_bwd(cfg, p, hk2, y[B - 1:], k, fs2)
    wrong = 0.5 * (g1["head.W"] + g2["head.W"])
    assert np.abs(wrong - grads["head.W"]).max() > 1e-6 * np.abs(grads["head.W"]).max()


def test_grad_norm_slots_add_up_to_global_norm():
    w = SMALL_BERT
    cfg, p = oracle_params(w, seed=8, scale=0.3)
    x, y = batch(w)
    h, fs = orc.frozen_forward(cfg, p, x, 0)
    _, g, _ = orc.active_fwd_bwd(cfg, p, h, y, 0, fs)
    n = orc.layer_grad_norms(cfg, g, 0)
    assert n.shape == (cfg.L + 2,)
    flat = np.concatenate([a.ravel() for a in g.values()])
    assert abs((n ** 2).sum() - np.dot(flat, flat)) < 1e-12 * np.dot(flat, flat)
    blk1 = np.concatenate([g[f"blk1.{t}"].ravel() for t in orc.BLOCK_TENSORS])
    assert abs(n[2] - np.linalg.norm(blk1)) < 1e-14


# ---------------------------------------------------------------- optimizers
def _const_problem():
    cfg, p = oracle_params(SMALL_VIT, seed=1)
    rng = np.random.default_rng(0)
    g = {n: rng.standard_normal(a.shape) for n, a in p.items()}
    return cfg, p, g


def test_sgd_momentum_closed_form_and_torch():
    cfg, p, g = _const_problem()
    q = {n: a.copy() for n, a in p.items()}
    st = orc.new_opt_state(q)
    lr, mu, n_steps = 0.03, 0.9, 7
    for _ in range(n_steps):
        orc.sgdm_step(cfg, q, g, st, 0, lr, mu)
    coef = sum((1 - mu ** i) / (1 - mu) for i in range(1, n_steps + 1))
    for n in p:
        assert np.allclose(st["m"][n], g[n] * (1 - mu ** n_steps) / (1 - mu), atol=1e-13)
        assert np.allclose(q[n], p[n] - lr * coef * g[n], atol=1e-13)
    # varying gradients + weight decay against torch.optim.SGD
    rng = np.random.default_rng(1)
    name = "blk0.W1"
    tw = torch.tensor(p[name].copy(), requires_grad=True)
    opt = torch.optim.SGD([tw], lr=lr, momentum=mu, weight_decay=0.05)
    q = {n: a.copy() for n, a in p.items()}
    st = orc.new_opt_state(q)
    for _ in range(4):
        gg = {n: rng.standard_normal(a.shape) for n, a in p.items()}
        tw.grad = torch.tensor(gg[name])
        opt.step()
        orc.sgdm_step(cfg, q, gg, st, 0, lr, mu, 0.05)
    assert np.allclose(q[name], tw.detach().numpy(), atol=1e-14)
    assert orc.is_decayed(name) and not orc.is_decayed("blk0.b1") and not orc.is_decayed("front.pos")


def test_adamw_closed_forms_and_torch():
    cfg, p, g = _const_problem()
    lr, b1, b2, eps = 1e-3, 0.9, 0.999, 1e-8
    q = {n: a.copy() for n, a in p.items()}
    st = orc.new_opt_state(q)
    prev = {n: a.copy() for n, a in q.items()}
    for _ in range(5):   # constant g, no decay: every step moves by -lr g/(|g|+eps)
        orc.adamw_step(cfg, q, g, st, 0, lr, b1, b2, eps, 0.0)
        for n in p:
            assert np.allclose(q[n] - prev[n], -lr * g[n] / (np.abs(g[n]) + eps), rtol=1e-9, atol=1e-16)
        prev = {n: a.copy() for n, a in q.items()}
    assert st["t"] == 5
    # zero gradient, decay only: geometric shrink of decayed tensors, others fixed
    z = {n: np.zeros_like(a) for n, a in p.items()}
    q = {n: a.copy() for n, a in p.items()}
    st = orc.new_opt_state(q)
    for _ in range(6):
        orc.adamw_step(cfg, q, z, st, 0, lr, b1, b2, eps, 0.3)
    for n in p:
        f = (1 - lr * 0.3) ** 6 if orc.is_decayed(n) else 1.0
        assert np.allclose(q[n], p[n] * f, rtol=1e-13)
    # varying gradients against torch.optim.AdamW
    rng = np.random.default_rng(2)
    name = "blk1.Wo"
    tw = torch.tensor(p[name].copy(), requires_grad=True)
    opt = torch.optim.AdamW([tw], lr=lr, betas=(b1, b2), eps=eps, weight_decay=0.01)
    q = {n: a.copy() for n, a in p.items()}
    st = orc.new_opt_state(q)
    for _ in range(5):
        gg = {n: rng.standard_normal(a.shape) for n, a in p.items()}
        tw.grad = torch.tensor(gg[name])
        opt.step()
        orc.adamw_step(cfg, q, gg, st, 0, lr, b1, b2, eps, 0.01)
    assert np.allclose(q[name], tw.detach().numpy(), rtol=1e-12, atol=1e-15)


# ---------------------------------------------------------------- cache
@pytest.mark.parametrize("w", ARCHS, ids=ARCH_IDS)
def test_cache_hit_advance_and_permutation(w):
    cfg, p = oracle_params(w, seed=8, scale=0.3)
    x, y = batch(w)
    B = x.shape[0]
    ids = [10, 4, 7][:B]
    cache = orc.ActivationCache()
    h1, dec, runs = cache.frozen_forward(cfg, p, x, ids, 1)
    assert [d[0] for d in dec] == ["miss"] * B and runs == B * 1
    fresh1, _ = orc.frozen_forward(cfg, p, x, 1)
    assert np.allclose(h1, fresh1, atol=1e-14)
    h1b, dec, runs = cache.frozen_forward(cfg, p, x, ids, 1)
    assert [d[0] for d in dec] == ["hit"] * B and runs == 0
    assert np.array_equal(h1b, h1)
    # shuffled order returns the same per-sample rows (lookup by id, not position)
    perm = [2, 0, 1][:B]
    hp, dec, runs = cache.frozen_forward(cfg, p, x[perm], [ids[i] for i in perm], 1)
    assert runs == 0 and np.array_equal(hp, h1[perm])
    # boundary moves 1 -> 3: stale rows go through blocks 1, 2 only
    h3, dec, runs = cache.frozen_forward(cfg, p, x, ids, 3)
    assert dec == [("advance", 1)] * B and runs == B * 2
    fresh3, _ = orc.frozen_forward(cfg, p, x, 3)
    assert np.allclose(h3, fresh3, atol=1e-13)
    # a batch mixing a known and an unknown sample
    x2, _ = synth.gen_inputs(w, 99)
    x2 = x2.astype(np.float64) if cfg.arch == "vit" else x2
    mix_x = np.concatenate([x[:1], x2[:1]])
    hm, dec, runs = cache.frozen_forward(cfg, p, mix_x, [ids[0], 55], 3)
    assert [d[0] for d in dec] == ["hit", "miss"] and runs == 3


def test_cache_transition_example_from_the_paper():
    # Sec. 3.4: 3 frozen layers at T1, 4 more at T2 -> entries advance from the
    # output of layer 3 to layer 7 through the 4 newly frozen layers only.
    vals = {}
    with open(__file__.replace("test_oracle_pins.py", "golden/cache_transition.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split("=")
                vals[k.strip()] = int(v)
    w = dict(SMALL_VIT, L=vals["frozen_T2"] + vals["active_T2"])
    cfg, p = oracle_params(w, seed=8, scale=0.3)
    x, _ = batch(w)
    cache = orc.ActivationCache()
    cache.frozen_forward(cfg, p, x[:1], [0], vals["frozen_T1"])
    _, dec, runs = cache.frozen_forward(cfg, p, x[:1], [0], vals["frozen_T2"])
    assert dec == [("advance", vals["frozen_T1"])]
    assert runs == vals["newly_frozen"] == vals["frozen_T2"] - vals["frozen_T1"]


# ---------------------------------------------------------------- Eq. 1
def test_alpha_bound_closed_form():
    for L in (12, 24):
        for alpha in (1 / 5, 1 / 3, 2 / 5, 1 / 2):
            prev = 0.0
            for T in range(1, 12):
                rec = orc.alpha_bound_recursion(L, alpha, T)
                assert abs(rec - orc.alpha_bound_closed_form(L, alpha, T)) < 1e-10
                assert abs(rec - L * (1 - (1 - alpha) ** T)) < 1e-10
                assert prev < rec < L
                prev = rec


def test_next_boundary_rule():
    L = 12
    flat = np.ones(L + 2)
    # all norms equal -> argmin is the lowest active block -> never moves
    assert orc.next_boundary(flat, 0, L, 1 / 3) == 0
    # smallest norm at the top: the alpha bound decides; 4, 6, 8, 9, 10, 10
    n = np.ones(L + 2)
    n[L] = 0.1                       # block L-1
    k, seq = 0, []
    for _ in range(6):
        k = orc.next_boundary(n, k, L, 1 / 3)
        seq.append(k)
    assert seq == [4, 6, 8, 9, 10, 10]
    # smallest norm at block 2: argmin decides
    n = np.ones(L + 2)
    n[1 + 2] = 0.1
    assert orc.next_boundary(n, 0, L, 1 / 2) == 2
    assert orc.next_boundary(n, 5, L, 1 / 2) == 5     # argmin over blocks >= 5 ties -> lowest -> stays
    # front-end and head slots are ignored
    n = np.ones(L + 2); n[0] = 0.0; n[L + 1] = 0.0; n[1 + 3] = 0.5
    assert orc.next_boundary(n, 0, L, 1 / 2) == 3
