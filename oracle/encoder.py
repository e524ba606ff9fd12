"""Plain numpy oracle of one training step of a Transformer encoder split at a
freeze boundary k (TEST INFRASTRUCTURE, not the product path).

What it follows in the paper (PipeTransformer, arXiv 2102.03161):

* Sec. 2.1 "Training task and model definition": the model is the composition
  F = f_0 o ... o f_{L-1} of L layers, each with its own parameter set.
* App. A.1: the layers are Transformer encoder blocks; ViT places LayerNorm
  before each sub-layer (pre-LN), BERT after the residual add (post-LN).  ViT
  splits the image into fixed-size patches, embeds them linearly and adds
  position embeddings; BERT adds token and position embeddings.
* Sec. 3.2.1 item 2: a frozen layer keeps no backward activation maps, no
  gradients and no optimizer state; the frozen layers form their own
  forward-only model F_frozen, the rest is F_pipe.
* Sec. 3.1, Eq. 1: the freeze rule reads the norm of every layer's gradient.
* Sec. 3.3 / App. D.2: the optimizer (and data parallelism) is built over
  F_pipe only, so frozen parameters are never updated.
* Sec. 3.4 / App. D.1 item 2: the output of the last frozen layer is cached per
  sample under a unique sample id; after the boundary moves, a stale entry is
  advanced through the newly frozen layers only and then overwritten.

Freezing is exact: the step at boundary k is the ordinary forward, backward and
update of the whole network with the derivatives of layers below k simply not
evaluated.  So this file is that definition written out in numpy, in whatever
floating type the caller's arrays have (fp64 in the parity tests and in the
timed CPU baseline).  The paper delegates the block arithmetic to the ViT and BERT
papers; the choices it leaves open (exact-erf GELU, no dropout, no attention
mask, biased LayerNorm variance, mean-of-two cross-entropies for span QA,
final LayerNorm before the ViT classifier, front end trained iff k == 0) are
spelled out where they are used.

Layout conventions (the oracle's own): activations [B, S, D]; every linear map
is y = x @ W + b with W of shape [in, out]; the packed QKV weight has columns
[Q | K | V] and head h owns columns h*dh .. (h+1)*dh-1 of each third.

Parity pins: tests/test_oracle_*.py (finite differences, closed forms,
invariants, brute force).  No function here is "parity unpinned".
"""
from __future__ import annotations

import math
from collections import OrderedDict
from dataclasses import dataclass

import numpy as np
from scipy.special import erf


# --------------------------------------------------------------------------
# configuration and parameter inventory
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Config:
    arch: str            # "vit" (pre-LN) or "bert" (post-LN); App. A.1
    L: int               # number of encoder blocks (layers f_0 .. f_{L-1})
    D: int               # hidden size
    H: int               # attention heads
    F: int               # MLP width
    S: int               # sequence length (ViT: patches + 1 CLS token)
    n_out: int           # classes (ViT) or 2 (BERT span QA: start / end logit)
    img: int = 0         # ViT: square image side
    patch: int = 0       # ViT: square patch side
    chans: int = 0       # ViT: image channels
    vocab: int = 0       # BERT: vocabulary size
    max_pos: int = 0     # BERT: rows of the learned position table (>= S)
    ln_eps: float = 1e-6
    head: str = "default"  # "default": ViT classifier / BERT span QA; "cls": BERT sequence classification


BLOCK_TENSORS = ("ln1_g", "ln1_b", "Wqkv", "bqkv", "Wo", "bo",
                 "ln2_g", "ln2_b", "W1", "b1", "W2", "b2")


def param_shapes(cfg: Config) -> "OrderedDict[str, tuple]":
    """Name -> shape of every parameter tensor, front end first, head last."""
    D, F = cfg.D, cfg.F
    sh: "OrderedDict[str, tuple]" = OrderedDict()
    if cfg.arch == "vit":
        n_patch = (cfg.img // cfg.patch) ** 2
        assert n_patch + 1 == cfg.S
        sh["front.W_pe"] = (cfg.chans * cfg.patch * cfg.patch, D)
        sh["front.b_pe"] = (D,)
        sh["front.cls"] = (D,)
        sh["front.pos"] = (cfg.S, D)
    else:
        sh["front.E_w"] = (cfg.vocab, D)
        sh["front.E_p"] = (cfg.max_pos, D)
        sh["front.ln_g"] = (D,)
        sh["front.ln_b"] = (D,)
    for l in range(cfg.L):
        pre = f"blk{l}."
        sh[pre + "ln1_g"] = (D,)
        sh[pre + "ln1_b"] = (D,)
        sh[pre + "Wqkv"] = (D, 3 * D)
        sh[pre + "bqkv"] = (3 * D,)
        sh[pre + "Wo"] = (D, D)
        sh[pre + "bo"] = (D,)
        sh[pre + "ln2_g"] = (D,)
        sh[pre + "ln2_b"] = (D,)
        sh[pre + "W1"] = (D, F)
        sh[pre + "b1"] = (F,)
        sh[pre + "W2"] = (F, D)
        sh[pre + "b2"] = (D,)
    if cfg.arch == "vit":
        sh["head.ln_g"] = (D,)
        sh["head.ln_b"] = (D,)
    sh["head.W"] = (D, cfg.n_out)
    sh["head.b"] = (cfg.n_out,)
    return sh


def group_of(name: str, cfg: Config) -> int:
    """Gradient-norm slot of a tensor: 0 = front end, 1+l = block l, L+1 = head."""
    if name.startswith("front."):
        return 0
    if name.startswith("head."):
        return cfg.L + 1
    return 1 + int(name[3:name.index(".")])


def is_active(name: str, cfg: Config, k: int) -> bool:
    """A tensor is trained iff its layer is not below the boundary.  The front
    end belongs to the prefix (no gradient can reach it once block 0 is
    frozen, Sec. 3.2.1), so it is trained iff k == 0; the head always is."""
    g = group_of(name, cfg)
    if g == 0:
        return k == 0
    if g == cfg.L + 1:
        return True
    return (g - 1) >= k


def is_decayed(name: str) -> bool:
    """Weight decay applies to matrices and the token table; not to biases,
    LayerNorm parameters, the CLS token or position embeddings."""
    leaf = name.split(".", 1)[1]
    return leaf in ("W_pe", "E_w", "Wqkv", "Wo", "W1", "W2", "W")


# --------------------------------------------------------------------------
# elementary operations
# --------------------------------------------------------------------------
def layer_norm(x, g, b, eps):
    """LN(x) = g * (x - mean) / sqrt(var + eps) + b, biased variance over D."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    return xhat * g + b, (xhat, rstd)


def layer_norm_bwd(dy, saved, g):
    xhat, rstd = saved
    red = tuple(range(dy.ndim - 1))
    dg = (dy * xhat).sum(axis=red)
    db = dy.sum(axis=red)
    dxhat = dy * g
    m1 = dxhat.mean(axis=-1, keepdims=True)
    m2 = (dxhat * xhat).mean(axis=-1, keepdims=True)
    dx = (dxhat - m1 - xhat * m2) * rstd
    return dx, dg, db


def gelu(h):
    """Exact GELU: h * Phi(h) with the Gaussian CDF Phi."""
    return 0.5 * h * (1.0 + erf(h / math.sqrt(2.0)))


def gelu_grad(h):
    """d/dh [h Phi(h)] = Phi(h) + h phi(h)."""
    cdf = 0.5 * (1.0 + erf(h / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * h * h) / math.sqrt(2.0 * math.pi)
    return cdf + h * pdf


def softmax_lastaxis(s):
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=-1, keepdims=True)


def _split_heads(t, H):
    B, S, D = t.shape
    return t.reshape(B, S, H, D // H).transpose(0, 2, 1, 3)


def _merge_heads(t):
    B, H, S, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(B, S, H * dh)


# --------------------------------------------------------------------------
# sub-layers: multi-head self-attention and MLP (no mask, no dropout)
# --------------------------------------------------------------------------
def mhsa_forward(cfg, p, pre, xin):
    D = cfg.D
    dh = D // cfg.H
    qkv = xin @ p[pre + "Wqkv"] + p[pre + "bqkv"]
    q = _split_heads(qkv[..., 0:D], cfg.H)
    k = _split_heads(qkv[..., D:2 * D], cfg.H)
    v = _split_heads(qkv[..., 2 * D:3 * D], cfg.H)
    P = softmax_lastaxis((q @ k.transpose(0, 1, 3, 2)) / math.sqrt(dh))
    c = _merge_heads(P @ v)
    a = c @ p[pre + "Wo"] + p[pre + "bo"]
    return a, (xin, q, k, v, P, c)


def mhsa_backward(cfg, p, pre, da, saved, grads):
    xin, q, k, v, P, c = saved
    D = cfg.D
    dh = D // cfg.H
    grads[pre + "Wo"] = c.reshape(-1, D).T @ da.reshape(-1, D)
    grads[pre + "bo"] = da.sum(axis=(0, 1))
    dc = _split_heads(da @ p[pre + "Wo"].T, cfg.H)
    dv = P.transpose(0, 1, 3, 2) @ dc
    dP = dc @ v.transpose(0, 1, 3, 2)
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    dq = (dS @ k) / math.sqrt(dh)
    dk = (dS.transpose(0, 1, 3, 2) @ q) / math.sqrt(dh)
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)
    grads[pre + "Wqkv"] = xin.reshape(-1, D).T @ dqkv.reshape(-1, 3 * D)
    grads[pre + "bqkv"] = dqkv.sum(axis=(0, 1))
    return dqkv @ p[pre + "Wqkv"].T


def mlp_forward(cfg, p, pre, xin):
    h = xin @ p[pre + "W1"] + p[pre + "b1"]
    g = gelu(h)
    return g @ p[pre + "W2"] + p[pre + "b2"], (xin, h, g)


def mlp_backward(cfg, p, pre, dout, saved, grads):
    xin, h, g = saved
    D, F = cfg.D, cfg.F
    grads[pre + "W2"] = g.reshape(-1, F).T @ dout.reshape(-1, D)
    grads[pre + "b2"] = dout.sum(axis=(0, 1))
    dh = (dout @ p[pre + "W2"].T) * gelu_grad(h)
    grads[pre + "W1"] = xin.reshape(-1, D).T @ dh.reshape(-1, F)
    grads[pre + "b1"] = dh.sum(axis=(0, 1))
    return dh @ p[pre + "W1"].T


# --------------------------------------------------------------------------
# encoder block f_l (App. A.1: pre-LN for ViT, post-LN for BERT)
# --------------------------------------------------------------------------
def block_forward(cfg, p, l, x):
    pre = f"blk{l}."
    eps = cfg.ln_eps
    if cfg.arch == "vit":
        u, s1 = layer_norm(x, p[pre + "ln1_g"], p[pre + "ln1_b"], eps)
        a, sa = mhsa_forward(cfg, p, pre, u)
        y = x + a
        w, s2 = layer_norm(y, p[pre + "ln2_g"], p[pre + "ln2_b"], eps)
        m, sm = mlp_forward(cfg, p, pre, w)
        out = y + m
    else:
        a, sa = mhsa_forward(cfg, p, pre, x)
        y, s1 = layer_norm(x + a, p[pre + "ln1_g"], p[pre + "ln1_b"], eps)
        m, sm = mlp_forward(cfg, p, pre, y)
        out, s2 = layer_norm(y + m, p[pre + "ln2_g"], p[pre + "ln2_b"], eps)
    return out, (s1, sa, s2, sm)


def block_backward(cfg, p, l, dout, saved, grads):
    pre = f"blk{l}."
    s1, sa, s2, sm = saved
    if cfg.arch == "vit":
        dw = mlp_backward(cfg, p, pre, dout, sm, grads)
        dy_ln, grads[pre + "ln2_g"], grads[pre + "ln2_b"] = layer_norm_bwd(dw, s2, p[pre + "ln2_g"])
        dy = dout + dy_ln
        du = mhsa_backward(cfg, p, pre, dy, sa, grads)
        dx_ln, grads[pre + "ln1_g"], grads[pre + "ln1_b"] = layer_norm_bwd(du, s1, p[pre + "ln1_g"])
        return dy + dx_ln
    dr2, grads[pre + "ln2_g"], grads[pre + "ln2_b"] = layer_norm_bwd(dout, s2, p[pre + "ln2_g"])
    dy = dr2 + mlp_backward(cfg, p, pre, dr2, sm, grads)
    dr1, grads[pre + "ln1_g"], grads[pre + "ln1_b"] = layer_norm_bwd(dy, s1, p[pre + "ln1_g"])
    return dr1 + mhsa_backward(cfg, p, pre, dr1, sa, grads)


# --------------------------------------------------------------------------
# front ends (part of the prefix: trained iff k == 0)
# --------------------------------------------------------------------------
def patchify(cfg, images):
    """[B, C, Hh, Ww] -> [B, N, C*p*p]; patches in row-major order over the
    image, each flattened in (channel, row, column) order."""
    B = images.shape[0]
    g = cfg.img // cfg.patch
    t = images.reshape(B, cfg.chans, g, cfg.patch, g, cfg.patch)
    return t.transpose(0, 2, 4, 1, 3, 5).reshape(B, g * g, cfg.chans * cfg.patch * cfg.patch)


def front_forward(cfg, p, inputs):
    """ViT: images -> [cls; patch embeddings] + pos.  BERT: LN(E_w[id] + E_p[t])."""
    if cfg.arch == "vit":
        pm = patchify(cfg, inputs)
        e = pm @ p["front.W_pe"] + p["front.b_pe"]
        B = e.shape[0]
        cls = np.broadcast_to(p["front.cls"], (B, 1, cfg.D))
        return np.concatenate([cls, e], axis=1) + p["front.pos"], (pm,)
    ids = np.asarray(inputs)
    emb = p["front.E_w"][ids] + p["front.E_p"][: cfg.S]
    x, s = layer_norm(emb, p["front.ln_g"], p["front.ln_b"], cfg.ln_eps)
    return x, (ids, s)


def front_backward(cfg, p, dx, saved, grads):
    if cfg.arch == "vit":
        (pm,) = saved
        grads["front.pos"] = dx.sum(axis=0)
        grads["front.cls"] = dx[:, 0, :].sum(axis=0)
        de = dx[:, 1:, :].reshape(-1, cfg.D)
        grads["front.W_pe"] = pm.reshape(-1, pm.shape[-1]).T @ de
        grads["front.b_pe"] = de.sum(axis=0)
        return
    ids, s = saved
    demb, grads["front.ln_g"], grads["front.ln_b"] = layer_norm_bwd(dx, s, p["front.ln_g"])
    gp = np.zeros_like(p["front.E_p"])
    gp[: cfg.S] = demb.sum(axis=0)
    grads["front.E_p"] = gp
    gw = np.zeros_like(p["front.E_w"])
    np.add.at(gw, ids.reshape(-1), demb.reshape(-1, cfg.D))   # duplicates accumulate
    grads["front.E_w"] = gw


# --------------------------------------------------------------------------
# task heads and losses
# --------------------------------------------------------------------------
def head_loss_forward(cfg, p, xL, labels):
    """ViT: final LN, CLS token, linear classifier, mean cross-entropy.
    BERT sequence classification (head "cls"): first token, linear classifier, mean cross-entropy.
    BERT span QA: per-token two-logit linear map; cross-entropy over the
    sequence axis for the start logit and for the end logit; their mean."""
    B = xL.shape[0]
    labels = np.asarray(labels)
    if cfg.arch == "vit":
        c, s = layer_norm(xL[:, 0, :], p["head.ln_g"], p["head.ln_b"], cfg.ln_eps)
        z = c @ p["head.W"] + p["head.b"]                       # [B, C]
        prob = softmax_lastaxis(z)
        lse = np.log(np.exp(z - z.max(-1, keepdims=True)).sum(-1)) + z.max(-1)
        loss = (lse - z[np.arange(B), labels]).mean()
        return loss, z, (c, s, prob, labels)
    if cfg.head == "cls":
        # sequence classification: first token's final activation -> linear classifier -> mean CE
        c = xL[:, 0, :]
        z = c @ p["head.W"] + p["head.b"]                       # [B, C]
        prob = softmax_lastaxis(z)
        lse = np.log(np.exp(z - z.max(-1, keepdims=True)).sum(-1)) + z.max(-1)
        loss = (lse - z[np.arange(B), labels]).mean()
        return loss, z, (c, prob, labels)
    z = xL @ p["head.W"] + p["head.b"]                          # [B, S, 2]
    zt = z.transpose(0, 2, 1)                                   # [B, 2, S]
    prob = softmax_lastaxis(zt)
    zmax = zt.max(-1)
    lse = np.log(np.exp(zt - zmax[..., None]).sum(-1)) + zmax   # [B, 2]
    picked = np.stack([zt[np.arange(B), 0, labels[:, 0]], zt[np.arange(B), 1, labels[:, 1]]], axis=1)
    loss = (0.5 * (lse - picked).sum(axis=1)).mean()
    return loss, z, (xL, prob, labels)


def head_loss_backward(cfg, p, saved, xL_shape, grads):
    B = xL_shape[0]
    if cfg.arch == "vit":
        c, s, prob, labels = saved
        dz = prob.copy()
        dz[np.arange(B), labels] -= 1.0
        dz /= B
        grads["head.W"] = c.T @ dz
        grads["head.b"] = dz.sum(axis=0)
        dc = dz @ p["head.W"].T
        dcls, grads["head.ln_g"], grads["head.ln_b"] = layer_norm_bwd(dc, s, p["head.ln_g"])
        dx = np.zeros(xL_shape, dtype=dcls.dtype)
        dx[:, 0, :] = dcls
        return dx
    if cfg.head == "cls":
        c, prob, labels = saved
        dz = prob.copy()
        dz[np.arange(B), labels] -= 1.0
        dz /= B
        grads["head.W"] = c.T @ dz
        grads["head.b"] = dz.sum(axis=0)
        dx = np.zeros(xL_shape, dtype=dz.dtype)
        dx[:, 0, :] = dz @ p["head.W"].T
        return dx
    xL, prob, labels = saved
    dzt = prob.copy()                                           # [B, 2, S]
    dzt[np.arange(B), 0, labels[:, 0]] -= 1.0
    dzt[np.arange(B), 1, labels[:, 1]] -= 1.0
    dzt *= 0.5 / B
    dz = dzt.transpose(0, 2, 1)                                 # [B, S, 2]
    grads["head.W"] = xL.reshape(-1, cfg.D).T @ dz.reshape(-1, 2)
    grads["head.b"] = dz.sum(axis=(0, 1))
    return dz @ p["head.W"].T


# --------------------------------------------------------------------------
# the step, split at the freeze boundary k
# --------------------------------------------------------------------------
def prefix_forward(cfg, p, h, lo, hi):
    """Forward-only through blocks lo .. hi-1; nothing is kept (Sec. 3.2.1)."""
    for l in range(lo, hi):
        h, _ = block_forward(cfg, p, l, h)
    return h


def frozen_forward(cfg, p, inputs, k):
    """F_frozen: front end and blocks 0 .. k-1.  Returns (h_k, front_saved);
    front_saved feeds the front-end backward, which only runs when k == 0."""
    h0, fsaved = front_forward(cfg, p, inputs)
    return prefix_forward(cfg, p, h0, 0, k), fsaved


def active_fwd_bwd(cfg, p, h_k, labels, k, front_saved=None):
    """F_pipe: forward and backward through blocks k .. L-1 and the head.
    Returns (loss, grads, aux); grads holds the active tensors only."""
    assert 0 <= k <= cfg.L
    h = h_k
    saved = []
    for l in range(k, cfg.L):
        h, s = block_forward(cfg, p, l, h)
        saved.append(s)
    loss, z, hs = head_loss_forward(cfg, p, h, labels)
    grads = {}
    dh = head_loss_backward(cfg, p, hs, h.shape, grads)
    for l in range(cfg.L - 1, k - 1, -1):
        dh = block_backward(cfg, p, l, dh, saved[l - k], grads)
    if k == 0:
        assert front_saved is not None
        front_backward(cfg, p, dh, front_saved, grads)
    return loss, grads, {"logits": z, "h_L": h, "dh_k": dh}


def accumulated_fwd_bwd(cfg, p, inputs, labels, k, sizes):
    """Micro-batch accumulation (Sec. 2.1, Sec. 3.2.3): the mini-batch is cut into micro-batches of
    the given sizes; each runs frozen forward + active forward/backward on its own, and the step's
    loss and gradient are the sample-weighted means  sum_i n_i * (.)_i / sum_i n_i.
    Returns (loss, grads)."""
    assert sum(sizes) == len(inputs)
    loss, grads, at = 0.0, None, 0
    for n in sizes:
        x, y = inputs[at:at + n], labels[at:at + n]
        at += n
        hk, fs = frozen_forward(cfg, p, x, k)
        li, gi, _ = active_fwd_bwd(cfg, p, hk, y, k, fs)
        loss += n * li
        if grads is None:
            grads = {name: n * g for name, g in gi.items()}
        else:
            for name, g in gi.items():
                grads[name] = grads[name] + n * g
    tot = float(sum(sizes))
    return loss / tot, {name: g / tot for name, g in grads.items()}


def layer_grad_norms(cfg, grads, k):
    """||g_l|| of Eq. 1 (Sec. 3.1): L2 norm over all tensors of a layer taken
    together, on the raw gradient of the mean loss.  Slots: [front end,
    block 0 .. L-1, head]; a frozen layer has no gradient and reads 0."""
    sq = np.zeros(cfg.L + 2, dtype=np.float64)
    for name, g in grads.items():
        if is_active(name, cfg, k):
            sq[group_of(name, cfg)] += float((np.asarray(g, dtype=np.float64) ** 2).sum())
    return np.sqrt(sq)


# --------------------------------------------------------------------------
# optimizers over the active set (Sec. 3.3, App. D.2)
# --------------------------------------------------------------------------
def new_opt_state(p):
    return {"t": 0, "m": {n: np.zeros_like(a) for n, a in p.items()},
            "v": {n: np.zeros_like(a) for n, a in p.items()}}


def drop_frozen_state(cfg, state, k):
    """A layer that freezes gives up its optimizer state for good."""
    for n in list(state["m"].keys()):
        if not is_active(n, cfg, k):
            del state["m"][n]
            state["v"].pop(n, None)


def sgdm_step(cfg, p, grads, state, k, lr, momentum, weight_decay=0.0):
    """v <- mu v + g (+ wd*w on decayed tensors); w <- w - lr v.  No dampening,
    no Nesterov, v_0 = 0.  Momentum buffers live in state["m"]."""
    state["t"] += 1
    for n in p:
        if not is_active(n, cfg, k):
            continue
        g = grads[n]
        if weight_decay != 0.0 and is_decayed(n):
            g = g + weight_decay * p[n]
        state["m"][n] = momentum * state["m"][n] + g
        p[n] = p[n] - lr * state["m"][n]


def adamw_step(cfg, p, grads, state, k, lr, beta1, beta2, eps, weight_decay):
    """Decoupled weight decay, bias-corrected moments, one step counter shared
    by all tensors (it keeps counting across boundary moves)."""
    state["t"] += 1
    t = state["t"]
    c1 = 1.0 - beta1 ** t
    c2 = 1.0 - beta2 ** t
    for n in p:
        if not is_active(n, cfg, k):
            continue
        g = grads[n]
        w = p[n]
        if weight_decay != 0.0 and is_decayed(n):
            w = w * (1.0 - lr * weight_decay)
        m = beta1 * state["m"][n] + (1.0 - beta1) * g
        v = beta2 * state["v"][n] + (1.0 - beta2) * g * g
        state["m"][n] = m
        state["v"][n] = v
        p[n] = w - lr * (m / c1) / (np.sqrt(v / c2) + eps)


# --------------------------------------------------------------------------
# frozen-prefix activation cache (Sec. 3.4; App. D.1 item 2)
# --------------------------------------------------------------------------
class ActivationCache:
    """sample id -> (k_written, row).  lookup() returns, per sample, the
    decision the method takes: "hit" (entry written at the current k),
    "advance" (entry written at a smaller k: run only blocks k_written..k-1)
    or "miss" (run the front end and blocks 0..k-1)."""

    def __init__(self):
        self.rows = {}

    def decision(self, sample_id, k):
        if sample_id not in self.rows:
            return "miss", -1
        kw, _ = self.rows[sample_id]
        return ("hit" if kw == k else "advance"), kw

    def frozen_forward(self, cfg, p, inputs, sample_ids, k):
        """Boundary activation h_k for a batch, served from / written to the
        cache sample by sample.  Returns (h_k, decisions, block_runs) where
        block_runs counts (sample, block) forward evaluations performed."""
        assert k >= 1
        out = []
        decisions = []
        runs = 0
        for i, sid in enumerate(sample_ids):
            what, kw = self.decision(sid, k)
            decisions.append((what, kw))
            if what == "hit":
                row = self.rows[sid][1]
            elif what == "advance":
                assert kw < k
                row = prefix_forward(cfg, p, self.rows[sid][1][None], kw, k)[0]
                runs += k - kw
            else:
                h0, _ = front_forward(cfg, p, inputs[i:i + 1])
                row = prefix_forward(cfg, p, h0, 0, k)[0]
                runs += k
            self.rows[sid] = (k, row)
            out.append(row)
        return np.stack(out, axis=0), decisions, runs


# --------------------------------------------------------------------------
# freeze rule, Eq. 1 (Sec. 3.1) and its closed form (App. B)
# --------------------------------------------------------------------------
def next_boundary(norms, k_prev, L, alpha):
    """L_frozen^(T) = min( L_frozen^(T-1) + alpha (L - L_frozen^(T-1)),
                           argmin_{l >= L_frozen^(T-1)} ||g_l^(T)|| ).
    Readings where the paper is silent: the argmin ranges over blocks
    k_prev .. L-1 (the printed range ends at L, one past the last layer), the
    bound is truncated to an integer, ties go to the lowest index, and the
    result never decreases.  `norms` has L+2 slots as layer_grad_norms()."""
    blocks = np.asarray(norms, dtype=np.float64)[1:L + 1]
    bound = int(math.floor(k_prev + alpha * (L - k_prev)))
    if k_prev >= L:
        return L
    arg = k_prev + int(np.argmin(blocks[k_prev:L]))
    return max(k_prev, min(bound, arg))


def alpha_bound_recursion(L, alpha, T):
    """Real-valued bound term of Eq. 1 iterated T times from 0."""
    x = 0.0
    for _ in range(T):
        x = x + alpha * (L - x)
    return x


def alpha_bound_closed_form(L, alpha, T):
    """App. B, Eq. 3: (1-a)^T [ aL/(1-a) + sum_{t=2..T} aL/(1-a)^t ]."""
    s = alpha * L / (1.0 - alpha)
    for t in range(2, T + 1):
        s += alpha * L / (1.0 - alpha) ** t
    return (1.0 - alpha) ** T * s
