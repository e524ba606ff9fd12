"""Model of the library's bf16 mode (test plumbing; no part of the oracle and no part of the product).

The arithmetic is the oracle's, called function by function in fp64; on top of it every tensor that the HIP
path stores in bf16 or hands to a matrix core as a bf16 operand is rounded to nearest-even at the point where
the kernels round it.  Everything the kernels keep in fp32 (accumulators, LayerNorm and softmax statistics,
the gradient of the residual stream, the two pre-LayerNorm sums of a post-LN block, parameter gradients) stays
unrounded.  The model answers one question: how far from the exact result does *any* implementation land that
stores these tensors in bf16?  Where that distance is above the 2e-2 bar of the 12-block workloads (tiny
widths, a handful of tokens: nothing averages the roundings out), the GPU result is held to the model instead,
which shows that the excess comes from the storage format and not from a kernel.

Rounding points (forward): patch matrix, patch embeddings, block inputs (pre-LN: the residual stream itself),
LayerNorm outputs, packed qkv, the unnormalised softmax probabilities fed to P.V, attention context, GELU
output, saved GELU', the classifier feature.  Backward: every dY that feeds a weight- or input-gradient
product (copies of the fp32 stream, dF, dQKV, dCTX, dLN-out), the recomputed probabilities fed to P^T.dO and
dS fed to dS.K / dS^T.Q, the classifier's dz and dc.
"""
import math

import numpy as np

from oracle import encoder as orc
from paper_2102_03161_amd import synth


ROUNDING = True   # False: every rounding point is the identity and the model is the oracle


def r(a):
    """Round to the nearest bf16 (ties to even), result in fp64."""
    if not ROUNDING:
        return np.asarray(a, dtype=np.float64)
    return synth.round_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)


def _rss_lin(rss, name, x, dy):
    """Root-sum-square of the summands x[t,i] dy[t,j] of a weight gradient, per element."""
    if rss is not None:
        rss[name] = np.sqrt((x * x).T @ (dy * dy))


def _rss_sum(rss, name, terms, axes):
    """Root-sum-square of the summands of a gradient that is a plain sum over `axes`."""
    if rss is not None:
        rss[name] = np.sqrt((terms * terms).sum(axis=axes))


def _ln_bwd(rss, gname, bname, dy, saved, g):
    out = orc.layer_norm_bwd(dy, saved, g)
    red = tuple(range(dy.ndim - 1))
    _rss_sum(rss, gname, dy * saved[0], red)
    _rss_sum(rss, bname, dy, red)
    return out


def _attn_fwd(cfg, qkv):
    D, H = cfg.D, cfg.H
    dh = D // H
    q = orc._split_heads(qkv[..., 0:D], H)
    k = orc._split_heads(qkv[..., D:2 * D], H)
    v = orc._split_heads(qkv[..., 2 * D:3 * D], H)
    s = (q @ k.transpose(0, 1, 3, 2)) / math.sqrt(dh)
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    lsum = e.sum(axis=-1, keepdims=True)
    ctx = (r(e) @ v) / lsum                      # P.V runs on bf16 probabilities, normalised afterwards in fp32
    lse = m + np.log(lsum)
    return r(orc._merge_heads(ctx)), (q, k, v, lse)


def _attn_bwd(cfg, saved, ctx, dctx, xin=None):
    """ctx, dctx: bf16-valued [B,S,D].  Returns the packed bf16 dqkv.  With xin (the input of the qkv product)
    also the root-sum-square of the summands of the packed weight's and bias's gradients, [D,3D] and [3D]:
    for the query and key thirds over the (query, key) pairs of the inner sums, and for the value third over
    the queries, W_v's gradient being sum_i (sum_j P_ij x_j) do_i^T and b_v's sum_i do_i (rows of P sum to one),
    so that a rounding error of do_i enters them once, not once per key."""
    q, k, v, lse = saved
    H = cfg.H
    dh = cfg.D // H
    o = orc._split_heads(ctx, H)
    do = orc._split_heads(dctx, H)
    P = np.exp((q @ k.transpose(0, 1, 3, 2)) / math.sqrt(dh) - lse)
    dv = r(P).transpose(0, 1, 3, 2) @ do
    dP = do @ v.transpose(0, 1, 3, 2)
    delta = (do * o).sum(axis=-1, keepdims=True)
    dS = r(P * (dP - delta))
    dq = (dS @ k) / math.sqrt(dh)
    dk = (dS.transpose(0, 1, 3, 2) @ q) / math.sqrt(dh)
    out = r(np.concatenate([orc._merge_heads(dq), orc._merge_heads(dk), orc._merge_heads(dv)], axis=-1))
    if xin is None:
        return out
    sq = lambda a: a * a
    D = cfg.D
    x2 = sq(xin).reshape(-1, D)
    rq = orc._merge_heads(np.sqrt(sq(dS) @ sq(k)) / math.sqrt(dh)).reshape(-1, D)
    rk = orc._merge_heads(np.sqrt(sq(dS).transpose(0, 1, 3, 2) @ sq(q)) / math.sqrt(dh)).reshape(-1, D)
    rW = np.zeros((D, 3 * D))
    rW[:, 0:D] = np.sqrt(x2.T @ sq(rq))
    rW[:, D:2 * D] = np.sqrt(x2.T @ sq(rk))
    for h in range(H):
        xbar = P[:, h] @ xin                                   # [B,S,D]: attention-weighted mean input per query
        rW[:, 2 * D + h * dh:2 * D + (h + 1) * dh] = np.sqrt(sq(xbar).reshape(-1, D).T @ sq(do[:, h]).reshape(-1, dh))
    rb = np.concatenate([np.sqrt(sq(rq).sum(0)), np.sqrt(sq(rk).sum(0)), np.sqrt(sq(dctx).reshape(-1, D).sum(0))])
    return out, rW, rb


def _block_fwd(cfg, p, l, x):
    pre = f"blk{l}."
    eps = cfg.ln_eps
    if cfg.arch == "vit":
        u, s1 = orc.layer_norm(x, p[pre + "ln1_g"], p[pre + "ln1_b"], eps)
        u = r(u)
        qkv = r(u @ p[pre + "Wqkv"] + p[pre + "bqkv"])
        ctx, sa = _attn_fwd(cfg, qkv)
        y = r(x + ctx @ p[pre + "Wo"] + p[pre + "bo"])
        w, s2 = orc.layer_norm(y, p[pre + "ln2_g"], p[pre + "ln2_b"], eps)
        w = r(w)
        h = w @ p[pre + "W1"] + p[pre + "b1"]
        g, hp = r(orc.gelu(h)), r(orc.gelu_grad(h))
        out = r(y + g @ p[pre + "W2"] + p[pre + "b2"])
        return out, dict(x=x, u=u, s1=s1, sa=sa, ctx=ctx, y=y, w=w, s2=s2, g=g, hp=hp)
    qkv = r(x @ p[pre + "Wqkv"] + p[pre + "bqkv"])
    ctx, sa = _attn_fwd(cfg, qkv)
    u = x + ctx @ p[pre + "Wo"] + p[pre + "bo"]                       # fp32 in the library
    y, s1 = orc.layer_norm(u, p[pre + "ln1_g"], p[pre + "ln1_b"], eps)
    y = r(y)
    h = y @ p[pre + "W1"] + p[pre + "b1"]
    g, hp = r(orc.gelu(h)), r(orc.gelu_grad(h))
    wn = y + g @ p[pre + "W2"] + p[pre + "b2"]                        # fp32 in the library
    out, s2 = orc.layer_norm(wn, p[pre + "ln2_g"], p[pre + "ln2_b"], eps)
    return r(out), dict(x=x, sa=sa, ctx=ctx, s1=s1, y=y, s2=s2, g=g, hp=hp)


def _block_bwd(cfg, p, l, dout, sv, grads, rss=None):
    """dout: fp32-valued gradient of the residual stream (unrounded).  Returns the same for the block's input.
    rss (optional dict): receives, per gradient tensor, the root-sum-square of its summands."""
    pre = f"blk{l}."
    D, F = cfg.D, cfg.F
    T2 = lambda a, n: a.reshape(-1, n)

    def lin(name, bname, x, nx, dy, ny, dy_for_bias):
        grads[pre + name] = T2(x, nx).T @ T2(dy, ny)
        grads[pre + bname] = dy_for_bias.sum(axis=(0, 1))
        _rss_lin(rss, pre + name, T2(x, nx), T2(dy, ny))
        _rss_sum(rss, pre + bname, dy_for_bias, (0, 1))

    def attn_bwd(dctx, xin):
        """dqkv; the qkv product's gradients' summand scale also covers the inner sums of the attention"""
        if rss is None:
            return _attn_bwd(cfg, sv["sa"], sv["ctx"], dctx)
        dqkv, rW, rb = _attn_bwd(cfg, sv["sa"], sv["ctx"], dctx, xin)
        lin("Wqkv", "bqkv", xin, D, dqkv, 3 * D, dqkv)
        rss[pre + "Wqkv"] = np.maximum(rss[pre + "Wqkv"], rW)
        rss[pre + "bqkv"] = np.maximum(rss[pre + "bqkv"], rb)
        return dqkv

    if cfg.arch == "vit":
        do = r(dout)
        lin("W2", "b2", sv["g"], F, do, D, dout)
        dF = r((do @ p[pre + "W2"].T) * sv["hp"])
        lin("W1", "b1", sv["w"], D, dF, F, dF)
        dw = r(dF @ p[pre + "W1"].T)
        dy_ln, grads[pre + "ln2_g"], grads[pre + "ln2_b"] = _ln_bwd(rss, pre + "ln2_g", pre + "ln2_b", dw, sv["s2"], p[pre + "ln2_g"])
        dy = dout + dy_ln
        dyo = r(dy)
        lin("Wo", "bo", sv["ctx"], D, dyo, D, dy)
        dctx = r(dyo @ p[pre + "Wo"].T)
        dqkv = attn_bwd(dctx, sv["u"])
        lin("Wqkv", "bqkv", sv["u"], D, dqkv, 3 * D, dqkv) if rss is None else None
        du = r(dqkv @ p[pre + "Wqkv"].T)
        dx_ln, grads[pre + "ln1_g"], grads[pre + "ln1_b"] = _ln_bwd(rss, pre + "ln1_g", pre + "ln1_b", du, sv["s1"], p[pre + "ln1_g"])
        return dy + dx_ln
    dr2, grads[pre + "ln2_g"], grads[pre + "ln2_b"] = _ln_bwd(rss, pre + "ln2_g", pre + "ln2_b", dout, sv["s2"], p[pre + "ln2_g"])
    dr2o = r(dr2)
    lin("W2", "b2", sv["g"], F, dr2o, D, dr2)
    dF = r((dr2o @ p[pre + "W2"].T) * sv["hp"])
    lin("W1", "b1", sv["y"], D, dF, F, dF)
    dy = dF @ p[pre + "W1"].T + dr2
    dr1, grads[pre + "ln1_g"], grads[pre + "ln1_b"] = _ln_bwd(rss, pre + "ln1_g", pre + "ln1_b", dy, sv["s1"], p[pre + "ln1_g"])
    dr1o = r(dr1)
    lin("Wo", "bo", sv["ctx"], D, dr1o, D, dr1)
    dctx = r(dr1o @ p[pre + "Wo"].T)
    dqkv = attn_bwd(dctx, sv["x"])
    lin("Wqkv", "bqkv", sv["x"], D, dqkv, 3 * D, dqkv) if rss is None else None
    return dqkv @ p[pre + "Wqkv"].T + dr1


def step(cfg, p, inputs, labels, k, rss=None):
    """Forward, loss and backward at boundary k with the library's bf16 storage points.
    p: fp64 arrays holding bf16-representable values.  Returns (loss, grads, aux).
    rss (optional dict): receives, per gradient tensor, the root-sum-square of its summands over the tokens."""
    if cfg.arch == "vit":
        pm = r(orc.patchify(cfg, np.asarray(inputs, dtype=np.float64)))
        e = r(pm @ p["front.W_pe"] + p["front.b_pe"])
        B = e.shape[0]
        cls = np.broadcast_to(p["front.cls"], (B, 1, cfg.D))
        h = r(np.concatenate([cls, e], axis=1) + p["front.pos"])
        fs = (pm,)
    else:
        ids = np.asarray(inputs)
        emb = p["front.E_w"][ids] + p["front.E_p"][: cfg.S]
        h, s_e = orc.layer_norm(emb, p["front.ln_g"], p["front.ln_b"], cfg.ln_eps)
        h = r(h)
        fs = (ids, s_e)
    saved = {}
    hk = None
    for l in range(cfg.L):
        if l == k:
            hk = h
        h, sv = _block_fwd(cfg, p, l, h)
        if l >= k:
            saved[l] = sv
    if k == cfg.L:
        hk = h
    grads = {}
    B = h.shape[0]
    labels = np.asarray(labels)
    if cfg.arch == "vit" or cfg.head == "cls":
        if cfg.arch == "vit":
            c, s = orc.layer_norm(h[:, 0, :], p["head.ln_g"], p["head.ln_b"], cfg.ln_eps)
            c = r(c)
        else:
            c = h[:, 0, :]
        z = c @ p["head.W"] + p["head.b"]
        if rss is not None:   # the logits are sums too (two-class heads: 768 terms of order 0.1 giving 0.05)
            rss["act:logits"] = np.sqrt((c * c) @ (p["head.W"] * p["head.W"]) + p["head.b"] ** 2)
        prob = orc.softmax_lastaxis(z)
        lse = np.log(np.exp(z - z.max(-1, keepdims=True)).sum(-1)) + z.max(-1)
        loss = (lse - z[np.arange(B), labels]).mean()
        dz = prob.copy()
        dz[np.arange(B), labels] -= 1.0
        dz = r(dz / B)
        grads["head.W"] = c.T @ dz
        grads["head.b"] = dz.sum(axis=0)
        _rss_lin(rss, "head.W", c, dz)
        _rss_sum(rss, "head.b", dz, 0)
        dh = np.zeros(h.shape)
        if cfg.arch == "vit":
            dc = r(dz @ p["head.W"].T)
            dh[:, 0, :], grads["head.ln_g"], grads["head.ln_b"] = _ln_bwd(rss, "head.ln_g", "head.ln_b", dc, s, p["head.ln_g"])
        else:
            dh[:, 0, :] = dz @ p["head.W"].T
    else:
        loss, z, hs = orc.head_loss_forward(cfg, p, h, labels)
        dh = orc.head_loss_backward(cfg, p, hs, h.shape, grads)
        if rss is not None:
            rss["act:logits"] = np.sqrt((h * h) @ (p["head.W"] * p["head.W"]) + p["head.b"] ** 2)
            dz = (dh.reshape(-1, cfg.D) @ np.linalg.pinv(p["head.W"].T)).reshape(B, cfg.S, 2)   # dh = dz W^T, W has rank 2
            _rss_lin(rss, "head.W", h.reshape(-1, cfg.D), dz.reshape(-1, 2))
            _rss_sum(rss, "head.b", dz, (0, 1))
    for l in range(cfg.L - 1, k - 1, -1):
        dh = _block_bwd(cfg, p, l, dh, saved[l], grads, rss)
    if k == 0:
        if cfg.arch == "vit":
            grads["front.pos"] = dh.sum(axis=0)
            grads["front.cls"] = dh[:, 0, :].sum(axis=0)
            de = r(dh[:, 1:, :]).reshape(-1, cfg.D)
            pm2 = fs[0].reshape(-1, fs[0].shape[-1])
            grads["front.W_pe"] = pm2.T @ de
            grads["front.b_pe"] = de.sum(axis=0)      # column sums ride on the product's bf16 operand
            _rss_sum(rss, "front.pos", dh, 0)
            _rss_sum(rss, "front.cls", dh[:, 0, :], 0)
            _rss_lin(rss, "front.W_pe", pm2, de)
            _rss_sum(rss, "front.b_pe", de, 0)
        else:
            orc.front_backward(cfg, p, dh, fs, grads)
            if rss is not None:
                ids, s_e = fs
                demb, _, _ = _ln_bwd(rss, "front.ln_g", "front.ln_b", dh, s_e, p["front.ln_g"])
                gp = np.zeros_like(p["front.E_p"])
                gp[: cfg.S] = (demb * demb).sum(axis=0)
                rss["front.E_p"] = np.sqrt(gp)
                gw = np.zeros_like(p["front.E_w"])
                np.add.at(gw, ids.reshape(-1), (demb * demb).reshape(-1, cfg.D))
                rss["front.E_w"] = np.sqrt(gw)
    return loss, grads, {"logits": z, "h_L": h, "h_k": hk}


def summand_rss(cfg, p, inputs, labels, k):
    """Per gradient tensor and element, the root-sum-square of the summands (over the tokens of the batch)
    that the exact gradient adds up, from the exact intermediates (rounding switched off).  An element whose
    summands carry independent relative errors of size e is uncertain by about e times this, however small the
    sum itself comes out: it is the scale a cancelling gradient has to be measured against."""
    global ROUNDING
    was = ROUNDING
    ROUNDING = False
    try:
        rss = {}
        step(cfg, p, inputs, labels, k, rss)
    finally:
        ROUNDING = was
    return rss
