"""CPU fp64 oracle for one node's local training step with partial parameter updates.

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow reference that the HIP path is checked
against.  Only tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
product library never does, and this file imports nothing from the product.

What it computes (paper: "Partial Parameter Updates", Algorithm 1 and Section 2.2; Appendix
"Partial Backward" for the per-block backward; Appendix "FLOPs calculation"):

  * forward():           standard forward pass of a decoder-only transformer over ALL parameters
                         (Section 2.2, "the forward pass is standard"), next-token loss Eq. (2.2)
                         taken as a mean over the valid positions.
  * backward_full():     ordinary back-propagation for every parameter.
  * masked_gradient():   DEFINITION path of Alg. 1's gradient line: the full gradient restricted
                         to the index set I_train (g[i] = dL/dtheta[i] if i in I_train, else 0).
  * backward_restricted(): the restricted backward of Appendix "Partial Backward": weight
                         gradients only for trainable slices, input gradients through ALL slices
                         and ALL heads, and nothing propagated below the lowest trainable
                         parameter.  Counts the matmul FLOPs it executes.
                         With jacobian_extra: the detach-all-but-k (+ random) ablation of
                         Appendix "Additional Results".
  * adamw_update():      InnerOpt of Alg. 1 (decoupled AdamW, Experimental Setup) applied to
                         theta[I_train] only; frozen coordinates are not touched at all (no
                         weight decay either).
  * outer_step():        Alg. 1's delta, count normalisation and OuterOpt (Nesterov-momentum SGD,
                         Experimental Setup) for the node's own trainable subset.
  * flops_forward / flops_backward_ffn_slice / flops_backward_all: closed forms for the matmul
                         FLOPs the step executes;  paper_flops: the paper's own closed forms.

Architecture details the paper leaves open follow the benchmark configs: pre-norm RMSNorm
(eps inside the square root), rotary embeddings with half-split pairing (i, i+dh/2) and angle
pos * base^(-2i/dh), causal attention, SwiGLU FFN  y = (silu(x Wg^T) * (x Wu^T)) Wd  with
Wg, Wu, Wd all stored (d_ff x d_model), untied embedding / lm_head, no biases, no dropout.

Pins (tests/test_oracle_pins.py): central finite differences for every tensor; library routines
(rms_norm, scaled-dot-product attention, cross entropy, AdamW, Nesterov SGD) on the cases that
reduce to them; LocalTrainer as a whole (decay_mask_for and the packed order included) against
library autograd + library AdamW with decayed / undecayed parameter groups; its bf16-storage mode
against the library's bf16 cast; closed forms (rotary, AdamW step 1, Nesterov step 1, loss ~ ln V at init);
invariants (causality, slice additivity of the FFN, masked == slice of full, frozen unchanged);
the detach ablation against library autograd with the dropped units' activations detached;
FLOP counter == closed form; the paper's FLOP formulas reproduce its "15% fewer FLOPs" and its
rho=1 identity; Table 1's trainable-parameter column.
Parity unpinned: Table 1 perplexities / memory GB and the 0.44 s step time (need the paper's
data, weights and hardware).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# =============================================================================== building blocks
def rmsnorm_fwd(x, gamma, eps):
    """y = gamma * x * rsqrt(mean(x^2) + eps) along the last axis; returns (y, rstd)."""
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * rstd * gamma, rstd[..., 0]


def rmsnorm_bwd(dy, x, rstd, gamma):
    """Gradient of rmsnorm_fwd wrt x and gamma.  With xh = x*rstd:
    dx = rstd * (gamma*dy - xh * mean(gamma*dy*xh)),  dgamma = sum_t dy*xh."""
    xh = x * rstd[:, None]
    gdy = dy * gamma
    dx = rstd[:, None] * (gdy - xh * np.mean(gdy * xh, axis=-1, keepdims=True))
    dgamma = np.sum(dy * xh, axis=0)
    return dx, dgamma


def rope_tables(S, dh, base):
    half = dh // 2
    inv = base ** (-2.0 * np.arange(half, dtype=F64) / dh)
    ang = np.arange(S, dtype=F64)[:, None] * inv[None, :]
    return np.cos(ang), np.sin(ang)


def rope_apply(x, cos, sin, inverse=False):
    """x: [B,S,h,dh].  Rotates the pair (x[i], x[i+dh/2]) by +angle (or -angle if inverse).
    The inverse rotation is also the backward of the forward rotation (the map is orthogonal)."""
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    c = cos[None, :, None, :]
    s = sin[None, :, None, :]
    if inverse:
        s = -s
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def silu(z):
    return z / (1.0 + np.exp(-z))


def attention_fwd(q, k, v):
    """Causal softmax attention per (batch, head).  q,k,v: [B,S,h,dh] -> (o [B,S,h,dh], P [B,h,S,S]).
    Appendix "MHA with frozen heads": S = q k^T / sqrt(dh), A = row-softmax(S), U = A v; the causal
    mask (position i sees j <= i) comes from the autoregressive factorisation of Section 2.1."""
    B, S, h, dh = q.shape
    scale = 1.0 / np.sqrt(dh)
    o = np.empty_like(q)
    P = np.empty((B, h, S, S), dtype=F64)
    causal = np.tril(np.ones((S, S), dtype=bool))
    for b in range(B):
        for j in range(h):
            s = (q[b, :, j, :] @ k[b, :, j, :].T) * scale
            s = np.where(causal, s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            e = np.exp(s)
            p = e / e.sum(axis=-1, keepdims=True)
            P[b, j] = p
            o[b, :, j, :] = p @ v[b, :, j, :]
    return o, P


def attention_bwd(do, q, k, v, P):
    """Appendix "MHA with frozen heads", steps 2-4, for every head:
    dV = P^T dO; dP = dO V^T; dS = P * (dP - rowsum(dP*P)); dQ = dS K / sqrt(dh); dK = dS^T Q / sqrt(dh)."""
    B, S, h, dh = q.shape
    scale = 1.0 / np.sqrt(dh)
    dq = np.empty_like(q)
    dk = np.empty_like(k)
    dv = np.empty_like(v)
    for b in range(B):
        for j in range(h):
            p = P[b, j]
            dO = do[b, :, j, :]
            dv[b, :, j, :] = p.T @ dO
            dp = dO @ v[b, :, j, :].T
            ds = p * (dp - np.sum(dp * p, axis=-1, keepdims=True))
            dq[b, :, j, :] = (ds @ k[b, :, j, :]) * scale
            dk[b, :, j, :] = (ds.T @ q[b, :, j, :]) * scale
    return dq, dk, dv


# =============================================================================== forward
def to_f64(params):
    return {k: np.array(v, dtype=F64) for k, v in params.items()}   # always a private copy


def forward(cfg, params, tokens, targets, keep_probs=True):
    """Full forward over all parameters.  Returns (loss, cache).  tokens/targets: [B,S] ints,
    target -1 = position ignored; loss = mean over valid positions of (logsumexp(z) - z[target])."""
    B, S = tokens.shape
    T = B * S
    d, h, L = cfg["d_model"], cfg["n_heads"], cfg["n_layers"]
    dh = d // h
    eps = cfg["rms_eps"]
    cos, sin = rope_tables(S, dh, cfg["rope_base"])
    x = params["embed"][tokens.reshape(-1)]
    layers = []
    for l in range(L):
        p = f"layers.{l}."
        c = {"x": x}
        n1, c["rstd1"] = rmsnorm_fwd(x, params[p + "attn_norm"], eps)
        qkv = n1 @ params[p + "wqkv"].T
        q = rope_apply(qkv[:, :d].reshape(B, S, h, dh), cos, sin)
        k = rope_apply(qkv[:, d:2 * d].reshape(B, S, h, dh), cos, sin)
        v = qkv[:, 2 * d:].reshape(B, S, h, dh)
        o, P = attention_fwd(q, k, v)
        o2 = o.reshape(T, d)
        xm = x + o2 @ params[p + "wo"].T
        n2, c["rstd2"] = rmsnorm_fwd(xm, params[p + "ffn_norm"], eps)
        g = n2 @ params[p + "wg"].T
        u = n2 @ params[p + "wu"].T
        a = silu(g) * u
        x = xm + a @ params[p + "wd"]
        c.update(n1=n1, q=q, k=k, v=v, P=P if keep_probs else None, o=o2, xm=xm, n2=n2, g=g, u=u, a=a)
        layers.append(c)
    nf, rstdf = rmsnorm_fwd(x, params["final_norm"], eps)
    z = nf @ params["lm_head"].T
    tg = targets.reshape(-1)
    valid = tg >= 0
    n_valid = int(valid.sum())
    zmax = z.max(axis=-1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=-1))
    picked = z[np.arange(T), np.where(valid, tg, 0)]
    loss = float(np.sum((lse - picked)[valid]) / max(n_valid, 1))
    cache = dict(B=B, S=S, tokens=tokens.reshape(-1), targets=tg, valid=valid, n_valid=n_valid,
                 layers=layers, xL=x, rstdf=rstdf, nf=nf, z=z, lse=lse, cos=cos, sin=sin)
    return loss, cache


def _dlogits(cache):
    """dL/dz = (softmax(z) - onehot(target)) / n_valid on valid rows, 0 on ignored rows."""
    z, lse, tg, valid = cache["z"], cache["lse"], cache["targets"], cache["valid"]
    dz = np.exp(z - lse[:, None])
    rows = np.nonzero(valid)[0]
    dz[rows, tg[rows]] -= 1.0
    dz[~valid] = 0.0
    return dz / max(cache["n_valid"], 1)


# =============================================================================== backward (full)
def backward_full(cfg, params, cache):
    """Plain back-propagation: gradients for every tensor (same names/shapes as params)."""
    B, S = cache["B"], cache["S"]
    T = B * S
    d, h, L = cfg["d_model"], cfg["n_heads"], cfg["n_layers"]
    dh = d // h
    cos, sin = cache["cos"], cache["sin"]
    grads = {}
    dz = _dlogits(cache)
    grads["lm_head"] = dz.T @ cache["nf"]
    dnf = dz @ params["lm_head"]
    dx, grads["final_norm"] = rmsnorm_bwd(dnf, cache["xL"], cache["rstdf"], params["final_norm"])
    for l in reversed(range(L)):
        p = f"layers.{l}."
        c = cache["layers"][l]
        # FFN block (Appendix "MLP with frozen slices", SwiGLU in place of ReLU)
        G = dx
        grads[p + "wd"] = c["a"].T @ G
        dA = G @ params[p + "wd"].T
        sg = 1.0 / (1.0 + np.exp(-c["g"]))
        dU = dA * (c["g"] * sg)
        dG = dA * c["u"] * (sg * (1.0 + c["g"] * (1.0 - sg)))
        grads[p + "wg"] = dG.T @ c["n2"]
        grads[p + "wu"] = dU.T @ c["n2"]
        dn2 = dG @ params[p + "wg"] + dU @ params[p + "wu"]
        dxm_n, grads[p + "ffn_norm"] = rmsnorm_bwd(dn2, c["xm"], c["rstd2"], params[p + "ffn_norm"])
        dxm = dx + dxm_n
        # attention block (Appendix "MHA with frozen heads")
        grads[p + "wo"] = dxm.T @ c["o"]
        do = (dxm @ params[p + "wo"]).reshape(B, S, h, dh)
        dq, dk, dv = attention_bwd(do, c["q"], c["k"], c["v"], c["P"])
        dq = rope_apply(dq, cos, sin, inverse=True)
        dk = rope_apply(dk, cos, sin, inverse=True)
        dqkv = np.concatenate([dq.reshape(T, d), dk.reshape(T, d), dv.reshape(T, d)], axis=1)
        grads[p + "wqkv"] = dqkv.T @ c["n1"]
        dn1 = dqkv @ params[p + "wqkv"]
        dx_n, grads[p + "attn_norm"] = rmsnorm_bwd(dn1, c["x"], c["rstd1"], params[p + "attn_norm"])
        dx = dxm + dx_n
    ge = np.zeros_like(params["embed"])
    np.add.at(ge, cache["tokens"], dx)
    grads["embed"] = ge
    return grads


# =============================================================================== masks
def mask_segments(cfg, mask):
    """I_train as an ordered list of (tensor name, row_lo, row_hi) row blocks, bottom of the network
    first.  Every trainable set the paper uses is a union of such blocks: an FFN hidden-unit range
    is rows [lo,hi) of wg, wu and wd; a head range is rows of the Q, K and V blocks of wqkv."""
    d, h, L = cfg["d_model"], cfg["n_heads"], cfg["n_layers"]
    dh = d // h
    segs = []
    if mask.get("train_embed"):
        segs.append(("embed", 0, cfg["vocab"]))
    for l in range(L):
        p = f"layers.{l}."
        if mask.get("train_norms"):
            segs.append((p + "attn_norm", 0, 1))
        if mask["head_hi"] > mask["head_lo"]:
            for blk in range(3):
                segs.append((p + "wqkv", blk * d + mask["head_lo"] * dh, blk * d + mask["head_hi"] * dh))
        if mask.get("train_wo"):
            segs.append((p + "wo", 0, d))
        if mask.get("train_norms"):
            segs.append((p + "ffn_norm", 0, 1))
        if mask["ffn_hi"] > mask["ffn_lo"]:
            for nm in ("wg", "wu", "wd"):
                segs.append((p + nm, mask["ffn_lo"], mask["ffn_hi"]))
    if mask.get("train_norms"):
        segs.append(("final_norm", 0, 1))
    if mask.get("train_lm_head"):
        segs.append(("lm_head", 0, cfg["vocab"]))
    return segs


def _rows(arr, lo, hi):
    return arr.reshape(1, -1) if arr.ndim == 1 else arr[lo:hi]


def pack(tensors, segs):
    """Concatenate the segments' rows into one flat vector (the packed trainable subset)."""
    if not segs:
        return np.zeros(0, dtype=F64)
    return np.concatenate([_rows(tensors[n], lo, hi).reshape(-1) for n, lo, hi in segs])


def unpack_into(tensors, segs, flat):
    """Write a packed vector back into the segments' rows; everything else is left untouched."""
    off = 0
    for n, lo, hi in segs:
        view = _rows(tensors[n], lo, hi)
        cnt = view.size
        view[...] = flat[off:off + cnt].reshape(view.shape)
        off += cnt


def count_trainable(cfg, mask):
    d = cfg["d_model"]
    return sum((hi - lo) * d for _, lo, hi in mask_segments(cfg, mask))


def masked_gradient(cfg, params, cache, mask):
    """Definition (Alg. 1, gradient line): the I_train slice of the full gradient, packed."""
    return pack(backward_full(cfg, params, cache), mask_segments(cfg, mask))


# =============================================================================== backward (restricted)
def backward_restricted(cfg, params, cache, mask, jacobian_extra=None):
    """Restricted backward.  Returns (packed gradient over I_train, info) where info holds the
    executed matmul FLOPs of the backward ('flops_bwd', causal pairs counted exactly) and the
    activation gradients it produced (for tests).

    Weight gradients are formed only for trainable row blocks; input gradients always run through
    every FFN slice and every head; the chain stops as soon as no trainable parameter lies below.
    At the layer where the FFN slice is the lowest trainable thing, only the slice's columns of
    dA are formed (dW of the gate/up slice needs nothing else).

    jacobian_extra = None is the method.  A (lo, hi) range of FFN hidden units (possibly empty)
    switches to the ablation of Appendix "Additional Results": the FFN's input gradient is summed
    only over the trainable slice k ("detach-all-but-k") and over the units lo..hi-1 of one more
    slice g ("... + random"; the caller draws g); every other unit's dL/dH is taken as zero.
    SwiGLU stands where the appendix writes a ReLU MLP: the mask I(H > 0) becomes the SwiGLU
    derivative.  Weight gradients, attention and everything else are unchanged."""
    B, S = cache["B"], cache["S"]
    T = B * S
    d, h, L, F, V = cfg["d_model"], cfg["n_heads"], cfg["n_layers"], cfg["d_ff"], cfg["vocab"]
    dh = d // h
    cos, sin = cache["cos"], cache["sin"]
    pairs = B * S * (S + 1) // 2
    t_emb, t_norm, t_wo, t_head = (bool(mask.get(k)) for k in
                                   ("train_embed", "train_norms", "train_wo", "train_lm_head"))
    hl, hh = mask["head_lo"], mask["head_hi"]
    fl, fh = mask["ffn_lo"], mask["ffn_hi"]
    t_heads, t_ffn = hh > hl, fh > fl
    any_layer_param = t_norm or t_heads or t_wo or t_ffn
    flops = 0
    g = {}
    info = {"dx": {}}

    def below_layer(l):      # anything trainable strictly below layer l's first parameter
        return t_emb or (l > 0 and any_layer_param)

    if not (any_layer_param or t_emb or t_head):
        return np.zeros(0, dtype=F64), {"flops_bwd": 0, "dx": {}}

    dz = _dlogits(cache)
    if t_head:
        g["lm_head"] = dz.T @ cache["nf"]
        flops += 2 * T * d * V
    if not (any_layer_param or t_emb or t_norm):
        return pack(g, mask_segments(cfg, mask)), {"flops_bwd": flops, "dx": {}}
    dnf = dz @ params["lm_head"]
    flops += 2 * T * d * V
    need_x = any_layer_param or t_emb
    dx, dgf = rmsnorm_bwd(dnf, cache["xL"], cache["rstdf"], params["final_norm"])
    if t_norm:
        g["final_norm"] = dgf
    if need_x:
        for l in reversed(range(L)):
            p = f"layers.{l}."
            c = cache["layers"][l]
            info["dx"][l + 1] = dx
            below_ffn_w = t_norm or t_wo or t_heads or below_layer(l)     # below wg/wu
            G = dx
            dn2 = None
            if t_ffn or below_ffn_w:
                cols = slice(0, F) if below_ffn_w else slice(fl, fh)
                nc = cols.stop - cols.start
                if t_ffn:
                    g[p + "wd"] = c["a"][:, fl:fh].T @ G
                    flops += 2 * T * d * (fh - fl)
                dA = G @ params[p + "wd"][cols].T
                nj = nc                # hidden units that enter the input Jacobian
                if jacobian_extra is not None and below_ffn_w:
                    kept = np.zeros(F, dtype=bool)
                    kept[fl:fh] = True
                    kept[jacobian_extra[0]:jacobian_extra[1]] = True
                    dA = dA * kept[None, :]
                    nj = int(kept.sum())
                flops += 2 * T * d * nj
                gg, uu = c["g"][:, cols], c["u"][:, cols]
                sg = 1.0 / (1.0 + np.exp(-gg))
                dU = dA * (gg * sg)
                dG = dA * uu * (sg * (1.0 + gg * (1.0 - sg)))
                if t_ffn:
                    o0 = fl - cols.start
                    g[p + "wg"] = dG[:, o0:o0 + fh - fl].T @ c["n2"]
                    g[p + "wu"] = dU[:, o0:o0 + fh - fl].T @ c["n2"]
                    flops += 4 * T * d * (fh - fl)
                if below_ffn_w:
                    dn2 = dG @ params[p + "wg"] + dU @ params[p + "wu"]
                    flops += 4 * T * d * nj
            if not below_ffn_w:
                break
            dxm_n, dg2 = rmsnorm_bwd(dn2, c["xm"], c["rstd2"], params[p + "ffn_norm"])
            if t_norm:
                g[p + "ffn_norm"] = dg2
            below_norm2 = t_wo or t_heads or t_norm or below_layer(l)
            if not below_norm2:
                break
            dxm = dx + dxm_n
            if t_wo:
                g[p + "wo"] = dxm.T @ c["o"]
                flops += 2 * T * d * d
            below_wo = t_heads or t_norm or below_layer(l)
            if not below_wo:
                break
            do = (dxm @ params[p + "wo"]).reshape(B, S, h, dh)
            flops += 2 * T * d * d
            dq, dk, dv = attention_bwd(do, c["q"], c["k"], c["v"], c["P"])
            flops += 8 * pairs * d
            dq = rope_apply(dq, cos, sin, inverse=True)
            dk = rope_apply(dk, cos, sin, inverse=True)
            dqkv = np.concatenate([dq.reshape(T, d), dk.reshape(T, d), dv.reshape(T, d)], axis=1)
            if t_heads:
                full = np.zeros((3 * d, d), dtype=F64)
                for blk in range(3):
                    r0, r1 = blk * d + hl * dh, blk * d + hh * dh
                    full[r0:r1] = dqkv[:, r0:r1].T @ c["n1"]
                    flops += 2 * T * d * (r1 - r0)
                g[p + "wqkv"] = full
            below_wqkv = t_norm or below_layer(l)
            if not below_wqkv:
                break
            dn1 = dqkv @ params[p + "wqkv"]
            flops += 6 * T * d * d
            dx_n, dg1 = rmsnorm_bwd(dn1, c["x"], c["rstd1"], params[p + "attn_norm"])
            if t_norm:
                g[p + "attn_norm"] = dg1
            if not below_layer(l):
                break
            dx = dxm + dx_n
        else:
            info["dx"][0] = dx
            if t_emb:
                ge = np.zeros_like(params["embed"])
                np.add.at(ge, cache["tokens"], dx)
                g["embed"] = ge
    # expand slice-only FFN gradients to full-shape holders so that pack() can address rows
    for name, lo, hi in mask_segments(cfg, mask):
        if name.split(".")[-1] in ("wg", "wu", "wd") and g[name].shape[0] == hi - lo and (hi - lo) != F:
            full = np.zeros((F, d), dtype=F64)
            full[lo:hi] = g[name]
            g[name] = full
    info["flops_bwd"] = flops
    return pack(g, mask_segments(cfg, mask)), info


# =============================================================================== FLOP closed forms
def flops_forward(cfg, B, S, causal=True):
    """Executed forward matmul FLOPs for the SwiGLU model: per layer QKV 6Td^2, attention
    4*pairs*d, out-proj 2Td^2, FFN 6TdF (three matrices); lm_head 2TdV.  Appendix "FLOPs
    calculation / Forward", with the FFN term adapted from 2 to 3 matrices and the attention
    term counting causal pairs exactly when causal=True."""
    T = B * S
    d, L, F, V = cfg["d_model"], cfg["n_layers"], cfg["d_ff"], cfg["vocab"]
    pairs = B * S * (S + 1) // 2 if causal else B * S * S
    return L * (8 * T * d * d + 4 * pairs * d + 6 * T * d * F) + 2 * T * d * V


def flops_backward_ffn_slice(cfg, B, S, rho, causal=True):
    """Executed backward matmul FLOPs when only a fraction rho of every layer's FFN hidden units
    is trainable (the benchmark mask; lowest trainable parameter is layer 0's gate/up slice)."""
    T = B * S
    d, L, F, V = cfg["d_model"], cfg["n_layers"], cfg["d_ff"], cfg["vocab"]
    pairs = B * S * (S + 1) // 2 if causal else B * S * S
    Fk = int(round(F * rho))
    return (2 * T * d * V
            + L * 6 * T * d * Fk
            + (L - 1) * 2 * T * d * F + 2 * T * d * Fk
            + (L - 1) * 4 * T * d * F
            + (L - 1) * (8 * T * d * d + 8 * pairs * d))


def flops_backward_all(cfg, B, S, causal=True):
    """mask = ALL: every matmul of the forward has two backward matmuls, except that nothing is
    propagated below layer 0's attention norm (the embedding gradient is a scatter-add)."""
    return 2 * flops_forward(cfg, B, S, causal)


def paper_flops(B, S, H, L, Dff, V, rho_mlp=1.0, rho_attn=1.0):
    """The paper's own closed forms, Appendix "FLOPs calculation" (2-matrix MLP, non-causal
    attention count, embedding and softmax terms included).  Returns (forward, backward)."""
    emb = B * S * H
    proj = 6 * B * S * H * H
    attn = 4 * B * S * S * H
    outp = 2 * B * S * H * H
    mha = proj + attn + outp
    ffn = 4 * B * S * H * Dff
    out = 2 * B * S * H * V + 3 * B * S * V
    fwd = emb + (mha + ffn) * L + out
    mha_b = 8 * B * S * S * H + (10 + 6 * rho_attn) * B * S * H * H
    ffn_b = 4 * B * S * H * Dff + 4 * rho_mlp * B * S * H * Dff
    bwd = 2 * emb + L * (mha_b + ffn_b) + 2 * out
    return fwd, bwd


def paper_trainable_params(L, d, V, n_mlp=1, n_heads=1):
    """Trainable parameters per node for a 2-matrix-MLP GPT (12 L d^2 + V d in total) when 1/n_mlp
    of each MLP and 1/n_heads of each Q/K/V projection are trained (Parameter Slicing)."""
    return 12 * L * d * d + V * d - (1 - 1 / n_mlp) * 8 * L * d * d - (1 - 1 / n_heads) * 3 * L * d * d


def comm_time(K, M_bytes, bw_bytes_per_s):
    """Ring all-reduce time model, Section "Communication Overhead": 2(K-1)/K * M / B."""
    return 2 * (K - 1) / K * M_bytes / bw_bytes_per_s


# =============================================================================== optimizers
def adamw_update(p, m, v, g, t, lr, beta1, beta2, eps, weight_decay, decay_mask=None):
    """Decoupled AdamW on the packed subset, step index t >= 1:
    p <- p (1 - lr*wd);  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
    p <- p - lr * (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps).
    decay_mask (0/1 per element) switches weight decay off for norm gains."""
    wd = weight_decay if decay_mask is None else weight_decay * decay_mask
    p = p * (1.0 - lr * wd)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    p = p - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


def decay_mask_for(cfg, mask):
    """1 for matrix elements, 0 for RMSNorm gains, in packed order."""
    d = cfg["d_model"]
    parts = [np.full((hi - lo) * d, 0.0 if n.endswith("norm") else 1.0) for n, lo, hi in mask_segments(cfg, mask)]
    return np.concatenate(parts) if parts else np.zeros(0)


class LocalTrainer:
    """One node's state for Alg. 1's inner loop: all parameters, plus AdamW moments for I_train only."""

    def __init__(self, cfg, params, mask, storage="f64"):
        self.cfg, self.mask = cfg, mask
        self.params = to_f64(params)
        self.segs = mask_segments(cfg, mask)
        n = count_trainable(cfg, mask)
        self.m = np.zeros(n)
        self.v = np.zeros(n)
        self.master = pack(self.params, self.segs)
        self.t = 0
        self.decay = decay_mask_for(cfg, mask)
        self.storage = storage

    def step(self, tokens, targets, hp, restricted=False):
        """forward -> gradient on I_train -> AdamW on I_train.  Returns (loss, packed gradient)."""
        loss, cache = forward(self.cfg, self.params, tokens, targets)
        if restricted:
            g, _ = backward_restricted(self.cfg, self.params, cache, self.mask)
        else:
            g = masked_gradient(self.cfg, self.params, cache, self.mask)
        self.t += 1
        self.master, self.m, self.v = adamw_update(self.master, self.m, self.v, g, self.t, hp["lr"], hp["beta1"],
                                                   hp["beta2"], hp["eps"], hp["weight_decay"], self.decay)
        new = self.master
        if self.storage == "bf16":
            # mixed precision (Memory Usage paragraph): fp32/fp64 master kept, compute copy is its bf16 rounding
            f = new.astype(np.float32).view(np.uint32)
            f = (f + np.uint32(0x7FFF) + ((f >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
            new = f.view(np.float32).astype(F64)
        unpack_into(self.params, self.segs, new)
        return loss, g


def outer_step(theta_g, theta_l, others_sum, momentum_buf, lr, mu, m_count, nesterov=True):
    """Alg. 1, delta / normalisation / OuterOpt lines, for the node's own packed subset, in the
    pseudo-gradient convention: delta_own = theta_g - theta_l; delta = (delta_own + others_sum)/m;
    b <- mu b + delta;  theta_g <- theta_g - lr (delta + mu b)   [Nesterov]  or  - lr b  [plain momentum].
    Returns (new theta_g, new momentum buffer, delta)."""
    if m_count < 1:
        raise ValueError("count vector entries must be >= 1")
    delta = (theta_g - theta_l + (0.0 if others_sum is None else others_sum)) / m_count
    b = mu * momentum_buf + delta
    upd = delta + mu * b if nesterov else b
    return theta_g - lr * upd, b, delta
