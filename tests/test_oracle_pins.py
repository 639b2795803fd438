"""Pins for the CPU fp64 oracle: it is checked against things other than itself -- finite
differences, library routines on the cases that reduce to them, closed forms, invariants the
paper states, and the few numbers the paper prints.  No GPU needed."""
import math
import os

import numpy as np
import pytest
import torch

import pp_inputs as gen
from oracle import pp_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
HP = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def small_cfg(**over):
    c = gen.make_config("tiny", n_layers=2, d_model=32, n_heads=4, d_ff=64, vocab=50, batch=2, seq=12)
    c.update(over)
    return c


def setup(cfg, seed=3, std=0.2):
    params = O.to_f64(gen.make_weights(cfg, seed, std=std))
    # norm gains away from 1 so that a dropped gamma shows up
    for k in params:
        if k.endswith("norm"):
            params[k] = 1.0 + 0.1 * gen.normal(gen.stream_key(seed, gen.STREAM_MISC, gen.fnv1a64(k)), params[k].size)
    tok, tgt = gen.make_tokens(cfg, seed)
    return params, tok, tgt


def read_table(name):
    rows = []
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append([float(x) for x in line.split()])
    return rows


# ------------------------------------------------------------------ gradients: finite differences
def test_full_gradient_matches_central_differences():
    cfg = small_cfg()
    params, tok, tgt = setup(cfg)
    loss, cache = O.forward(cfg, params, tok, tgt)
    grads = O.backward_full(cfg, params, cache)
    h = 1e-5
    rng = np.random.default_rng(0)
    for name, w in params.items():
        flat = w.reshape(-1)
        idx = rng.choice(flat.size, size=min(6, flat.size), replace=False)
        if name == "embed":      # make sure sampled rows are tokens that occur
            used = np.unique(tok)
            idx = np.array([int(t) * cfg["d_model"] + int(j) for t, j in zip(used[:4], rng.integers(0, cfg["d_model"], 4))])
        for i in idx:
            old = flat[i]
            flat[i] = old + h
            lp, _ = O.forward(cfg, params, tok, tgt)
            flat[i] = old - h
            lm, _ = O.forward(cfg, params, tok, tgt)
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            an = grads[name].reshape(-1)[i]
            assert abs(fd - an) <= 1e-7 * max(1.0, abs(an)) + 2e-9, (name, i, fd, an)


# ------------------------------------------------------------------ building blocks vs library routines
def test_rmsnorm_matches_library():
    x = torch.randn(7, 32, dtype=torch.float64, generator=torch.Generator().manual_seed(1))
    g = torch.rand(32, dtype=torch.float64, generator=torch.Generator().manual_seed(2)) + 0.5
    ref = torch.nn.functional.rms_norm(x, (32,), weight=g, eps=1e-5)
    y, rstd = O.rmsnorm_fwd(x.numpy(), g.numpy(), 1e-5)
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-13)


def test_attention_matches_library_sdpa():
    gtr = torch.Generator().manual_seed(5)
    q, k, v = (torch.randn(2, 9, 3, 8, dtype=torch.float64, generator=gtr) for _ in range(3))
    ref = torch.nn.functional.scaled_dot_product_attention(
        q.permute(0, 2, 1, 3), k.permute(0, 2, 1, 3), v.permute(0, 2, 1, 3), is_causal=True).permute(0, 2, 1, 3)
    o, P = O.attention_fwd(q.numpy(), k.numpy(), v.numpy())
    np.testing.assert_allclose(o, ref.numpy(), rtol=1e-11, atol=1e-12)
    # rows of P are probability vectors supported on the causal prefix
    np.testing.assert_allclose(P.sum(-1), 1.0, rtol=1e-12)
    assert np.all(np.triu(P[0, 0], 1) == 0.0)


def test_attention_single_position_returns_v():
    rng = np.random.default_rng(0)
    q, k, v = (rng.standard_normal((1, 1, 2, 4)) for _ in range(3))
    o, _ = O.attention_fwd(q, k, v)
    np.testing.assert_allclose(o, v, rtol=0, atol=0)


def test_loss_matches_library_cross_entropy_and_lnV_at_init():
    cfg = gen.make_config("tiny")
    params = O.to_f64(gen.make_weights(cfg, 11))
    tok, tgt = gen.make_tokens(cfg, 11)
    loss, cache = O.forward(cfg, params, tok, tgt)
    ref = torch.nn.functional.cross_entropy(torch.from_numpy(cache["z"]), torch.from_numpy(tgt.reshape(-1)).long(),
                                            ignore_index=-1, reduction="mean")
    assert abs(loss - float(ref)) < 1e-12
    # N(0, 0.02) weights give near-uniform predictions: loss within 1% of ln V
    assert abs(loss - math.log(cfg["vocab"])) < 0.01 * math.log(cfg["vocab"])
    assert cache["n_valid"] == cfg["batch"] * (cfg["seq"] - 1)


def test_silu_matches_library():
    z = np.linspace(-8, 8, 41)
    np.testing.assert_allclose(O.silu(z), torch.nn.functional.silu(torch.from_numpy(z)).numpy(), rtol=1e-13)


# ------------------------------------------------------------------ rotary: closed forms
def test_rope_closed_forms():
    S, dh, base = 6, 8, 10000.0
    cos, sin = O.rope_tables(S, dh, base)
    # pair (i, i+dh/2) = (1, 0) at position p becomes (cos(p w_i), sin(p w_i)), w_i = base^(-2i/dh)
    x = np.zeros((1, S, 1, dh))
    x[..., 1] = 1.0
    y = O.rope_apply(x, cos, sin)
    w1 = base ** (-2.0 / dh)
    for p in range(S):
        assert abs(y[0, p, 0, 1] - math.cos(p * w1)) < 1e-14
        assert abs(y[0, p, 0, 1 + dh // 2] - math.sin(p * w1)) < 1e-14
    rng = np.random.default_rng(1)
    q = rng.standard_normal((1, S, 2, dh))
    k = rng.standard_normal((1, S, 2, dh))
    # position 0 is the identity; norms are preserved; inverse undoes it
    np.testing.assert_allclose(O.rope_apply(q, cos, sin)[:, 0], q[:, 0], atol=0)
    np.testing.assert_allclose(np.linalg.norm(O.rope_apply(q, cos, sin), axis=-1), np.linalg.norm(q, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(O.rope_apply(O.rope_apply(q, cos, sin), cos, sin, inverse=True), q, atol=1e-14)
    # relative-position property: <R_m q, R_n k> depends on m-n only
    qq = np.broadcast_to(q[:, :1], q.shape)
    kk = np.broadcast_to(k[:, :1], k.shape)
    rq, rk = O.rope_apply(qq, cos, sin), O.rope_apply(kk, cos, sin)
    d1 = np.sum(rq[0, 3, 0] * rk[0, 1, 0])
    d2 = np.sum(rq[0, 5, 0] * rk[0, 3, 0])
    assert abs(d1 - d2) < 1e-12


# ------------------------------------------------------------------ invariants of the forward
def test_causality_changing_a_token_leaves_earlier_logits_unchanged():
    cfg = small_cfg()
    params, tok, tgt = setup(cfg)
    _, c0 = O.forward(cfg, params, tok, tgt)
    tok2 = tok.copy()
    s = 7
    tok2[0, s] = (tok2[0, s] + 1) % cfg["vocab"]
    _, c1 = O.forward(cfg, params, tok2, tgt)
    S = cfg["seq"]
    assert np.array_equal(c0["z"][:s], c1["z"][:s])          # batch 0, positions < s
    assert not np.array_equal(c0["z"][s:S], c1["z"][s:S])
    assert np.array_equal(c0["z"][S:], c1["z"][S:])          # batch 1 untouched


def test_ffn_is_additive_over_hidden_unit_slices():
    """MLP(x) = sum_n V_n act(W_n x) (Parameter Slicing): zeroing all but slice n and summing over n
    reproduces the FFN output."""
    cfg = small_cfg(n_layers=1)
    params, tok, tgt = setup(cfg)
    _, c = O.forward(cfg, params, tok, tgt)
    ffn_out = c["xL"] - c["layers"][0]["xm"]
    n2 = c["layers"][0]["n2"]
    acc = 0
    F, N = cfg["d_ff"], 4
    for n in range(N):
        r = slice(n * F // N, (n + 1) * F // N)
        acc = acc + (O.silu(n2 @ params["layers.0.wg"][r].T) * (n2 @ params["layers.0.wu"][r].T)) @ params["layers.0.wd"][r]
    np.testing.assert_allclose(acc, ffn_out, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ the restricted backward
MASKS = {
    "ffn_slice": lambda c: gen.ffn_slice_mask(c, node=1, n_slices=4),
    "all": gen.all_mask,
    "paper_mlp": lambda c: gen.paper_mlp_mask(c, node=2, n_slices=4),
    "paper_mlp_heads": lambda c: gen.paper_mlp_mask(c, node=1, n_slices=2, slice_heads=True),
    "heads_only": lambda c: dict(gen.ffn_slice_mask(c, 0, 4), ffn_lo=0, ffn_hi=0, head_lo=1, head_hi=3),
    "wo_only": lambda c: dict(gen.ffn_slice_mask(c, 0, 4), ffn_lo=0, ffn_hi=0, train_wo=1),
    "lm_head_only": lambda c: dict(gen.ffn_slice_mask(c, 0, 4), ffn_lo=0, ffn_hi=0, train_lm_head=1),
    "norms_only": lambda c: dict(gen.ffn_slice_mask(c, 0, 4), ffn_lo=0, ffn_hi=0, train_norms=1),
}


@pytest.mark.parametrize("mname", list(MASKS))
def test_restricted_backward_equals_slice_of_full_gradient(mname):
    cfg = small_cfg()
    params, tok, tgt = setup(cfg)
    mask = MASKS[mname](cfg)
    _, cache = O.forward(cfg, params, tok, tgt)
    g_def = O.masked_gradient(cfg, params, cache, mask)
    g_res, info = O.backward_restricted(cfg, params, cache, mask)
    assert g_def.shape == g_res.shape == (O.count_trainable(cfg, mask),)
    np.testing.assert_allclose(g_res, g_def, rtol=1e-12, atol=1e-15)
    assert np.linalg.norm(g_def) > 0


def test_frozen_slices_still_carry_the_input_gradient():
    """The input gradient must include every slice (Appendix Partial Backward: 'full Jacobian'):
    dropping the frozen slices' contribution (the detach variant) gives a different, wrong gradient."""
    cfg = small_cfg()
    params, tok, tgt = setup(cfg)
    mask = gen.ffn_slice_mask(cfg, node=0, n_slices=4)
    _, cache = O.forward(cfg, params, tok, tgt)
    g, info = O.backward_restricted(cfg, params, cache, mask)
    full = O.backward_full(cfg, params, cache)
    # detach variant at the top layer: zero the frozen rows of wg/wu there and recompute layer 0's gradient
    p2 = {k: v.copy() for k, v in params.items()}
    fl, fh = mask["ffn_lo"], mask["ffn_hi"]
    c1 = cache["layers"][1]
    G = info["dx"][2]
    dA = G @ params["layers.1.wd"].T
    sg = 1 / (1 + np.exp(-c1["g"]))
    dG = dA * c1["u"] * (sg * (1 + c1["g"] * (1 - sg)))
    dU = dA * c1["g"] * sg
    dn2_full = dG @ params["layers.1.wg"] + dU @ params["layers.1.wu"]
    dn2_detached = dG[:, fl:fh] @ params["layers.1.wg"][fl:fh] + dU[:, fl:fh] @ params["layers.1.wu"][fl:fh]
    assert np.linalg.norm(dn2_full - dn2_detached) > 0.1 * np.linalg.norm(dn2_full)
    # and the oracle's layer-0 gradient is the full-Jacobian one
    seg = [s for s in O.mask_segments(cfg, mask) if s[0] == "layers.0.wg"][0]
    off = 0
    for s in O.mask_segments(cfg, mask):
        if s == seg:
            break
        off += (s[2] - s[1]) * cfg["d_model"]
    got = g[off:off + (fh - fl) * cfg["d_model"]].reshape(fh - fl, -1)
    np.testing.assert_allclose(got, full["layers.0.wg"][fl:fh], rtol=1e-12, atol=1e-15)


def test_backward_stops_at_lowest_trainable_parameter():
    cfg = small_cfg(n_layers=3)
    params, tok, tgt = setup(cfg)
    _, cache = O.forward(cfg, params, tok, tgt)
    _, info = O.backward_restricted(cfg, params, cache, gen.ffn_slice_mask(cfg, 0, 4))
    assert sorted(info["dx"]) == [1, 2, 3]          # no gradient wrt layer 0's input or the embedding output
    _, info = O.backward_restricted(cfg, params, cache, gen.all_mask(cfg))
    assert sorted(info["dx"]) == [0, 1, 2, 3]
    _, info = O.backward_restricted(cfg, params, cache, MASKS["lm_head_only"](cfg))
    assert info["dx"] == {} and info["flops_bwd"] == 2 * cfg["batch"] * cfg["seq"] * cfg["d_model"] * cfg["vocab"]


# ------------------------------------------------------------------ the detach ablation (Appendix "Additional Results")
def _autograd_model_loss(cfg, tparams, tok, tgt, kept):
    """The decoder written again with library tensor ops (fp64, autograd), the FFN activations of the hidden units
    outside `kept` detached from the graph: their forward value is used, their Jacobian is dropped."""
    F_ = torch.nn.functional
    B, S = tok.shape
    d, h, L = cfg["d_model"], cfg["n_heads"], cfg["n_layers"]
    dh = d // h
    half = dh // 2
    pos = torch.arange(S, dtype=torch.float64)[:, None]
    ang = pos * cfg["rope_base"] ** (-2.0 * torch.arange(half, dtype=torch.float64) / dh)[None, :]
    cos, sin = torch.cos(ang)[None, :, None, :], torch.sin(ang)[None, :, None, :]

    def rot(t):
        a, b = t[..., :half], t[..., half:]
        return torch.cat([a * cos - b * sin, a * sin + b * cos], dim=-1)

    keep = torch.zeros(cfg["d_ff"], dtype=torch.bool)
    for lo, hi in kept:
        keep[lo:hi] = True
    x = tparams["embed"][torch.from_numpy(tok.reshape(-1)).long()]
    for l in range(L):
        p = f"layers.{l}."
        n1 = F_.rms_norm(x, (d,), weight=tparams[p + "attn_norm"], eps=cfg["rms_eps"])
        qkv = n1 @ tparams[p + "wqkv"].T
        q = rot(qkv[:, :d].reshape(B, S, h, dh)).transpose(1, 2)
        k = rot(qkv[:, d:2 * d].reshape(B, S, h, dh)).transpose(1, 2)
        v = qkv[:, 2 * d:].reshape(B, S, h, dh).transpose(1, 2)
        o = F_.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(B * S, d)
        xm = x + o @ tparams[p + "wo"].T
        n2 = F_.rms_norm(xm, (d,), weight=tparams[p + "ffn_norm"], eps=cfg["rms_eps"])
        a = F_.silu(n2 @ tparams[p + "wg"].T) * (n2 @ tparams[p + "wu"].T)
        a = torch.where(keep[None, :], a, a.detach())
        x = xm + a @ tparams[p + "wd"]
    z = F_.rms_norm(x, (d,), weight=tparams["final_norm"], eps=cfg["rms_eps"]) @ tparams["lm_head"].T
    return F_.cross_entropy(z, torch.from_numpy(tgt.reshape(-1)).long(), ignore_index=-1)


@pytest.mark.parametrize("mname,extra", [("ffn_slice", None), ("ffn_slice", (48, 64)), ("paper_mlp", (0, 16)),
                                         ("paper_mlp_heads", None)])
def test_detach_ablation_matches_autograd_with_detached_units(mname, extra):
    """detach-all-but-k (extra None -> empty range) and k + one more slice: the oracle's gradient over I_train equals
    what library autograd gives when the activations of all other hidden units are detached."""
    cfg = small_cfg(n_layers=3)
    params, tok, tgt = setup(cfg)
    mask = MASKS[mname](cfg)
    ex = extra or (0, 0)
    loss, cache = O.forward(cfg, params, tok, tgt)
    g, info = O.backward_restricted(cfg, params, cache, mask, jacobian_extra=ex)
    tparams = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in params.items()}
    tl = _autograd_model_loss(cfg, tparams, tok, tgt, [(mask["ffn_lo"], mask["ffn_hi"]), ex])
    assert abs(float(tl.detach()) - loss) <= 1e-12 * abs(loss)
    tl.backward()
    ref = O.pack({k: v.grad.numpy() for k, v in tparams.items()}, O.mask_segments(cfg, mask))
    np.testing.assert_allclose(g, ref, rtol=1e-9, atol=1e-13)
    # and it is a different gradient from the method's (full Jacobian) wherever something trainable lies below an FFN
    g_full, info_full = O.backward_restricted(cfg, params, cache, mask)
    assert np.linalg.norm(g - g_full) > 1e-3 * np.linalg.norm(g_full)
    # executed FLOPs: per layer whose FFN input gradient is formed, 6 T d (F - kept) fewer
    T, d, F = tok.size, cfg["d_model"], cfg["d_ff"]
    n_kept = (mask["ffn_hi"] - mask["ffn_lo"]) + (ex[1] - ex[0])
    layers_with_dn = cfg["n_layers"] if mname != "ffn_slice" else cfg["n_layers"] - 1
    assert info_full["flops_bwd"] - info["flops_bwd"] == layers_with_dn * 6 * T * d * (F - n_kept)


def test_detach_ablation_with_every_unit_kept_is_the_method():
    cfg = small_cfg()
    params, tok, tgt = setup(cfg)
    mask = gen.ffn_slice_mask(cfg, node=0, n_slices=4)
    _, cache = O.forward(cfg, params, tok, tgt)
    g0, i0 = O.backward_restricted(cfg, params, cache, mask)
    g1, i1 = O.backward_restricted(cfg, params, cache, mask, jacobian_extra=(mask["ffn_hi"], cfg["d_ff"]))
    np.testing.assert_array_equal(g0, g1)
    assert i0["flops_bwd"] == i1["flops_bwd"]


# ------------------------------------------------------------------ FLOP accounting
@pytest.mark.parametrize("name,N", [("tiny", 4), ("tiny", 2)])
def test_flop_counter_equals_closed_form(name, N):
    cfg = gen.make_config(name)
    params = O.to_f64(gen.make_weights(cfg, 1))
    tok, tgt = gen.make_tokens(cfg, 1)
    B, S = tok.shape
    _, cache = O.forward(cfg, params, tok, tgt)
    _, info = O.backward_restricted(cfg, params, cache, gen.ffn_slice_mask(cfg, 0, N))
    assert info["flops_bwd"] == O.flops_backward_ffn_slice(cfg, B, S, 1.0 / N)
    _, info = O.backward_restricted(cfg, params, cache, gen.all_mask(cfg))
    assert info["flops_bwd"] == O.flops_backward_all(cfg, B, S) == 2 * O.flops_forward(cfg, B, S)


def test_closed_form_values_at_benchmark_shapes():
    c3 = gen.make_config("1p3b")
    f = O.flops_forward(c3, 8, 2048)
    tot32 = f + O.flops_backward_ffn_slice(c3, 8, 2048, 1 / 32)
    tot8 = f + O.flops_backward_ffn_slice(c3, 8, 2048, 1 / 8)
    full = f + O.flops_backward_all(c3, 8, 2048)
    assert abs(tot32 / 1.1853e14 - 1) < 1e-3 and abs(tot8 / 1.2229e14 - 1) < 1e-3 and abs(full / 1.7467e14 - 1) < 1e-3
    c1 = gen.make_config("tiny")
    assert abs((O.flops_forward(c1, 4, 32) + O.flops_backward_ffn_slice(c1, 4, 32, 0.25)) / 6.82e7 - 1) < 2e-3


def test_paper_flop_formulas_reproduce_printed_saving_and_rho1_identity():
    (B, S, H, L, Dff, V, N, printed), = read_table("paper_flops_saving.txt")
    B, S, H, L, Dff, V, N = map(int, (B, S, H, L, Dff, V, N))
    f1, b1 = O.paper_flops(B, S, H, L, Dff, V, 1.0, 1.0)
    fN, bN = O.paper_flops(B, S, H, L, Dff, V, 1.0 / N, 1.0)
    saving = 100 * (1 - (fN + bN) / (f1 + b1))
    assert round(saving) == printed and abs(saving - 14.65) < 0.01
    # rho = 1: backward of the MHA and FFN blocks is exactly twice their forward (Appendix, MHA backward)
    emb = B * S * H
    out = 2 * B * S * H * V + 3 * B * S * V
    assert b1 - 2 * emb - 2 * out == 2 * (f1 - emb - out)


def test_paper_trainable_parameter_column():
    for n_mlp, n_heads, printed in read_table("paper_table1_trainable_params.txt"):
        val = O.paper_trainable_params(24, 2048, 32000, n_mlp, n_heads) / 1e9
        digits = 1 if printed == 1.3 else 2
        assert round(val, digits) == printed, (n_mlp, n_heads, val)


def test_comm_time_model():
    (K, M, B, printed), = read_table("paper_comm_time.txt")
    assert abs(O.comm_time(int(K), M * 1e9, B * 1e9) - printed) < 0.005


def test_mask_parameter_count_swiglu():
    cfg = gen.make_config("1p3b")
    assert O.count_trainable(cfg, gen.ffn_slice_mask(cfg, 0, 32)) == 3 * 2048 * 256 * 24 == 37748736
    total = sum(int(np.prod(s)) for s in gen.tensor_shapes(cfg).values())
    assert O.count_trainable(cfg, gen.all_mask(cfg)) == total


# ------------------------------------------------------------------ optimizers
def test_adamw_step1_closed_form_and_library():
    rng = np.random.default_rng(4)
    p0 = rng.standard_normal(200)
    g = rng.standard_normal(200) * 1e-2
    p1, m1, v1 = O.adamw_update(p0, np.zeros(200), np.zeros(200), g, 1, **HP)
    np.testing.assert_allclose(p1, p0 * (1 - HP["lr"] * HP["weight_decay"]) - HP["lr"] * g / (np.abs(g) + HP["eps"]), rtol=1e-12)
    # zero gradient, no decay: unchanged
    pz, _, _ = O.adamw_update(p0, np.zeros(200), np.zeros(200), np.zeros(200), 1, 1e-3, 0.9, 0.95, 1e-8, 0.0)
    assert np.array_equal(pz, p0)
    # five steps against the library optimizer
    tp = torch.tensor(p0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"], weight_decay=HP["weight_decay"])
    p, m, v = p0, np.zeros(200), np.zeros(200)
    for t in range(1, 6):
        gt = rng.standard_normal(200) * 1e-2
        tp.grad = torch.tensor(gt)
        opt.step()
        p, m, v = O.adamw_update(p, m, v, gt, t, **HP)
    np.testing.assert_allclose(p, tp.detach().numpy(), rtol=1e-10, atol=1e-13)


def test_outer_step_closed_form_and_library_nesterov():
    rng = np.random.default_rng(7)
    n = 64
    tg, tl = rng.standard_normal(n), rng.standard_normal(n)
    others = rng.standard_normal(n) * 1e-2
    lr, mu, m = 0.7, 0.9, 32
    new, b, delta = O.outer_step(tg, tl, others, np.zeros(n), lr, mu, m)
    np.testing.assert_allclose(delta, (tg - tl + others) / m, rtol=1e-14)
    np.testing.assert_allclose(new, tg - lr * (1 + mu) * delta, rtol=1e-13)      # step 1, b0 = 0
    # several rounds against library Nesterov SGD fed the same pseudo-gradients
    tp = torch.tensor(tg, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([tp], lr=lr, momentum=mu, nesterov=True)
    cur, buf = tg, np.zeros(n)
    for r in range(4):
        tl = cur + rng.standard_normal(n) * 1e-2
        others = rng.standard_normal(n) * 1e-2
        tp.grad = torch.tensor((cur - tl + others) / m)
        opt.step()
        cur, buf, _ = O.outer_step(cur, tl, others, buf, lr, mu, m)
        np.testing.assert_allclose(cur, tp.detach().numpy(), rtol=1e-12, atol=1e-14)
    with pytest.raises(ValueError):
        O.outer_step(tg, tl, None, np.zeros(n), lr, mu, 0)


def test_frozen_parameters_unchanged_after_H_steps_and_subset_moves():
    cfg = small_cfg()
    params, tok, tgt = setup(cfg)
    mask = gen.ffn_slice_mask(cfg, node=1, n_slices=4)
    tr = O.LocalTrainer(cfg, params, mask)
    before = {k: v.copy() for k, v in tr.params.items()}
    losses = []
    for h in range(3):
        tok, tgt = gen.make_tokens(cfg, 3, step=0)
        losses.append(tr.step(tok, tgt, HP, restricted=(h % 2 == 1))[0])
    fl, fh = mask["ffn_lo"], mask["ffn_hi"]
    for k, v in tr.params.items():
        if k.split(".")[-1] in ("wg", "wu", "wd"):
            keep = np.ones(v.shape[0], bool)
            keep[fl:fh] = False
            assert np.array_equal(v[keep], before[k][keep])
            assert not np.array_equal(v[fl:fh], before[k][fl:fh])
        else:
            assert np.array_equal(v, before[k]), k
    assert losses[2] < losses[0]          # same batch three times: the subset update lowers its loss


def test_definition_and_restricted_paths_give_same_training_trajectory():
    cfg = small_cfg()
    params, tok, tgt = setup(cfg)
    mask = gen.paper_mlp_mask(cfg, node=0, n_slices=4)
    a, b = O.LocalTrainer(cfg, params, mask), O.LocalTrainer(cfg, params, mask)
    for h in range(2):
        tok, tgt = gen.make_tokens(cfg, 5, step=h)
        la, _ = a.step(tok, tgt, HP, restricted=False)
        lb, _ = b.step(tok, tgt, HP, restricted=True)
        assert abs(la - lb) < 1e-12
    for k in a.params:
        np.testing.assert_allclose(a.params[k], b.params[k], rtol=1e-9, atol=1e-12)


# ------------------------------------------------------------------ the trainer as a whole: library autograd + library AdamW
def _leaf_params(cfg, params, mask):
    """torch leaves for a mask: every whole trainable tensor is one leaf; a sliced FFN tensor is three row blocks
    (below / trainable / above) of which only the middle one is a leaf that the optimizer sees.  Returns
    (tensors for the model, decayed leaves, undecayed leaves, readers name -> callable giving the full array)."""
    fl, fh = mask["ffn_lo"], mask["ffn_hi"]
    hl, hh = mask["head_lo"], mask["head_hi"]
    d, dh = cfg["d_model"], cfg["d_model"] // cfg["n_heads"]
    model, decay, no_decay = {}, [], []
    for name, w in params.items():
        kind = name.split(".")[-1]
        t = lambda a, rg: torch.tensor(np.array(a), dtype=torch.float64, requires_grad=rg)
        if kind in ("wg", "wu", "wd") and fh > fl:
            lo, mid, hi = t(w[:fl], False), t(w[fl:fh], True), t(w[fh:], False)
            decay.append(mid)
            model[name] = (lo, mid, hi)
        elif kind == "wqkv" and hh > hl:
            blocks = []
            for blk in range(3):
                r0, r1 = blk * d + hl * dh, blk * d + hh * dh
                a, b, c = t(w[blk * d:r0], False), t(w[r0:r1], True), t(w[r1:(blk + 1) * d], False)
                decay.append(b)
                blocks += [a, b, c]
            model[name] = tuple(blocks)
        else:
            flag = {"embed": "train_embed", "lm_head": "train_lm_head", "wo": "train_wo"}.get(kind, "train_norms" if kind.endswith("norm") else None)
            leaf = t(w, bool(flag and mask.get(flag)))
            if leaf.requires_grad:
                (no_decay if kind.endswith("norm") else decay).append(leaf)
            model[name] = (leaf,)
    return model, decay, no_decay


@pytest.mark.parametrize("mname", ["all", "paper_mlp", "paper_mlp_heads", "ffn_slice"])
def test_local_trainer_matches_library_autograd_with_adamw_parameter_groups(mname):
    """Three inner steps of Alg. 1 by the oracle's LocalTrainer against library autograd + library AdamW with two
    parameter groups (matrices decayed, norm gains not).  The norm gains sit between the matrices in the packed order,
    so a decay vector that is misaligned with that order, or that decays the gains, moves parameters differently; the
    frozen row blocks are not leaves of the library optimizer at all, so they must stay exactly as they were."""
    cfg = small_cfg(n_layers=2)
    params, _, _ = setup(cfg)
    mask = MASKS[mname](cfg)
    model, decay, no_decay = _leaf_params(cfg, params, mask)
    hp = dict(HP, lr=3e-3, weight_decay=0.3)          # decay large enough that a wrong decay flag shows at once
    groups = [dict(params=decay, weight_decay=hp["weight_decay"])]
    if no_decay:
        groups.append(dict(params=no_decay, weight_decay=0.0))
    opt = torch.optim.AdamW(groups, lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"])
    tr = O.LocalTrainer(cfg, params, mask)
    assert tr.decay.size == tr.master.size
    n_gain_elems = sum(x.numel() for x in no_decay)
    assert int((tr.decay == 0).sum()) == n_gain_elems and int((tr.decay == 1).sum()) == tr.master.size - n_gain_elems
    for step in range(3):
        tok, tgt = gen.make_tokens(cfg, 17, step=step)
        loss_o, _ = tr.step(tok, tgt, hp, restricted=(step == 1))
        opt.zero_grad()
        tparams = {k: (v[0] if len(v) == 1 else torch.cat(v, dim=0)) for k, v in model.items()}
        loss_t = _autograd_model_loss(cfg, tparams, tok, tgt, [(0, cfg["d_ff"])])
        assert abs(float(loss_t.detach()) - loss_o) <= 1e-11 * abs(loss_o), step
        loss_t.backward()
        opt.step()
    for k, v in model.items():
        now = (v[0] if len(v) == 1 else torch.cat(v, dim=0)).detach().numpy()
        np.testing.assert_allclose(tr.params[k], now, rtol=1e-8, atol=1e-11, err_msg=k)


def test_local_trainer_bf16_storage_keeps_master_and_rounds_compute_copy_like_the_library():
    """Mixed precision of the Memory Usage paragraph (full-precision master, bf16 compute copy): after a step with
    storage='bf16' the master equals the full-precision trainer's master (same start, same gradient), the trainable
    rows of the parameters are the library's round-to-nearest-even bf16 cast of that master, and frozen rows are untouched."""
    cfg = small_cfg()
    params = O.to_f64(gen.make_weights(dict(cfg, dtype="bf16"), seed=8, std=0.2))
    mask = gen.paper_mlp_mask(cfg, node=1, n_slices=4)
    tok, tgt = gen.make_tokens(cfg, 8)
    a = O.LocalTrainer(cfg, params, mask)
    b = O.LocalTrainer(cfg, params, mask, storage="bf16")
    la, ga = a.step(tok, tgt, HP)
    lb, gb = b.step(tok, tgt, HP)
    assert la == lb and np.array_equal(ga, gb)
    np.testing.assert_array_equal(a.master, b.master)
    want = torch.tensor(b.master, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got = O.pack(b.params, b.segs)
    np.testing.assert_array_equal(got, want)
    assert np.any(got != b.master)                       # the compute copy really is coarser than the master
    np.testing.assert_array_equal(O.pack(a.params, a.segs), a.master)
    fl, fh = mask["ffn_lo"], mask["ffn_hi"]
    keep = np.ones(cfg["d_ff"], bool)
    keep[fl:fh] = False
    for l in range(cfg["n_layers"]):
        for nm in ("wg", "wu", "wd"):
            k = f"layers.{l}.{nm}"
            assert np.array_equal(b.params[k][keep], params[k][keep])
    # the next step starts from the rounded copy: its loss differs from the full-precision trainer's
    tok2, tgt2 = gen.make_tokens(cfg, 8, step=1)
    assert a.step(tok2, tgt2, HP)[0] != b.step(tok2, tgt2, HP)[0]
