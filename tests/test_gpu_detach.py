"""The detach-all-but-k (+ one more slice) ablation of Appendix "Additional Results" on the GPU against the oracle's
same option: gradients over I_train, executed FLOPs, frozen bytes; switching it off restores the method's gradient."""
import numpy as np
import pytest

import pp_inputs as gen
from oracle import pp_oracle as O
from harness import HP, cosine, segment_slices, make_gpu_model, frozen_bytes_equal

pytestmark = pytest.mark.gpu


def _grad(m, tok, tgt):
    td, gd = m.upload_tokens(tok, tgt)
    loss = float(m.step(td, gd, None).item())          # gradients only, no update
    return loss, m.get_state("g"), m.counters()


@pytest.mark.parametrize("mname,node,extra_slice", [("ffn", 1, None), ("ffn", 0, 3), ("paper_mlp", 2, 0)])
def test_tiny_fp32_detach_matches_oracle(mname, node, extra_slice):
    cfg = gen.make_config("tiny")
    F, N = cfg["d_ff"], 4
    weights = gen.make_weights(cfg, seed=4)
    tok, tgt = gen.make_tokens(cfg, seed=4)
    mask = gen.ffn_slice_mask(cfg, node, N) if mname == "ffn" else gen.paper_mlp_mask(cfg, node, N)
    extra = (0, 0) if extra_slice is None else (extra_slice * F // N, (extra_slice + 1) * F // N)
    print(f"case detach tiny/{mname}/k={node}/g={extra_slice}", flush=True)
    m = make_gpu_model(cfg, weights, mask)
    params = O.to_f64(weights)
    loss_ref, cache = O.forward(cfg, params, tok, tgt)
    g_full, info_full = O.backward_restricted(cfg, params, cache, mask)
    g_ref, info = O.backward_restricted(cfg, params, cache, mask, jacobian_extra=extra)

    m.set_jacobian_slices(1, *extra)
    loss, g, cnt = _grad(m, tok, tgt)
    assert abs(loss - loss_ref) <= 1e-5 * abs(loss_ref)
    for name, off, n in segment_slices(cfg, mask):
        a, b = g[off:off + n], g_ref[off:off + n]
        assert cosine(a, b) >= 0.999, (name, cosine(a, b))
        assert np.max(np.abs(a - b)) <= 1e-4 * np.max(np.abs(b)) + 1e-9, name
    assert cnt["flops_bwd"] == info["flops_bwd"] < info_full["flops_bwd"]
    # the ablation is a different gradient; switching it off gives the method's again
    assert np.linalg.norm(g - g_full) > 1e-3 * np.linalg.norm(g_full)
    m.set_jacobian_slices(0)
    _, g0, cnt0 = _grad(m, tok, tgt)
    assert np.max(np.abs(g0 - g_full)) <= 1e-4 * np.max(np.abs(g_full)) + 1e-9
    assert cnt0["flops_bwd"] == info_full["flops_bwd"]
    assert frozen_bytes_equal(cfg, m, weights, mask) == []
    m.close()


@pytest.mark.parametrize("plain,recompute", [(False, 0), (True, 0), (False, 1)])
def test_small_bf16_detach_matches_oracle(plain, recompute):
    """bf16, several GEMM tiles (T = 384, d = 256, slice of 128 hidden units + one more slice), both kernel paths and the
    recomputation mode; then one update step: frozen bytes unchanged."""
    cfg = gen.make_config("tiny", n_layers=3, d_model=256, n_heads=2, d_ff=512, vocab=512, batch=2, seq=192, dtype="bf16")
    cfg = dict(cfg, recompute=recompute)
    weights = gen.make_weights(cfg, seed=6)
    tok, tgt = gen.make_tokens(cfg, seed=6)
    mask = gen.paper_mlp_mask(cfg, 1, 4)
    extra = (384, 512)
    print(f"case detach small-bf16/plain={plain}/recompute={recompute}", flush=True)
    m = make_gpu_model(cfg, weights, mask, force_plain=plain)
    m.set_jacobian_slices(1, *extra)
    loss, g, cnt = _grad(m, tok, tgt)
    params = O.to_f64(weights)
    loss_ref, cache = O.forward(cfg, params, tok, tgt)
    g_ref, info = O.backward_restricted(cfg, params, cache, mask, jacobian_extra=extra)
    g_full, _ = O.backward_restricted(cfg, params, cache, mask)
    assert abs(loss - loss_ref) <= 1e-2 * abs(loss_ref)
    worst, worst_full = 1.0, 1.0
    for name, off, n in segment_slices(cfg, mask):
        worst = min(worst, cosine(g[off:off + n], g_ref[off:off + n]))
        worst_full = min(worst_full, cosine(g[off:off + n], g_full[off:off + n]))
    print(f"worst cosine vs ablation oracle {worst:.6f}, vs full-Jacobian oracle {worst_full:.6f}", flush=True)
    assert worst >= 0.999
    assert worst_full < 0.999          # the tolerance separates the ablation from the method
    assert cnt["flops_bwd"] == info["flops_bwd"]
    td, gd = m.upload_tokens(tok, tgt)
    m.step(td, gd, HP).item()
    assert frozen_bytes_equal(cfg, m, weights, mask) == []
    m.close()


def test_detach_argument_checks():
    import paper_2509_22418_amd as pp
    cfg = gen.make_config("tiny")
    weights = gen.make_weights(cfg, seed=4)
    tok, tgt = gen.make_tokens(cfg, seed=4)
    m = make_gpu_model(cfg, weights, gen.ffn_slice_mask(cfg, 0, 4))
    F = cfg["d_ff"]
    for bad in [(2, 0, 0), (1, -8, 0), (1, 16, 8), (1, 0, F + 8), (1, 4, 12)]:
        with pytest.raises(pp.PPError):
            m.set_jacobian_slices(*bad)
    td, gd = m.upload_tokens(tok, tgt)
    m.set_jacobian_slices(1, 0, 8)          # overlaps the trainable slice [0, F/4): refused by the step
    with pytest.raises(pp.PPError):
        m.step(td, gd, None)
    m.set_jacobian_slices(0)
    m.step(td, gd, None).item()
    m.close()
    m2 = make_gpu_model(cfg, weights, dict(gen.ffn_slice_mask(cfg, 0, 4), ffn_lo=0, ffn_hi=0, train_lm_head=1))
    m2.set_jacobian_slices(1)          # no trainable FFN slice: refused by the step
    with pytest.raises(pp.PPError):
        m2.step(*m2.upload_tokens(tok, tgt), None)
    m2.close()
