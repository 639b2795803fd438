"""HIP path vs CPU fp64 oracle on the tiny fp32 configuration: loss, every trainable gradient, the updated
weights, frozen bytes, and the executed-FLOP counters, for the benchmark mask and the paper's masks."""
import numpy as np
import pytest

import pp_inputs as gen
from oracle import pp_oracle as O
from harness import HP, cosine, segment_slices, make_gpu_model, frozen_bytes_equal, expand_mask

pytestmark = pytest.mark.gpu

MASKS = {
    "ffn_quarter": lambda c: gen.ffn_slice_mask(c, node=0, n_slices=4),
    "ffn_quarter_node2": lambda c: gen.ffn_slice_mask(c, node=2, n_slices=4),
    "all": lambda c: dict(all=1),
    "paper_mlp": lambda c: gen.paper_mlp_mask(c, node=1, n_slices=4),
    "paper_mlp_heads": lambda c: gen.paper_mlp_mask(c, node=1, n_slices=2, slice_heads=True),
    "heads_only": lambda c: dict(gen.ffn_slice_mask(c, 0, 4), ffn_lo=0, ffn_hi=0, head_lo=1, head_hi=3),
    "lm_head_only": lambda c: dict(gen.ffn_slice_mask(c, 0, 4), ffn_lo=0, ffn_hi=0, train_lm_head=1),
}


@pytest.mark.parametrize("mname", list(MASKS))
def test_tiny_fp32_step_matches_oracle(mname):
    cfg = gen.make_config("tiny")
    weights = gen.make_weights(cfg, seed=1)
    tok, tgt = gen.make_tokens(cfg, seed=1)
    mask = MASKS[mname](cfg)
    omask = expand_mask(cfg, mask)
    print(f"case tiny/{mname}", flush=True)
    m = make_gpu_model(cfg, weights, mask)
    td, gd = m.upload_tokens(tok, tgt)
    loss_gpu = float(m.step(td, gd, HP).item())
    g_gpu = m.get_state("g")
    cnt = m.counters()

    tr = O.LocalTrainer(cfg, weights, omask)
    loss_ref, g_ref = tr.step(tok, tgt, HP)
    assert abs(loss_gpu - loss_ref) <= 1e-5 * abs(loss_ref), (loss_gpu, loss_ref)
    assert g_gpu.shape == g_ref.shape
    for name, off, n in segment_slices(cfg, omask):
        a, b = g_gpu[off:off + n], g_ref[off:off + n]
        assert cosine(a, b) >= 0.999, (name, cosine(a, b))
        assert np.max(np.abs(a - b)) <= 1e-4 * np.max(np.abs(b)) + 1e-9, name
    # FLOPs launched == closed form for the mask
    B, S = tok.shape
    _, cache = O.forward(cfg, O.to_f64(weights), tok, tgt)
    _, info = O.backward_restricted(cfg, O.to_f64(weights), cache, omask)
    assert cnt["flops_fwd"] == O.flops_forward(cfg, B, S)
    assert cnt["flops_bwd"] == info["flops_bwd"]
    # updated subset: fp32 master vs oracle's fp64 AdamW (step 1 moves every element by ~lr, so compare updates)
    p_gpu = m.get_state("p")
    upd_gpu = p_gpu - O.pack(O.to_f64(weights), tr.segs)
    upd_ref = tr.master - O.pack(O.to_f64(weights), tr.segs)
    big = np.abs(g_ref) > 1e-3 * np.max(np.abs(g_ref))          # elements whose gradient sign is well determined
    assert np.max(np.abs(upd_gpu[big] - upd_ref[big])) <= 2e-2 * HP["lr"]
    # weights written back == masters; frozen elements bit-identical
    assert frozen_bytes_equal(cfg, m, weights, mask) == []
    flat_now = O.pack({k: m.get_weight(k, s).astype(np.float64) for k, s in gen.tensor_shapes(cfg).items()}, tr.segs)
    assert np.array_equal(flat_now.astype(np.float32), p_gpu)
    m.close()


def test_tiny_three_steps_track_oracle_and_freeze_holds():
    cfg = gen.make_config("tiny")
    weights = gen.make_weights(cfg, seed=2)
    mask = gen.ffn_slice_mask(cfg, node=1, n_slices=4)
    m = make_gpu_model(cfg, weights, mask)
    tr = O.LocalTrainer(cfg, weights, mask)
    for h in range(3):
        tok, tgt = gen.make_tokens(cfg, seed=2, step=h)
        td, gd = m.upload_tokens(tok, tgt)
        lg = float(m.step(td, gd, HP).item())
        lr_, _ = tr.step(tok, tgt, HP)
        assert abs(lg - lr_) <= 1e-5 * abs(lr_), (h, lg, lr_)
    assert frozen_bytes_equal(cfg, m, weights, mask) == []
    p_gpu = m.get_state("p")
    assert np.max(np.abs(p_gpu - tr.master)) <= 0.1 * 3 * HP["lr"]
    m.close()


def test_ragged_batch_and_ignored_targets():
    """B and S below the maxima, with extra ignored positions."""
    cfg = gen.make_config("tiny")
    weights = gen.make_weights(cfg, seed=3)
    mask = gen.ffn_slice_mask(cfg, node=3, n_slices=4)
    tok, tgt = gen.make_tokens(cfg, seed=3, batch=3, seq=19)
    tgt[1, 5:9] = -1
    m = make_gpu_model(cfg, weights, mask)
    td, gd = m.upload_tokens(tok, tgt)
    lg = float(m.step(td, gd, None).item())
    g_gpu = m.get_state("g")
    tr = O.LocalTrainer(cfg, weights, mask)
    loss_ref, cache = O.forward(cfg, tr.params, tok, tgt)
    g_ref = O.masked_gradient(cfg, tr.params, cache, mask)
    assert abs(lg - loss_ref) <= 1e-5 * abs(loss_ref)
    assert cosine(g_gpu, g_ref) >= 0.99999
    # opt == NULL: no update happened
    assert frozen_bytes_equal(cfg, m, weights, dict(gen.ffn_slice_mask(cfg, 0, 4), ffn_lo=0, ffn_hi=0)) == []
    m.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_degenerate_batches(dtype):
    """The method's degenerate inputs: a single token (B = S = 1: one key per query, softmax of one element), and a batch
    whose targets are all ignored (no valid position: the loss is 0 by the mean-over-valid-positions convention, every
    gradient is 0 and an AdamW step with zero gradients only applies the decoupled weight decay)."""
    cfg = gen.make_config("tiny", dtype=dtype)
    weights = gen.make_weights(cfg, seed=4)
    mask = gen.paper_mlp_mask(cfg, 0, 4)
    tol = 1e-5 if dtype == "fp32" else 1e-2
    # one token
    tok, tgt = np.array([[5]], dtype=np.int32), np.array([[7]], dtype=np.int32)
    m = make_gpu_model(cfg, weights, mask)
    lg = float(m.step(*m.upload_tokens(tok, tgt), None).item())
    g_gpu = m.get_state("g")
    params = O.to_f64(weights)
    loss_ref, cache = O.forward(cfg, params, tok, tgt)
    g_ref = O.masked_gradient(cfg, params, cache, mask)
    assert abs(lg - loss_ref) <= tol * abs(loss_ref)
    assert cosine(g_gpu, g_ref) >= (0.99999 if dtype == "fp32" else 0.999)
    # nothing to predict
    tok, tgt = gen.make_tokens(cfg, seed=4, batch=2, seq=9)
    tgt[:] = -1
    lg = float(m.step(*m.upload_tokens(tok, tgt), None).item())
    assert lg == 0.0
    assert not np.any(m.get_state("g"))
    p_before = m.get_state("p").copy()
    m.step(*m.upload_tokens(tok, tgt), HP)
    tr = O.LocalTrainer(cfg, weights, mask)
    loss_o, g_o = tr.step(tok, tgt, HP)
    assert loss_o == 0.0 and not np.any(g_o)
    np.testing.assert_allclose(m.get_state("p"), tr.master, rtol=1e-6, atol=1e-9)
    assert np.any(m.get_state("p") != p_before)          # decayed
    m.close()
