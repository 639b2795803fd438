"""Outer pseudo-gradient step (Alg. 1: delta, count normalisation, Nesterov OuterOpt) and the on-device synthetic
deltas, HIP path vs oracle / host generator."""
import numpy as np
import pytest
import torch

import pp_inputs as gen
import paper_2509_22418_amd as pp
from oracle import pp_oracle as O
from harness import HP, make_gpu_model, frozen_bytes_equal

pytestmark = pytest.mark.gpu

SMALL = dict(n_layers=2, d_model=256, n_heads=2, d_ff=512, vocab=512, batch=2, seq=64, dtype="bf16")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_outer_step_matches_oracle(dtype):
    cfg = gen.make_config("tiny", **dict(SMALL, dtype=dtype))
    weights = gen.make_weights(cfg, seed=21)
    mask = gen.ffn_slice_mask(cfg, 2, 4)
    m = make_gpu_model(cfg, weights, mask)
    segs = O.mask_segments(cfg, mask)
    theta_g0 = O.pack(O.to_f64(weights), segs)
    n = theta_g0.size
    for h in range(2):          # two local steps so that theta_l != theta_g
        tok, tgt = gen.make_tokens(cfg, seed=21, step=h)
        m.step(*m.upload_tokens(tok, tgt), HP)
    names = gen.tensor_shapes(cfg)
    theta_l = O.pack({k: m.get_weight(k, s).astype(np.float64) for k, s in names.items()}, segs)
    assert np.any(theta_l != theta_g0)
    keys = [gen.stream_key(77, gen.STREAM_DELTAS, j + 1) for j in range(31)]
    others_ref = gen.synthetic_delta_sum(77, n, 31, 1e-4)
    tg = torch.from_numpy(theta_g0.astype(np.float32)).cuda()
    mom = torch.zeros(n, dtype=torch.float32, device="cuda")
    others = torch.empty(n, dtype=torch.float32, device="cuda")
    delta = torch.empty(n, dtype=torch.float32, device="cuda")
    pp.pp_synth_delta_sum(m.h, others.data_ptr(), n, keys, 1e-4)
    torch.cuda.synchronize()
    got_others = others.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got_others - others_ref)) <= 1e-6 * np.max(np.abs(others_ref))          # fp32 rounding of an fp64 sum
    buf = np.zeros(n)
    cur = theta_g0.astype(np.float32).astype(np.float64)
    for rnd, (lr, mu, cnt) in enumerate([(0.7, 0.9, 32.0), (0.4, 0.9, 1.0)]):
        opt = pp.PPOuter(lr, mu, 1, cnt)
        pp.pp_outer_delta(m.h, tg.data_ptr(), mom.data_ptr(), others.data_ptr(), opt, delta.data_ptr())
        torch.cuda.synchronize()
        ref_new, buf, ref_delta = O.outer_step(cur, theta_l, got_others, buf, lr, mu, cnt)
        np.testing.assert_allclose(delta.cpu().numpy(), ref_delta, rtol=2e-5, atol=1e-9)
        np.testing.assert_allclose(tg.cpu().numpy(), ref_new, rtol=2e-6, atol=1e-8)
        np.testing.assert_allclose(mom.cpu().numpy(), buf, rtol=2e-5, atol=1e-9)
        # the local copy restarts from the new global values: masters == theta_g, weights == storage rounding of it
        assert np.array_equal(m.get_state("p"), tg.cpu().numpy())
        now = O.pack({k: m.get_weight(k, s).astype(np.float64) for k, s in names.items()}, segs)
        expect = tg.cpu().numpy()
        expect = gen.round_to_bf16(expect) if dtype == "bf16" else expect
        assert np.array_equal(now.astype(np.float32), expect)
        theta_l, cur = now, tg.cpu().numpy().astype(np.float64)
    assert frozen_bytes_equal(cfg, m, weights, mask) == []
    wd = m.get_weight("layers.1.wd", (cfg["d_ff"], cfg["d_model"]))
    assert np.array_equal(wd.T, m.get_weight("shadow.layers.1.wd", (cfg["d_model"], cfg["d_ff"])))
    # error paths
    lib = pp.load_library()
    bad = pp.PPOuter(0.7, 0.9, 1, 0.0)
    import ctypes
    assert lib.pp_outer_delta(m.h, tg.data_ptr(), mom.data_ptr(), None, ctypes.byref(bad), None) == -1
    m.close()


def test_outer_step_by_layer_group_touches_only_the_group():
    """Streaming synchronisation (Experimental Setup): one call updates the packed elements of one group of layers (or of
    the embeddings / output norm / head) by the same formulas and leaves every other element of theta_g, the momentum
    buffer, the fp32 masters and the weights bit-identical.  Mask = the paper's MLP-only slicing (everything outside the
    FFN trainable + one FFN slice), so all three kinds of packed range occur."""
    cfg = gen.make_config("tiny", **dict(SMALL, n_layers=3))
    weights = gen.make_weights(cfg, seed=23)
    mask = gen.paper_mlp_mask(cfg, 1, 4)
    m = make_gpu_model(cfg, weights, mask)
    segs = O.mask_segments(cfg, mask)
    d = cfg["d_model"]
    # packed element range of every segment, and which group it belongs to
    offs, o = [], 0
    for name, lo, hi in segs:
        n_el = (hi - lo) * (d if "norm" not in name else d)
        layer = int(name.split(".")[1]) if name.startswith("layers.") else -1
        offs.append((layer, o, o + n_el)); o += n_el
    theta_g0 = O.pack(O.to_f64(weights), segs)
    n = theta_g0.size
    assert o == n
    for h in range(2):
        tok, tgt = gen.make_tokens(cfg, seed=23, step=h)
        m.step(*m.upload_tokens(tok, tgt), HP)
    names = gen.tensor_shapes(cfg)
    read_weights = lambda: O.pack({k: m.get_weight(k, s).astype(np.float64) for k, s in names.items()}, segs)
    rng = np.random.default_rng(5)
    others_h = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    tg = torch.from_numpy(theta_g0.astype(np.float32)).cuda()
    mom = torch.from_numpy((rng.standard_normal(n) * 1e-3).astype(np.float32)).cuda()
    others = torch.from_numpy(others_h).cuda()
    delta = torch.full((n,), 7.0, dtype=torch.float32, device="cuda")
    for (l0, l1, ends) in [(1, 2, 0), (0, 0, 1), (0, 3, 0)]:
        sel = np.zeros(n, dtype=bool)
        for layer, a, b in offs:
            if (layer >= 0 and l0 <= layer < l1) or (layer < 0 and ends):
                sel[a:b] = True
        assert sel.any() and not sel.all()
        tg0, mom0, p0, w0 = tg.cpu().numpy(), mom.cpu().numpy(), m.get_state("p"), read_weights()
        delta.fill_(7.0)
        opt = pp.PPOuter(0.7, 0.9, 1, 4.0)
        pp.pp_outer_delta_group(m.h, l0, l1, ends, tg.data_ptr(), mom.data_ptr(), others.data_ptr(), opt, delta.data_ptr())
        torch.cuda.synchronize()
        ref_new, ref_b, ref_delta = O.outer_step(tg0.astype(np.float64), w0, others_h.astype(np.float64), mom0.astype(np.float64), 0.7, 0.9, 4.0)
        tg1, mom1, p1, w1, dl = tg.cpu().numpy(), mom.cpu().numpy(), m.get_state("p"), read_weights(), delta.cpu().numpy()
        np.testing.assert_allclose(tg1[sel], ref_new[sel], rtol=2e-6, atol=1e-8)
        np.testing.assert_allclose(mom1[sel], ref_b[sel], rtol=2e-5, atol=1e-9)
        np.testing.assert_allclose(dl[sel], ref_delta[sel], rtol=2e-5, atol=1e-9)
        assert np.array_equal(p1[sel], tg1[sel])
        assert np.array_equal(w1[sel].astype(np.float32), gen.round_to_bf16(tg1[sel]))
        # outside the group: nothing moved
        assert np.array_equal(tg1[~sel], tg0[~sel]) and np.array_equal(mom1[~sel], mom0[~sel])
        assert np.array_equal(p1[~sel], p0[~sel]) and np.array_equal(w1[~sel], w0[~sel])
        assert np.all(dl[~sel] == 7.0)
    lib = pp.load_library()
    assert lib.pp_outer_delta_group(m.h, 2, 1, 0, tg.data_ptr(), mom.data_ptr(), None, None, None) == -1
    m.close()


def test_two_rounds_of_algorithm_1_track_the_oracle():
    """Algorithm 1 for one node, end to end through the C ABI: two rounds of H = 3 local steps on I_train followed by
    the synchronisation (own delta + the other nodes' reduced deltas, count normalisation, Nesterov outer step, restart
    of the local copy from the new global values), tiny fp32 configuration with the paper's MLP-only mask.  The fp64
    oracle runs the same schedule; losses agree to 1e-5 relative at every local step and the global parameters stay
    within a fraction of the accumulated step sizes."""
    cfg = gen.make_config("tiny")
    weights = gen.make_weights(cfg, seed=61)
    mask = gen.paper_mlp_mask(cfg, 2, 4)
    m = make_gpu_model(cfg, weights, mask)
    tr = O.LocalTrainer(cfg, weights, mask)
    n = tr.master.size
    theta_g_ref, buf_ref = tr.master.copy(), np.zeros(n)
    tg = torch.from_numpy(theta_g_ref.astype(np.float32)).cuda()
    mom = torch.zeros(n, dtype=torch.float32, device="cuda")
    others = torch.empty(n, dtype=torch.float32, device="cuda")
    H, lr_out, mu, cnt = 3, 0.7, 0.9, 4.0
    step = 0
    for rnd in range(2):
        for h in range(H):
            tok, tgt = gen.make_tokens(cfg, seed=61, step=step); step += 1
            lg = float(m.step(*m.upload_tokens(tok, tgt), HP).item())
            lo, _ = tr.step(tok, tgt, HP)
            assert abs(lg - lo) <= 1e-5 * abs(lo), (rnd, h, lg, lo)
        keys = [gen.stream_key(100 + rnd, gen.STREAM_DELTAS, j + 1) for j in range(3)]
        pp.pp_synth_delta_sum(m.h, others.data_ptr(), n, keys, 1e-4)
        others_ref = gen.synthetic_delta_sum(100 + rnd, n, 3, 1e-4)
        pp.pp_outer_delta(m.h, tg.data_ptr(), mom.data_ptr(), others.data_ptr(), pp.PPOuter(lr_out, mu, 1, cnt), None)
        torch.cuda.synchronize()
        theta_g_ref, buf_ref, _ = O.outer_step(theta_g_ref, tr.master, others_ref, buf_ref, lr_out, mu, cnt)
        tr.master = theta_g_ref.copy()                       # the local copy restarts from the new global values
        O.unpack_into(tr.params, tr.segs, tr.master)
        got = tg.cpu().numpy().astype(np.float64)
        budget = (rnd + 1) * (H * HP["lr"] + 1e-4) * lr_out * (1 + mu)          # what one round can move an element by, per round
        assert np.max(np.abs(got - theta_g_ref)) <= 0.1 * budget, (rnd, np.max(np.abs(got - theta_g_ref)), budget)
        assert np.array_equal(m.get_state("p"), tg.cpu().numpy())
    assert frozen_bytes_equal(cfg, m, weights, mask) == []
    m.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_more_than_65535_packed_rows_through_adamw_and_outer_step(dtype):
    """A narrow, deep-FFN model with every parameter trainable has 76 k packed rows of d_model = 64 elements -- more than
    one grid dimension of 65535 would cover.  AdamW on all of them, then the outer step, against the oracle."""
    cfg = gen.make_config("tiny", n_layers=6, d_model=64, n_heads=4, d_ff=4096, vocab=256, batch=2, seq=16, dtype=dtype)
    weights = gen.make_weights(cfg, seed=61)
    mask = gen.all_mask(cfg)
    m = make_gpu_model(cfg, weights, dict(all=1))
    segs = O.mask_segments(cfg, mask)
    n_rows = sum(hi - lo for _, lo, hi in segs)
    assert n_rows > 65535, n_rows
    tok, tgt = gen.make_tokens(cfg, seed=61)
    tr = O.LocalTrainer(cfg, weights, mask)
    p0 = tr.master.copy()
    loss = float(m.step(*m.upload_tokens(tok, tgt), HP).item())
    loss_ref, g_ref = tr.step(tok, tgt, HP)
    tol = 1e-5 if dtype == "f32" else 1e-2
    assert abs(loss - loss_ref) <= tol * abs(loss_ref)
    p = m.get_state("p").astype(np.float64)
    rows = p.size // cfg["d_model"]
    assert rows == n_rows
    if dtype == "f32":
        big = np.abs(g_ref) > 1e-3 * np.max(np.abs(g_ref))
        assert np.max(np.abs((p - p0) - (tr.master - p0))[big]) <= 2e-2 * HP["lr"]
    # every packed row moved (decay and update reach the last rows too) and the first / last rows match the oracle
    moved = np.any((p != p0.astype(np.float32)).reshape(rows, -1), axis=1)
    gains = (O.decay_mask_for(cfg, mask).reshape(rows, -1)[:, 0] == 0)
    assert np.all(moved | gains)
    from harness import cosine
    assert cosine(p - p0, tr.master - p0) >= (0.9999 if dtype == "f32" else 0.97)
    names = gen.tensor_shapes(cfg)
    now = O.pack({k: m.get_weight(k, s).astype(np.float64) for k, s in names.items()}, segs).astype(np.float32)
    expect = m.get_state("p")
    expect = gen.round_to_bf16(expect) if dtype == "bf16" else expect
    assert np.array_equal(now, expect)
    # outer step over all 76 k rows
    n = p.size
    theta_g0 = p0.astype(np.float32)
    tg = torch.from_numpy(theta_g0.copy()).cuda()
    mom = torch.zeros(n, dtype=torch.float32, device="cuda")
    delta = torch.empty(n, dtype=torch.float32, device="cuda")
    pp.pp_outer_delta(m.h, tg.data_ptr(), mom.data_ptr(), None, pp.PPOuter(0.7, 0.9, 1, 2.0), delta.data_ptr())
    torch.cuda.synchronize()
    ref_new, buf, ref_delta = O.outer_step(theta_g0.astype(np.float64), now.astype(np.float64), None, np.zeros(n), 0.7, 0.9, 2.0)
    np.testing.assert_allclose(delta.cpu().numpy(), ref_delta, rtol=2e-5, atol=1e-9)
    np.testing.assert_allclose(tg.cpu().numpy(), ref_new, rtol=2e-6, atol=1e-8)
    np.testing.assert_allclose(mom.cpu().numpy(), buf, rtol=2e-5, atol=1e-9)
    assert np.array_equal(m.get_state("p"), tg.cpu().numpy())
    m.close()
