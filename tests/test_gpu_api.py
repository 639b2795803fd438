"""Boundary behaviour on the GPU: error codes, option handling, run-to-run reproducibility, mask re-arming."""
import ctypes

import numpy as np
import pytest
import torch

import pp_inputs as gen
import paper_2509_22418_amd as pp
from paper_2509_22418_amd import binding as b
from harness import HP, make_gpu_model

pytestmark = pytest.mark.gpu

SMALL = dict(n_layers=2, d_model=256, n_heads=2, d_ff=512, vocab=512, batch=2, seq=192, dtype="bf16")


def test_error_codes_and_state_machine():
    cfg = gen.make_config("tiny")
    lib = pp.load_library()
    m = pp.LocalStepModel(cfg, gen.ffn_slice_mask(cfg, 0, 4))
    m.load_weights(gen.make_weights(cfg, 1))
    tok, tgt = gen.make_tokens(cfg, 1)
    td, gd = m.upload_tokens(tok, tgt)
    opt = pp.PPAdamW(1e-3, 0.9, 0.95, 1e-8, 0.1)
    # step before the mask is set
    assert lib.pp_local_step(m.h, td.data_ptr(), gd.data_ptr(), 4, 32, ctypes.byref(opt), m.loss.data_ptr()) == -3
    assert b"pp_set_trainable_mask" in lib.pp_last_error()
    m.set_mask()
    # shapes beyond the maxima, null pointers, bad hyper-parameters
    assert lib.pp_local_step(m.h, td.data_ptr(), gd.data_ptr(), 5, 32, ctypes.byref(opt), m.loss.data_ptr()) == -1
    assert lib.pp_local_step(m.h, td.data_ptr(), gd.data_ptr(), 4, 33, ctypes.byref(opt), m.loss.data_ptr()) == -1
    assert lib.pp_local_step(m.h, None, gd.data_ptr(), 4, 32, ctypes.byref(opt), m.loss.data_ptr()) == -1
    bad = pp.PPAdamW(1e-3, 1.5, 0.95, 1e-8, 0.1)
    assert lib.pp_local_step(m.h, td.data_ptr(), gd.data_ptr(), 4, 32, ctypes.byref(bad), m.loss.data_ptr()) == -1
    # tensor I/O: unknown names and wrong sizes
    buf = np.zeros(10, dtype=np.float32)
    assert lib.pp_get_tensor(m.h, b"layers.9.wq", buf.ctypes.data, buf.nbytes) == -1
    assert lib.pp_get_tensor(m.h, b"embed", buf.ctypes.data, buf.nbytes) == -1
    assert lib.pp_set_option(m.h, b"no_such_option", 1) == -1
    # undersized state buffer for a bigger mask
    big = b.make_mask(dict(all=1))
    assert lib.pp_set_trainable_mask(m.h, ctypes.byref(big), m.state.data_ptr(), 256) == -1
    # a valid step still works afterwards
    loss = float(m.step(td, gd, HP).item())
    assert np.isfinite(loss)
    m.close()


def test_step_is_bit_reproducible_and_mask_can_be_rearmed():
    """Split-K partial sums, attention backward and the norm-gain reductions use fixed orders: two runs from the same
    state give bit-identical gradients, losses and weights.  Setting the mask again restarts the optimizer state."""
    cfg = gen.make_config("tiny", **SMALL)
    weights = gen.make_weights(cfg, seed=31)
    mask = gen.paper_mlp_mask(cfg, 1, 4)
    tok, tgt = gen.make_tokens(cfg, seed=31)
    runs = []
    for rep in range(2):
        m = make_gpu_model(cfg, weights, mask)
        td, gd = m.upload_tokens(tok, tgt)
        l1 = float(m.step(td, gd, HP).item())
        g1 = m.get_state("g").copy()
        l2 = float(m.step(td, gd, HP).item())
        p2 = m.get_state("p").copy()
        runs.append((l1, g1, l2, p2))
        if rep == 1:
            m.set_mask()          # re-arm: masters re-read from the current weights, m = v = 0, step counter 0
            assert np.all(m.get_state("m") == 0) and np.all(m.get_state("v") == 0)
            flat = m.get_state("p")
            wq = m.get_weight("layers.0.wo", (cfg["d_model"], cfg["d_model"]))
            assert np.isin(wq.reshape(-1)[:8], flat).all()
        m.close()
    assert runs[0][0] == runs[1][0] and runs[0][2] == runs[1][2]
    assert np.array_equal(runs[0][1], runs[1][1])
    assert np.array_equal(runs[0][3], runs[1][3])


def test_plain_and_mfma_paths_agree():
    cfg = gen.make_config("tiny", **SMALL)
    weights = gen.make_weights(cfg, seed=32)
    mask = gen.ffn_slice_mask(cfg, 0, 4)
    tok, tgt = gen.make_tokens(cfg, seed=32)
    out = []
    for plain in (False, True):
        m = make_gpu_model(cfg, weights, mask, force_plain=plain)
        td, gd = m.upload_tokens(tok, tgt)
        loss = float(m.step(td, gd, None).item())
        out.append((loss, m.get_state("g").astype(np.float64)))
        m.close()
    assert abs(out[0][0] - out[1][0]) <= 2e-3 * abs(out[1][0])
    a, bb = out[0][1], out[1][1]
    assert float(a @ bb / (np.linalg.norm(a) * np.linalg.norm(bb))) >= 0.9999


@pytest.mark.parametrize("mname", ["ffn", "paper_mlp", "all"])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_activation_recomputation_gives_the_same_bits_with_less_workspace(mname, dtype):
    """recompute = 1 keeps only each layer's input and runs the layer forward again in the backward pass (the paper's
    memory regime, Experimental Setup / Table 1).  Every kernel is deterministic, so losses, gradients and the weights
    after two AdamW steps are bit-identical to the stored-activation run; the activation part of the workspace shrinks
    to (n_layers x one [T x d] tensor) + one layer's worth."""
    base = dict(SMALL, n_layers=3, dtype=dtype)
    cfg0 = gen.make_config("tiny", **base)
    cfg1 = dict(cfg0, recompute=1)
    weights = gen.make_weights(cfg0, seed=41)
    mask = {"ffn": gen.ffn_slice_mask(cfg0, 1, 4), "paper_mlp": gen.paper_mlp_mask(cfg0, 1, 4), "all": dict(all=1)}[mname]
    out = []
    for cfg in (cfg0, cfg1):
        m = make_gpu_model(cfg, weights, mask)
        losses = []
        for step in range(2):
            tok, tgt = gen.make_tokens(cfg, seed=41, step=step)
            td, gd = m.upload_tokens(tok, tgt)
            losses.append(float(m.step(td, gd, HP).item()))
        rep = m.memory_report()
        out.append((losses, m.get_state("g"), m.get_state("p"), m.counters(), rep))
        m.close()
    (l0, g0, p0, c0, r0), (l1, g1, p1, c1, r1) = out
    assert l0 == l1
    assert np.array_equal(g0, g1) and np.array_equal(p0, p1)
    assert c0["flops_fwd"] == c1["flops_fwd"] and c0["flops_bwd"] == c1["flops_bwd"]          # recomputation is not counted
    es = 2 if dtype == "bf16" else 4
    T, d, L = cfg0["batch"] * cfg0["seq"], cfg0["d_model"], cfg0["n_layers"]
    assert r1["activations"] < r0["activations"]
    saved = r0["activations"] - r1["activations"]
    per_layer_rest = (r0["activations"] - T * (2 * d + cfg0["vocab"]) * es) / L - T * d * es          # all but x, roughly
    assert saved > 0.9 * (L - 1) * per_layer_rest


def test_parameters_filled_by_device_copy_give_the_same_step():
    """The parameter buffer may be filled without pp_set_tensor (device-to-device copy, checkpoint load): the transposed
    weight copies are formed from it when the mask is set, so loss, gradients and updated weights are bit-identical to a
    model that was filled tensor by tensor."""
    cfg = gen.make_config("tiny", **SMALL)
    weights = gen.make_weights(cfg, seed=37)
    mask = gen.paper_mlp_mask(cfg, 0, 4)
    tok, tgt = gen.make_tokens(cfg, seed=37)
    a = make_gpu_model(cfg, weights, mask)
    b2 = pp.LocalStepModel(cfg, mask)
    pp.pp_free(b2.h)                               # start again over a workspace full of junk: whatever it held must not matter
    b2.ws.fill_(0x7f)
    torch.cuda.synchronize()
    b2.h = pp.pp_init_model(b2.ccfg, b2.params.data_ptr(), b2.bytes_params, b2.ws.data_ptr(), b2.bytes_ws, b2.stream.cuda_stream)
    b2.params.copy_(a.params)                      # device copy of the canonical buffer; no pp_set_tensor at all
    torch.cuda.synchronize()
    b2.set_mask()
    out = []
    for mdl in (a, b2):
        loss = float(mdl.step(*mdl.upload_tokens(tok, tgt), HP).item())
        out.append((loss, mdl.get_state("g").copy(), mdl.get_state("p").copy(),
                    mdl.get_weight("layers.1.wd", (cfg["d_ff"], cfg["d_model"])).copy(),
                    mdl.get_weight("shadow.layers.1.wd", (cfg["d_model"], cfg["d_ff"])).copy()))
    assert out[0][0] == out[1][0]
    for x, y in zip(out[0][1:], out[1][1:]):
        assert np.array_equal(x, y)
    assert np.array_equal(out[1][3].T, out[1][4])
    a.close()
    b2.close()


def test_vocab_above_32768_uses_the_register_cross_entropy():
    """bf16 rows of up to 65536 logits stay in registers (no LDS stage): a one-layer model with vocab 40000 against the oracle."""
    from oracle import pp_oracle as O
    from harness import cosine
    cfg = gen.make_config("tiny", n_layers=1, d_model=128, n_heads=2, d_ff=256, vocab=40000, batch=1, seq=24, dtype="bf16")
    weights = gen.make_weights(cfg, seed=43)
    mask = dict(gen.ffn_slice_mask(cfg, 0, 4), train_lm_head=1)
    tok, tgt = gen.make_tokens(cfg, seed=43)
    m = make_gpu_model(cfg, weights, mask)
    loss = float(m.step(*m.upload_tokens(tok, tgt), None).item())
    params = O.to_f64(weights)
    loss_ref, cache = O.forward(cfg, params, tok, tgt)
    g_ref, _ = O.backward_restricted(cfg, params, cache, mask)
    assert abs(loss - loss_ref) <= 1e-2 * abs(loss_ref)
    assert cosine(m.get_state("g"), g_ref) >= 0.999
    m.close()
    lib = pp.load_library()
    too_big = b.make_config(dict(cfg, vocab=65544))
    assert lib.pp_query_bytes(ctypes.byref(too_big), None, 0) == 0 and b"vocab" in lib.pp_last_error()
