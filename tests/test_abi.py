"""The C-ABI library builds, loads, and exports every symbol include/pp.h declares; argument checking that
needs no GPU works."""
import ctypes
import os
import re

import pytest

import pp_inputs as gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pp_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2509_22418_amd import binding
    lib = binding.load_library()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_query_bytes_and_argument_checks_without_gpu():
    from paper_2509_22418_amd import binding as b
    cfg = gen.make_config("1p3b")
    c = b.make_config(cfg)
    P = sum(s[0] * (s[1] if len(s) == 2 else 1) for s in gen.tensor_shapes(cfg).values())
    assert b.pp_query_bytes(c, None, b.PP_BYTES_PARAMS) == 2 * P
    m32 = b.make_mask(gen.ffn_slice_mask(cfg, 0, 32))
    m8 = b.make_mask(gen.ffn_slice_mask(cfg, 0, 8))
    # optimizer state exists only for I_train: 16 bytes per trainable element, nothing for frozen ones
    assert b.pp_query_bytes(c, m32, b.PP_BYTES_STATE) == 16 * 37748736
    assert b.pp_query_bytes(c, m8, b.PP_BYTES_STATE) == 16 * 4 * 37748736
    assert b.pp_query_bytes(c, b.make_mask(dict(all=1)), b.PP_BYTES_STATE) == 16 * P
    lib = b.load_library()
    bad = b.make_config(dict(cfg, n_heads=7))
    assert lib.pp_query_bytes(ctypes.byref(bad), None, 0) == 0 and b"n_heads" in lib.pp_last_error()
    badm = b.make_mask(dict(ffn_lo=0, ffn_hi=cfg["d_ff"] + 8))
    assert lib.pp_query_bytes(ctypes.byref(c), ctypes.byref(badm), 1) == 0 and b"ffn range" in lib.pp_last_error()
    assert lib.pp_local_step(None, None, None, 1, 1, None, None) == -1
    assert lib.pp_outer_delta(None, None, None, None, None, None) == -1
    assert lib.pp_set_jacobian_slices(None, 1, 0, 0) == -1


def test_recompute_shrinks_the_activation_plan_without_gpu():
    """pp_query_bytes is host logic: with recompute = 1 the activation part of the workspace is n_layers layer inputs
    plus ONE layer's intermediate tensors instead of n_layers of them; everything else is unchanged."""
    from paper_2509_22418_amd import binding as b
    cfg = gen.make_config("1p3b")
    c0, c1 = b.make_config(cfg), b.make_config(dict(cfg, recompute=1))
    m = b.make_mask(gen.ffn_slice_mask(cfg, 0, 32))
    act0, act1 = (b.pp_query_bytes(c, m, b.PP_BYTES_ACTIVATIONS) for c in (c0, c1))
    ws0, ws1 = (b.pp_query_bytes(c, m, b.PP_BYTES_WORKSPACE) for c in (c0, c1))
    T, d, F, L, V, h = 8 * 2048, cfg["d_model"], cfg["d_ff"], cfg["n_layers"], cfg["vocab"], cfg["n_heads"]
    per_layer_rest = (T * (7 * d + 3 * F)) * 2 + (2 * T + 8 * h * 2048) * 4          # n1, qkv(3), o, xm, n2, g, u, a + rstd1, rstd2, lse
    # (the one shared block keeps the layout of a full layer block, so it carries one unused [T x d] slot)
    assert act0 - act1 == pytest.approx((L - 1) * per_layer_rest - T * d * 2, rel=1e-4)
    assert ws0 - ws1 == act0 - act1
    assert b.pp_query_bytes(c0, m, b.PP_BYTES_STATE) == b.pp_query_bytes(c1, m, b.PP_BYTES_STATE)
    assert b.pp_query_bytes(c0, m, b.PP_BYTES_SHADOW) == b.pp_query_bytes(c1, m, b.PP_BYTES_SHADOW)
    lib = b.load_library()
    bad = b.make_config(dict(cfg, recompute=2))
    assert lib.pp_query_bytes(ctypes.byref(bad), None, 0) == 0 and b"recompute" in lib.pp_last_error()
    assert lib.pp_outer_delta_group(None, 0, 1, 0, None, None, None, None, None) == -1
