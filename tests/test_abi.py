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
