"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module holds input *generation* only: a counter-based integer generator, uniform /
normal variates from it, bf16 rounding of stored values, Zipf token draws, model-shape
configs and tensor name/shape tables.  None of the method's arithmetic (forward, backward,
optimizer, outer step) lives here, and it imports neither the oracle nor the HIP binding.

The paper trains on a web-text corpus with a 32000-entry subword vocabulary and fixed-length
sequences (Experimental Setup); neither is available offline, so heavy-tailed iid Zipf(1.1)
token ids over the same vocabulary size and N(0, 0.02) weights at the same tensor shapes
stand in for them.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_U64 = np.uint64
_GOLD = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK = (1 << 64) - 1

STREAM_WEIGHTS = 1
STREAM_TOKENS = 2
STREAM_DELTAS = 3
STREAM_MISC = 4


def _mix_int(z: int) -> int:
    """splitmix64 finaliser on a Python int (exact 64-bit wraparound)."""
    z = (z + _GOLD) & _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def _mix_arr(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser, vectorised over uint64 (wraparound arithmetic is intended)."""
    with np.errstate(over="ignore"):
        z = z + _U64(_GOLD)
        z = (z ^ (z >> _U64(30))) * _U64(_M1)
        z = (z ^ (z >> _U64(27))) * _U64(_M2)
        return z ^ (z >> _U64(31))


def stream_key(seed: int, stream: int, substream: int = 0) -> int:
    """64-bit key of a (seed, stream, substream) triple."""
    return _mix_int(_mix_int(_mix_int(seed & _MASK) ^ (stream & _MASK)) ^ (substream & _MASK))


def fnv1a64(name: str) -> int:
    h = 0xCBF29CE484222325
    for b in name.encode():
        h = ((h ^ b) * 0x100000001B3) & _MASK
    return h


def raw_u64(key: int, start: int, count: int) -> np.ndarray:
    """Values x_i = mix(key + i*GOLD) for i in [start, start+count): counter based, so any
    sub-range can be produced independently (and identically on a device)."""
    idx = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix_arr(_U64(key) + idx * _U64(_GOLD))


def uniform01(key: int, start: int, count: int) -> np.ndarray:
    """Uniform in (0,1): ((x >> 11) + 0.5) * 2^-53, fp64."""
    x = raw_u64(key, start, count) >> _U64(11)
    return (x.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _normal_chunk(key: int, start: int, count: int) -> np.ndarray:
    """Standard normals for element indices [start, start+count), start even.
    Element 2j uses r*cos, element 2j+1 uses r*sin of the Box-Muller pair drawn from
    uniforms 2j and 2j+1."""
    assert start % 2 == 0
    npair = (count + 1) // 2
    u = uniform01(key, start, 2 * npair)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    ang = (2.0 * math.pi) * u[1::2]
    out = np.empty(2 * npair, dtype=np.float64)
    out[0::2] = r * np.cos(ang)
    out[1::2] = r * np.sin(ang)
    return out[:count]


def normal(key: int, count: int, std: float = 1.0, threads: int = 8) -> np.ndarray:
    """`count` N(0, std^2) variates in fp64 (chunked over a thread pool; the result does not
    depend on the chunking because every element is a function of its own index)."""
    chunk = 1 << 22
    if count <= chunk:
        return _normal_chunk(key, 0, count) * std
    out = np.empty(count, dtype=np.float64)
    starts = list(range(0, count, chunk))

    def work(s):
        n = min(chunk, count - s)
        out[s:s + n] = _normal_chunk(key, s, n) * std

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, starts))
    return out


# ----------------------------------------------------------------------------- bf16 storage
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp64/fp32 values to the nearest bf16 (ties to even); returned as float32 holding
    exactly representable bf16 values."""
    f = np.asarray(x, dtype=np.float32)
    b = f.view(np.uint32)
    rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already exactly representable in bf16."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- model shapes
CONFIGS = {
    # name: (n_layers, d_model, n_heads, d_ff, vocab, batch, seq, dtype, n_slices)
    "tiny": dict(n_layers=2, d_model=64, n_heads=4, d_ff=256, vocab=256, batch=4, seq=32,
                 dtype="f32", n_slices=4),
    "125m": dict(n_layers=12, d_model=768, n_heads=12, d_ff=3072, vocab=32000, batch=8, seq=1024,
                 dtype="bf16", n_slices=8),
    "1p3b": dict(n_layers=24, d_model=2048, n_heads=16, d_ff=8192, vocab=32000, batch=8, seq=2048,
                 dtype="bf16", n_slices=32),
}
RMS_EPS = 1e-5
ROPE_BASE = 10000.0


def make_config(name: str, **over) -> dict:
    c = dict(CONFIGS[name])
    c.update(rms_eps=RMS_EPS, rope_base=ROPE_BASE)
    c.update(over)
    return c


def tensor_shapes(cfg: dict) -> dict:
    """Canonical tensor names and shapes, bottom of the network first.
    wqkv rows are [Wq; Wk; Wv], each (out x in), head j owning rows j*dh..(j+1)*dh of its block.
    wo is (out x in).  wg, wu, wd are all (d_ff x d_model), i.e. hidden-unit major, so a slice of
    hidden units is one contiguous row block of each."""
    d, F, V, L = cfg["d_model"], cfg["d_ff"], cfg["vocab"], cfg["n_layers"]
    t = {"embed": (V, d)}
    for l in range(L):
        p = f"layers.{l}."
        t[p + "attn_norm"] = (d,)
        t[p + "wqkv"] = (3 * d, d)
        t[p + "wo"] = (d, d)
        t[p + "ffn_norm"] = (d,)
        t[p + "wg"] = (F, d)
        t[p + "wu"] = (F, d)
        t[p + "wd"] = (F, d)
    t["final_norm"] = (d,)
    t["lm_head"] = (V, d)
    return t


def make_weights(cfg: dict, seed: int, std: float = 0.02, threads: int = 8) -> dict:
    """All tensors as float32 arrays holding the *stored* values: matrices N(0, std) drawn in
    fp64 and rounded once to the storage dtype (bf16 or fp32); norm gains 1.0."""
    out = {}
    for name, shape in tensor_shapes(cfg).items():
        if name.endswith("norm"):
            out[name] = np.ones(shape, dtype=np.float32)
            continue
        key = stream_key(seed, STREAM_WEIGHTS, fnv1a64(name))
        w = normal(key, int(np.prod(shape)), std, threads=threads)
        w = round_to_bf16(w) if cfg["dtype"] == "bf16" else w.astype(np.float32)
        out[name] = w.reshape(shape)
    return out


_zipf_cache: dict = {}


def zipf_cdf(vocab: int, s: float = 1.1) -> np.ndarray:
    k = (vocab, s)
    if k not in _zipf_cache:
        p = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
        c = np.cumsum(p)
        _zipf_cache[k] = c / c[-1]
    return _zipf_cache[k]


def make_tokens(cfg: dict, seed: int, step: int = 0, batch: int | None = None, seq: int | None = None,
                s: float = 1.1):
    """iid Zipf(s) token ids [B,S] int32 (rank r has id r-1) and next-token targets [B,S] int32
    (targets[b,t] = tokens[b,t+1]; the last position of each sequence is -1 = ignored)."""
    B = batch or cfg["batch"]
    S = seq or cfg["seq"]
    key = stream_key(seed, STREAM_TOKENS, step)
    u = uniform01(key, 0, B * S)
    tok = np.searchsorted(zipf_cdf(cfg["vocab"], s), u, side="left").astype(np.int32)
    tok = np.minimum(tok, cfg["vocab"] - 1).reshape(B, S)
    tgt = np.full((B, S), -1, dtype=np.int32)
    tgt[:, :-1] = tok[:, 1:]
    return tok, tgt


def ffn_slice_mask(cfg: dict, node: int = 0, n_slices: int | None = None) -> dict:
    """The benchmark mask: node k trains hidden units [n*F/N, (n+1)*F/N), n = k mod N, of every
    layer's FFN; everything else frozen."""
    N = n_slices or cfg["n_slices"]
    F = cfg["d_ff"]
    assert F % N == 0
    n = node % N
    return dict(ffn_lo=n * F // N, ffn_hi=(n + 1) * F // N, head_lo=0, head_hi=0,
                train_wo=0, train_norms=0, train_embed=0, train_lm_head=0)


def all_mask(cfg: dict) -> dict:
    return dict(ffn_lo=0, ffn_hi=cfg["d_ff"], head_lo=0, head_hi=cfg["n_heads"],
                train_wo=1, train_norms=1, train_embed=1, train_lm_head=1)


def paper_mlp_mask(cfg: dict, node: int = 0, n_slices: int = 4, slice_heads: bool = False) -> dict:
    """The paper's masks (Parameter Slicing): an FFN slice plus every non-MLP parameter; with
    slice_heads the Q/K/V projections are restricted to the node's head group."""
    m = ffn_slice_mask(cfg, node, n_slices)
    h = cfg["n_heads"]
    n = node % n_slices
    lo, hi = (n * h // n_slices, (n + 1) * h // n_slices) if slice_heads else (0, h)
    m.update(head_lo=lo, head_hi=hi, train_wo=1, train_norms=1, train_embed=1, train_lm_head=1)
    return m


def synthetic_delta_sum(seed: int, count: int, n_nodes: int = 31, std: float = 1e-4) -> np.ndarray:
    """Sum of n_nodes seeded N(0, std) vectors: stands for the all-reduce result of the other
    nodes' deltas on the same trainable subset."""
    acc = np.zeros(count, dtype=np.float64)
    for j in range(n_nodes):
        acc += normal(stream_key(seed, STREAM_DELTAS, j + 1), count, std)
    return acc
