"""Op-level parity of the dense-contraction kernels against their plain definitions (numpy fp64 on the same
bf16-rounded inputs): the MFMA GEMM in all the forms the local step uses, and causal attention fwd/bwd."""
import numpy as np
import pytest
import torch

import pp_inputs as gen
import paper_2509_22418_amd as pp
from oracle import pp_oracle as O

pytestmark = pytest.mark.gpu


def dev_bf16(x):
    """numpy float array -> (device uint16 tensor of bf16 bits, float64 array of the rounded values)."""
    r = gen.round_to_bf16(x)
    return torch.from_numpy(gen.bf16_bits(r).astype(np.int16)).cuda(), r.astype(np.float64)


def from_bf16(t):
    return gen.bf16_bits_to_f32(t.cpu().numpy().view(np.uint16)).astype(np.float64)


def rnd(shape, seed, std=1.0):
    return gen.normal(gen.stream_key(seed, gen.STREAM_MISC, 0), int(np.prod(shape)), std).reshape(shape)


GEMM_CASES = [
    # M, N, K, residual, out_f32, splits
    (512, 512, 256, False, False, 1),        # 2x2 tiles
    (300, 200, 128, True, False, 1),         # ragged M and N inside one tile
    (777, 1000, 192, False, False, 1),       # several tiles with ragged tails
    (256, 768, 2048, True, False, 1),        # long K
    (512, 256, 4096, False, True, 8),        # weight-gradient form: few tiles, split K, fp32 out
    (128, 320, 1024, False, True, 1),
    (64, 64, 100, False, False, 1),          # K not a multiple of 64: plain path
]


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("M,N,K,res,f32,splits", GEMM_CASES)
def test_gemm_nt_matches_definition(M, N, K, res, f32, splits, variant):
    """variant 0: register-staged MFMA kernel; 1: default dispatch (these shapes have few tiles: the 128 x 128-tile kernel for
    bf16 output, the direct-to-LDS 256 x 256 kernel for fp32 output); 2: direct-to-LDS 256 x 256 kernel throughout."""
    print(f"case gemm {M}x{N}x{K} res={res} f32={f32} splits={splits} variant={variant}", flush=True)
    pp.pp_set_option(None, "gemm_variant", min(variant, 1))
    pp.pp_set_option(None, "gemm_small_tiles", 0 if variant == 2 else 1)
    Ad, A = dev_bf16(rnd((M, K), 1))
    Bd, B = dev_bf16(rnd((N, K), 2))
    ref = A @ B.T
    st = torch.cuda.current_stream().cuda_stream
    Rd = None
    if res:
        Rd, R = dev_bf16(rnd((M, N), 3, std=4.0))
        ref = ref + R
    scale = np.sqrt(K)
    for path in (0, 1):
        if f32:
            Cd = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
            scratch = torch.empty(M * N * splits, dtype=torch.float32, device="cuda") if splits > 1 else None
            pp.pp_op_gemm_nt(st, pp.PP_BF16, Ad.data_ptr(), K, Bd.data_ptr(), K, Cd.data_ptr(), N, M, N, K, None, 1, splits,
                             None if scratch is None else scratch.data_ptr(), path)
            torch.cuda.synchronize()
            got = Cd.cpu().numpy().astype(np.float64)
            assert np.max(np.abs(got - ref)) <= 2e-5 * scale * 4, (path, np.max(np.abs(got - ref)))
        else:
            Cd = torch.zeros((M, N), dtype=torch.int16, device="cuda")
            pp.pp_op_gemm_nt(st, pp.PP_BF16, Ad.data_ptr(), K, Bd.data_ptr(), K, Cd.data_ptr(), N, M, N, K,
                             None if Rd is None else Rd.data_ptr(), 0, 1, None, path)
            torch.cuda.synchronize()
            got = from_bf16(Cd)
            # one bf16 rounding of the exact result: relative 2^-8, plus fp32 accumulation noise
            assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-4 * scale), (path, np.max(np.abs(got - ref)))


@pytest.mark.parametrize("M,N,res", [(4096, 4608, False), (4096, 4352, True), (4200, 4100, True)])
def test_gemm_with_more_tiles_than_compute_units_walks_tiles_identically(M, N, res):
    """288 tiles (a multiple of 8: XCD-aware walk), 272 tiles, and 17 x 17 ragged tiles on 256 compute units: some
    workgroups take two tiles.  Checked against the definition, and bit for bit against one workgroup per tile."""
    K = 128
    print(f"case gemm tile walk {M}x{N}x{K} res={res}", flush=True)
    pp.pp_set_option(None, "gemm_variant", 1)
    pp.pp_set_option(None, "gemm_small_tiles", 0)          # these tile counts would otherwise go to the 128 x 128-tile kernel
    Ad, A = dev_bf16(rnd((M, K), 11))
    Bd, B = dev_bf16(rnd((N, K), 12))
    ref = A @ B.T
    Rd = None
    if res:
        Rd, R = dev_bf16(rnd((M, N), 13, std=4.0))
        ref = ref + R
    st = torch.cuda.current_stream().cuda_stream
    out = {}
    try:
        for persistent in (1, 0):
            pp.pp_set_option(None, "gemm_persistent", persistent)
            Cd = torch.zeros((M, N), dtype=torch.int16, device="cuda")
            pp.pp_op_gemm_nt(st, pp.PP_BF16, Ad.data_ptr(), K, Bd.data_ptr(), K, Cd.data_ptr(), N, M, N, K,
                             None if Rd is None else Rd.data_ptr(), 0, 1, None, 0)
            torch.cuda.synchronize()
            out[persistent] = Cd.cpu().numpy()
    finally:
        pp.pp_set_option(None, "gemm_persistent", 1)
    got = from_bf16(torch.from_numpy(out[1]))
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-4 * np.sqrt(K))
    assert np.array_equal(out[0], out[1])


def test_gemm_with_leading_dimensions_and_column_slices():
    """Operands and result addressed inside wider matrices (how slices of weights / activations are passed)."""
    M, N, K, lda, ldb, ldc = 384, 320, 256, 512, 640, 1024
    Ad, A = dev_bf16(rnd((M, lda), 4))
    Bd, B = dev_bf16(rnd((N, ldb), 5))
    Cd = torch.zeros((M, ldc), dtype=torch.int16, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    a_off, b_off, c_off = 64, 128, 256
    pp.pp_op_gemm_nt(st, pp.PP_BF16, Ad.data_ptr() + 2 * a_off, lda, Bd.data_ptr() + 2 * b_off, ldb, Cd.data_ptr() + 2 * c_off, ldc,
                     M, N, K, None, 0, 1, None, 0)
    torch.cuda.synchronize()
    got = from_bf16(Cd)
    ref = A[:, a_off:a_off + K] @ B[:, b_off:b_off + K].T
    assert np.all(np.abs(got[:, c_off:c_off + N] - ref) <= 2.0 ** -8 * np.abs(ref) + 2e-3)
    assert np.all(got[:, :c_off] == 0) and np.all(got[:, c_off + N:] == 0)          # nothing written outside the slice


ATTN_CASES = [(2, 128, 2, 128), (1, 256, 3, 64), (2, 200, 2, 128), (1, 77, 2, 64), (1, 512, 1, 128), (2, 64, 4, 16)]


@pytest.mark.parametrize("B,S,h,dh", ATTN_CASES)
def test_attention_fwd_bwd_matches_definition(B, S, h, dh):
    print(f"case attention B={B} S={S} h={h} dh={dh}", flush=True)
    d = h * dh
    T = B * S
    qkv_d, qkv = dev_bf16(rnd((T, 3 * d), 6))
    dO_d, dO = dev_bf16(rnd((T, d), 7))
    q = qkv[:, :d].reshape(B, S, h, dh)
    k = qkv[:, d:2 * d].reshape(B, S, h, dh)
    v = qkv[:, 2 * d:].reshape(B, S, h, dh)
    o_ref, P = O.attention_fwd(q, k, v)
    dq, dk, dv = O.attention_bwd(dO.reshape(B, S, h, dh), q, k, v, P)
    dqkv_ref = np.concatenate([dq.reshape(T, d), dk.reshape(T, d), dv.reshape(T, d)], axis=1)
    st = torch.cuda.current_stream().cuda_stream
    for path in (0, 1):
        o_d = torch.zeros((T, d), dtype=torch.int16, device="cuda")
        lse_d = torch.zeros(B * h * S, dtype=torch.float32, device="cuda")
        D_d = torch.zeros(B * h * S, dtype=torch.float32, device="cuda")
        dqkv_d = torch.zeros((T, 3 * d), dtype=torch.int16, device="cuda")
        scratch = torch.zeros(3 * B * h * dh * ((S + 63) // 64 * 64), dtype=torch.int16, device="cuda")
        pp.pp_op_attention_fwd(st, pp.PP_BF16, qkv_d.data_ptr(), o_d.data_ptr(), lse_d.data_ptr(), scratch.data_ptr(), B, S, h, dh, path)
        pp.pp_op_attention_bwd(st, pp.PP_BF16, qkv_d.data_ptr(), o_d.data_ptr(), lse_d.data_ptr(), dO_d.data_ptr(), dqkv_d.data_ptr(),
                               D_d.data_ptr(), scratch.data_ptr(), B, S, h, dh, path)
        torch.cuda.synchronize()
        o = from_bf16(o_d)
        err = np.max(np.abs(o - o_ref.reshape(T, d)))
        assert err <= 2e-2, (path, err)
        got = from_bf16(dqkv_d)
        for part, name in enumerate(("dq", "dk", "dv")):
            a, b = got[:, part * d:(part + 1) * d], dqkv_ref[:, part * d:(part + 1) * d]
            cos = float((a * b).sum() / (np.linalg.norm(a) * np.linalg.norm(b)))
            assert cos >= 0.9995, (path, name, cos)
            assert np.max(np.abs(a - b)) <= 0.03 * np.max(np.abs(b)), (path, name)
        # log-sum-exp against the definition
        s = np.einsum("bihc,bjhc->bhij", q, k) / np.sqrt(dh)
        s = np.where(np.tril(np.ones((S, S), bool)), s, -np.inf)
        lse_ref = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
        assert np.max(np.abs(lse_d.cpu().numpy().reshape(B, h, S) - lse_ref)) <= 2e-3


TN_CASES = [
    # K (tokens), M, N, lda, m_blk, a_blk_stride, splits
    (256, 128, 128, 128, 128, 0, 1),            # one tile
    (512, 256, 384, 1024, 256, 0, 2),           # a column slice of a wider A (hidden-unit slice), several tiles, split K
    (384, 256, 200, 1024, 128, 512, 1),         # two column blocks 512 apart (gate | up), ragged N
    (1024, 72, 2048, 72, 72, 0, 4),             # ragged M inside one tile, wide N
    (2048, 384, 136, 1536, 128, 512, 8),        # three blocks (q | k | v of a head range), ragged N tile, 8 K ranges
]


@pytest.mark.parametrize("K,M,N,lda,m_blk,stride,splits", TN_CASES)
def test_gemm_tn_matches_definition(K, M, N, lda, m_blk, stride, splits):
    """Weight-gradient form C = A^T B with both operands token-major (LDS transpose reads), against numpy fp64 on the same
    bf16-rounded inputs; fp32 output, so the tolerance is fp32 accumulation over K."""
    print(f"case gemm_tn K={K} M={M} N={N} lda={lda} m_blk={m_blk} stride={stride} splits={splits}", flush=True)
    Ad, A = dev_bf16(rnd((K, lda), 5))
    Bd, B = dev_bf16(rnd((K, N), 6))
    cols = np.concatenate([np.arange(min(m_blk, M - b0)) + (b0 // m_blk) * stride for b0 in range(0, M, m_blk)])
    ref = A[:, cols].T @ B
    st = torch.cuda.current_stream().cuda_stream
    Cd = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    scratch = torch.empty(M * N * splits, dtype=torch.float32, device="cuda") if splits > 1 else None
    pp.pp_op_gemm_tn(st, Ad.data_ptr(), lda, m_blk, stride, Bd.data_ptr(), N, Cd.data_ptr(), N, M, N, K, splits,
                     None if scratch is None else scratch.data_ptr())
    torch.cuda.synchronize()
    got = Cd.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - ref)) <= 2e-5 * np.sqrt(K) * max(1.0, np.max(np.abs(ref)) / np.sqrt(K)) + 1e-6 * np.max(np.abs(ref))


def test_gemm_tn_rejects_shapes_it_does_not_take():
    st = torch.cuda.current_stream().cuda_stream
    x = torch.zeros(1 << 16, dtype=torch.int16, device="cuda")
    c = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
    with pytest.raises(pp.PPError, match="not taken"):
        pp.pp_op_gemm_tn(st, x.data_ptr(), 128, 128, 0, x.data_ptr(), 128, c.data_ptr(), 128, 128, 128, 100)          # K % 64
    with pytest.raises(pp.PPError, match="not taken"):
        pp.pp_op_gemm_tn(st, x.data_ptr(), 256, 64, 128, x.data_ptr(), 128, c.data_ptr(), 128, 128, 128, 128)       # blocks of 64 columns
