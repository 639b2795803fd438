"""The split-K GEMM entry point that allocates nothing (partials in a device array built into the library) against the
existing entry point that takes a caller's scratch buffer: same kernels, same summation order, so the outputs must agree
bit for bit -- on two calls in a row, the second smaller than the first (the built-in array then still holds the first
call's partials), for the MFMA path and the plain path, and both must match the definition A B^T."""
import numpy as np
import pytest
import torch

import pp_inputs as gen
import paper_2509_22418_amd as pp

pytestmark = pytest.mark.gpu


def _dev_bf16(x):
    r = gen.round_to_bf16(x)
    return torch.from_numpy(gen.bf16_bits(r).astype(np.int16)).cuda(), r.astype(np.float64)


def _rnd(shape, seed):
    return gen.normal(gen.stream_key(seed, gen.STREAM_MISC, 7), int(np.prod(shape)), 1.0).reshape(shape)


_set_up_done = False


def _both(M, N, K, splits, path, seed):
    global _set_up_done
    st = torch.cuda.current_stream().cuda_stream
    Ad, A = _dev_bf16(_rnd((M, K), seed))
    Bd, B = _dev_bf16(_rnd((N, K), seed + 1))
    ref = A @ B.T
    c_own = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    c_static = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    scratch = torch.empty(M * N * splits, dtype=torch.float32, device="cuda")
    pp.pp_op_gemm_nt(st, pp.PP_BF16, Ad.data_ptr(), K, Bd.data_ptr(), K, c_own.data_ptr(), N, M, N, K, None, 1, splits,
                     scratch.data_ptr(), path)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    pp.pp_op_gemm_nt_splitk_static(st, pp.PP_BF16, Ad.data_ptr(), K, Bd.data_ptr(), K, c_static.data_ptr(), N, M, N, K, splits, path)
    torch.cuda.synchronize()
    # the first call of the process on this GPU makes the runtime materialise the library's device array; none after it may
    # take device memory
    assert _set_up_done is False or torch.cuda.mem_get_info()[0] >= free_before
    _set_up_done = True
    a, b = c_own.cpu().numpy(), c_static.cpu().numpy()
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), (M, N, K, splits, path)
    assert np.max(np.abs(b - ref)) <= 1e-4 * np.sqrt(K) * max(1.0, np.max(np.abs(ref)) / np.sqrt(K)), (M, N, K, splits, path)


@pytest.mark.parametrize("path", [0, 1])
def test_static_scratch_splitk_gemm_equals_the_allocating_entry_point(path):
    print(f"case no-alloc split-K gemm path={path}: 512x256x4096/8 then 200x136x1024/4", flush=True)
    _both(512, 256, 4096, 8, path, seed=51)          # weight-gradient form: 2 x 1 tiles, 8 K-ranges
    _both(200, 136, 1024, 4, path, seed=53)          # smaller and ragged, right after: stale partials from the first call remain


def test_static_scratch_rejects_oversize_and_bad_splits():
    st = torch.cuda.current_stream().cuda_stream
    assert pp.PP_STATIC_SCRATCH_FLOATS == 4 << 20
    x = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(pp.PPError, match="exceeds the built-in scratch"):
        pp.pp_op_gemm_nt_splitk_static(st, pp.PP_BF16, x.data_ptr(), 4096, x.data_ptr(), 4096, x.data_ptr(), 2048, 2048, 2048, 4096, 2, 0)
    with pytest.raises(pp.PPError, match="splits"):
        pp.pp_op_gemm_nt_splitk_static(st, pp.PP_BF16, x.data_ptr(), 64, x.data_ptr(), 64, x.data_ptr(), 8, 8, 8, 64, 1, 0)
