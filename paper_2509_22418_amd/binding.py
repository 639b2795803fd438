"""ctypes binding of include/pp.h: argument marshalling only -- every step of the path runs in the HIP library.

The module-level pp_* functions mirror the C entry points one to one.  LocalStepModel is a convenience
holder that allocates the caller-owned device buffers with torch (torch is used for device memory and the
stream only) and forwards to those functions.  There is no CPU fallback: if the library is missing or no
GPU is present, calls fail loudly."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

PP_F32, PP_BF16 = 0, 1
PP_STATIC_SCRATCH_FLOATS = 4 << 20          # include/pp_ops.h
PP_BYTES_PARAMS, PP_BYTES_STATE, PP_BYTES_WORKSPACE, PP_BYTES_SHADOW, PP_BYTES_ACTIVATIONS = range(5)
EXPORTS = ["pp_query_bytes", "pp_init_model", "pp_set_tensor", "pp_get_tensor", "pp_set_trainable_mask", "pp_local_step",
           "pp_set_jacobian_slices", "pp_outer_delta", "pp_outer_delta_group", "pp_synth_delta_sum", "pp_get_counters", "pp_get_launch_counts", "pp_get_gemm_timing", "pp_set_option", "pp_last_error", "pp_free",
           "pp_op_gemm_nt", "pp_op_gemm_tn", "pp_op_gemm_nt_splitk_static", "pp_op_attention_fwd", "pp_op_attention_bwd"]


class PPError(RuntimeError):
    pass


class PPConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "d_ff", "vocab", "max_batch", "max_seq", "dtype")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float), ("recompute", C.c_int32)]


class PPMask(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("all", "ffn_lo", "ffn_hi", "head_lo", "head_hi", "train_wo", "train_norms",
                                         "train_embed", "train_lm_head")]


class PPAdamW(C.Structure):
    _fields_ = [(n, C.c_float) for n in ("lr", "beta1", "beta2", "eps", "weight_decay")]


class PPOuter(C.Structure):
    _fields_ = [("lr", C.c_float), ("momentum", C.c_float), ("nesterov", C.c_int32), ("m_count", C.c_float)]


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libpp_hip.so")


_lib = None


def load_library():
    """Loads the in-tree HIP library; builds it first only if it has never been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from .build import build
        build()
    import torch  # noqa: F401  -- first, so that the library binds to the HIP runtime torch ships (one runtime per process)
    lib = C.CDLL(path)
    vp, sz, i32, i64 = C.c_void_p, C.c_size_t, C.c_int32, C.c_int64
    lib.pp_query_bytes.restype = sz
    lib.pp_query_bytes.argtypes = [C.POINTER(PPConfig), C.POINTER(PPMask), C.c_int]
    lib.pp_init_model.restype = C.c_int
    lib.pp_init_model.argtypes = [C.POINTER(PPConfig), vp, sz, vp, sz, vp, C.POINTER(vp)]
    lib.pp_set_tensor.restype = C.c_int
    lib.pp_set_tensor.argtypes = [vp, C.c_char_p, vp, sz]
    lib.pp_get_tensor.restype = C.c_int
    lib.pp_get_tensor.argtypes = [vp, C.c_char_p, vp, sz]
    lib.pp_set_trainable_mask.restype = C.c_int
    lib.pp_set_trainable_mask.argtypes = [vp, C.POINTER(PPMask), vp, sz]
    lib.pp_local_step.restype = C.c_int
    lib.pp_local_step.argtypes = [vp, vp, vp, i32, i32, C.POINTER(PPAdamW), vp]
    lib.pp_outer_delta.restype = C.c_int
    lib.pp_outer_delta.argtypes = [vp, vp, vp, vp, C.POINTER(PPOuter), vp]
    lib.pp_set_jacobian_slices.restype = C.c_int
    lib.pp_set_jacobian_slices.argtypes = [vp, i32, i32, i32]
    lib.pp_outer_delta_group.restype = C.c_int
    lib.pp_outer_delta_group.argtypes = [vp, i32, i32, i32, vp, vp, vp, C.POINTER(PPOuter), vp]
    lib.pp_synth_delta_sum.restype = C.c_int
    lib.pp_synth_delta_sum.argtypes = [vp, vp, sz, C.POINTER(C.c_uint64), i32, C.c_float]
    lib.pp_get_counters.restype = C.c_int
    lib.pp_get_counters.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(i64)]
    lib.pp_get_launch_counts.restype = C.c_int
    lib.pp_get_launch_counts.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
    lib.pp_get_gemm_timing.restype = C.c_int
    lib.pp_get_gemm_timing.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(i64)]
    lib.pp_set_option.restype = C.c_int
    lib.pp_set_option.argtypes = [vp, C.c_char_p, i64]
    lib.pp_last_error.restype = C.c_char_p
    lib.pp_last_error.argtypes = []
    lib.pp_free.restype = None
    lib.pp_free.argtypes = [vp]
    lib.pp_op_gemm_nt.restype = C.c_int
    lib.pp_op_gemm_nt.argtypes = [vp, C.c_int, vp, C.c_int, vp, C.c_int, vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_int, C.c_int, vp, C.c_int]
    lib.pp_op_gemm_tn.restype = C.c_int
    lib.pp_op_gemm_tn.argtypes = [vp, vp, C.c_int, C.c_int, i64, vp, C.c_int, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, vp]
    lib.pp_op_gemm_nt_splitk_static.restype = C.c_int
    lib.pp_op_gemm_nt_splitk_static.argtypes = [vp, C.c_int, vp, C.c_int, vp, C.c_int, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
    lib.pp_op_attention_fwd.restype = C.c_int
    lib.pp_op_attention_fwd.argtypes = [vp, C.c_int, vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
    lib.pp_op_attention_bwd.restype = C.c_int
    lib.pp_op_attention_bwd.argtypes = [vp, C.c_int, vp, vp, vp, vp, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int]
    _lib = lib
    return lib


def pp_last_error() -> str:
    return load_library().pp_last_error().decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise PPError(f"{what} failed ({rc}): {pp_last_error()}")


def _mask_ptr(mask):
    return None if mask is None else C.byref(mask)


def pp_query_bytes(cfg: PPConfig, mask, which: int) -> int:
    n = load_library().pp_query_bytes(C.byref(cfg), _mask_ptr(mask), which)
    if n == 0 and which != PP_BYTES_STATE:
        raise PPError("pp_query_bytes failed: " + pp_last_error())
    if n == 0 and pp_last_error() and mask is None:
        raise PPError("pp_query_bytes failed: " + pp_last_error())
    return n


def pp_init_model(cfg: PPConfig, params_ptr: int, params_bytes: int, ws_ptr: int, ws_bytes: int, stream: int):
    h = C.c_void_p()
    _check(load_library().pp_init_model(C.byref(cfg), params_ptr, params_bytes, ws_ptr, ws_bytes, stream, C.byref(h)), "pp_init_model")
    return h


def pp_set_tensor(h, name: str, host: np.ndarray):
    host = np.ascontiguousarray(host)
    _check(load_library().pp_set_tensor(h, name.encode(), host.ctypes.data, host.nbytes), f"pp_set_tensor({name})")


def pp_get_tensor(h, name: str, host: np.ndarray):
    assert host.flags["C_CONTIGUOUS"]
    _check(load_library().pp_get_tensor(h, name.encode(), host.ctypes.data, host.nbytes), f"pp_get_tensor({name})")
    return host


def pp_set_trainable_mask(h, mask: PPMask, state_ptr: int, state_bytes: int):
    _check(load_library().pp_set_trainable_mask(h, C.byref(mask), state_ptr, state_bytes), "pp_set_trainable_mask")


def pp_local_step(h, tokens_ptr: int, targets_ptr: int, B: int, S: int, opt, loss_ptr: int):
    _check(load_library().pp_local_step(h, tokens_ptr, targets_ptr, B, S, None if opt is None else C.byref(opt), loss_ptr), "pp_local_step")


def pp_set_jacobian_slices(h, mode: int, extra_lo: int = 0, extra_hi: int = 0):
    _check(load_library().pp_set_jacobian_slices(h, mode, extra_lo, extra_hi), "pp_set_jacobian_slices")


def pp_outer_delta_group(h, layer_lo: int, layer_hi: int, ends: int, theta_g_ptr: int, momentum_ptr: int, others_ptr, opt: PPOuter, delta_out_ptr):
    _check(load_library().pp_outer_delta_group(h, layer_lo, layer_hi, ends, theta_g_ptr, momentum_ptr, others_ptr, C.byref(opt), delta_out_ptr),
           "pp_outer_delta_group")


def pp_outer_delta(h, theta_g_ptr: int, momentum_ptr: int, others_ptr, opt: PPOuter, delta_out_ptr):
    _check(load_library().pp_outer_delta(h, theta_g_ptr, momentum_ptr, others_ptr, C.byref(opt), delta_out_ptr), "pp_outer_delta")


def pp_synth_delta_sum(h, dst_ptr: int, n: int, keys, std: float):
    arr = (C.c_uint64 * len(keys))(*[int(k) for k in keys])
    _check(load_library().pp_synth_delta_sum(h, dst_ptr, n, arr, len(keys), std), "pp_synth_delta_sum")


def pp_get_counters(h):
    f, b, a, n = C.c_double(), C.c_double(), C.c_double(), C.c_int64()
    _check(load_library().pp_get_counters(h, C.byref(f), C.byref(b), C.byref(a), C.byref(n)), "pp_get_counters")
    return dict(flops_fwd=f.value, flops_bwd=b.value, adamw_bytes=a.value, n_trainable=n.value)


def pp_get_launch_counts(h):
    a, b = C.c_int64(), C.c_int64()
    _check(load_library().pp_get_launch_counts(h, C.byref(a), C.byref(b)), "pp_get_launch_counts")
    return dict(matrix_core_calls=a.value, plain_calls=b.value)


def pp_get_gemm_timing(h):
    ms, fl, n = C.c_double(), C.c_double(), C.c_int64()
    _check(load_library().pp_get_gemm_timing(h, C.byref(ms), C.byref(fl), C.byref(n)), "pp_get_gemm_timing")
    return dict(ms=ms.value, flops=fl.value, launches=n.value)


def pp_set_option(h, key: str, value: int):
    _check(load_library().pp_set_option(h, key.encode(), value), "pp_set_option")


def pp_free(h):
    load_library().pp_free(h)


def pp_op_gemm_nt(stream: int, dtype: int, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, M, N, K, R_ptr=None, out_f32=0, splits=1,
                  scratch_ptr=None, path=0):
    _check(load_library().pp_op_gemm_nt(stream, dtype, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, M, N, K, R_ptr, out_f32, splits,
                                        scratch_ptr, path), "pp_op_gemm_nt")


def pp_op_gemm_tn(stream: int, A_ptr, lda, m_blk, a_blk_stride, B_ptr, ldb, C_ptr, ldc, M, N, K, splits=1, scratch_ptr=None):
    _check(load_library().pp_op_gemm_tn(stream, A_ptr, lda, m_blk, a_blk_stride, B_ptr, ldb, C_ptr, ldc, M, N, K, splits, scratch_ptr), "pp_op_gemm_tn")


def pp_op_gemm_nt_splitk_static(stream: int, dtype: int, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, M, N, K, splits, path=0):
    _check(load_library().pp_op_gemm_nt_splitk_static(stream, dtype, A_ptr, lda, B_ptr, ldb, C_ptr, ldc, M, N, K, splits, path),
           "pp_op_gemm_nt_splitk_static")


def pp_op_attention_fwd(stream: int, dtype: int, qkv_ptr, o_ptr, lse_ptr, scratch_ptr, B, S, h, dh, path=0):
    _check(load_library().pp_op_attention_fwd(stream, dtype, qkv_ptr, o_ptr, lse_ptr, scratch_ptr, B, S, h, dh, path), "pp_op_attention_fwd")


def pp_op_attention_bwd(stream: int, dtype: int, qkv_ptr, o_ptr, lse_ptr, dO_ptr, dqkv_ptr, D_ptr, scratch_ptr, B, S, h, dh, path=0):
    _check(load_library().pp_op_attention_bwd(stream, dtype, qkv_ptr, o_ptr, lse_ptr, dO_ptr, dqkv_ptr, D_ptr, scratch_ptr, B, S, h, dh, path),
           "pp_op_attention_bwd")


# --------------------------------------------------------------------------------------------- convenience holder
def make_config(cfg: dict) -> PPConfig:
    return PPConfig(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["d_ff"], cfg["vocab"], cfg.get("max_batch", cfg["batch"]),
                    cfg.get("max_seq", cfg["seq"]), PP_BF16 if cfg["dtype"] == "bf16" else PP_F32, cfg["rms_eps"], cfg["rope_base"], int(cfg.get("recompute", 0)))


def make_mask(mask: dict) -> PPMask:
    return PPMask(int(mask.get("all", 0)), mask.get("ffn_lo", 0), mask.get("ffn_hi", 0), mask.get("head_lo", 0), mask.get("head_hi", 0),
                  int(mask.get("train_wo", 0)), int(mask.get("train_norms", 0)), int(mask.get("train_embed", 0)), int(mask.get("train_lm_head", 0)))


class LocalStepModel:
    """Owns the device buffers (torch allocations) for one pp_model handle and forwards to the C entry points."""

    def __init__(self, cfg: dict, mask: dict, device: str = "cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise PPError("no GPU visible: the HIP path has no CPU fallback")
        self.torch = torch
        self.dev = torch.device(device)
        self.cfg = dict(cfg)
        self.ccfg = make_config(cfg)
        self.cmask = make_mask(mask)
        self.bf16 = cfg["dtype"] == "bf16"
        self.stream = torch.cuda.current_stream(self.dev)
        self.bytes_params = pp_query_bytes(self.ccfg, None, PP_BYTES_PARAMS)
        self.bytes_ws = pp_query_bytes(self.ccfg, self.cmask, PP_BYTES_WORKSPACE)
        self.bytes_state = pp_query_bytes(self.ccfg, self.cmask, PP_BYTES_STATE)
        self.bytes_shadow = pp_query_bytes(self.ccfg, self.cmask, PP_BYTES_SHADOW)
        self.bytes_act = pp_query_bytes(self.ccfg, self.cmask, PP_BYTES_ACTIVATIONS)
        self.params = torch.zeros(self.bytes_params, dtype=torch.uint8, device=self.dev)
        self.ws = torch.empty(self.bytes_ws, dtype=torch.uint8, device=self.dev)
        self.state = torch.empty(max(self.bytes_state, 256), dtype=torch.uint8, device=self.dev)
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.dev)
        self.h = pp_init_model(self.ccfg, self.params.data_ptr(), self.bytes_params, self.ws.data_ptr(), self.bytes_ws, self.stream.cuda_stream)
        self.mask_set = False

    def close(self):
        if self.h is not None:
            self.torch.cuda.synchronize(self.dev)
            pp_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # weights are exchanged as float32 numpy arrays holding exactly representable storage values
    def _to_storage(self, w: np.ndarray) -> np.ndarray:
        w = np.ascontiguousarray(w, dtype=np.float32)
        if not self.bf16:
            return w
        return (w.view(np.uint32) >> np.uint32(16)).astype(np.uint16)

    def _from_storage(self, raw: np.ndarray) -> np.ndarray:
        if not self.bf16:
            return raw
        return (raw.astype(np.uint32) << np.uint32(16)).view(np.float32)

    def load_weights(self, weights: dict):
        for name, w in weights.items():
            pp_set_tensor(self.h, name, self._to_storage(w))

    def set_mask(self, mask: dict | None = None):
        if mask is not None:
            self.cmask = make_mask(mask)
            need_ws = pp_query_bytes(self.ccfg, self.cmask, PP_BYTES_WORKSPACE)
            need_state = pp_query_bytes(self.ccfg, self.cmask, PP_BYTES_STATE)
            if need_ws > self.bytes_ws:
                raise PPError("workspace was sized for a smaller mask")
            if need_state > self.state.numel():
                self.state = self.torch.empty(need_state, dtype=self.torch.uint8, device=self.dev)
            self.bytes_state = need_state
        pp_set_trainable_mask(self.h, self.cmask, self.state.data_ptr(), self.state.numel())
        self.mask_set = True
        self.n_trainable = pp_get_counters(self.h)["n_trainable"]

    def get_weight(self, name: str, shape) -> np.ndarray:
        raw = np.empty(shape, dtype=np.uint16 if self.bf16 else np.float32)
        pp_get_tensor(self.h, name, raw)
        return self._from_storage(raw)

    def get_raw(self, name: str, shape, dtype) -> np.ndarray:
        return pp_get_tensor(self.h, name, np.empty(shape, dtype=dtype))

    def get_state(self, which: str) -> np.ndarray:
        return pp_get_tensor(self.h, "state." + which, np.empty(self.n_trainable, dtype=np.float32))

    def upload_tokens(self, tokens: np.ndarray, targets: np.ndarray):
        t = self.torch
        return (t.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(self.dev),
                t.from_numpy(np.ascontiguousarray(targets, dtype=np.int32)).to(self.dev))

    def step(self, tokens_dev, targets_dev, hp: dict | None):
        """Enqueues one local step; returns the device loss tensor (no sync)."""
        B, S = tokens_dev.shape
        opt = None if hp is None else PPAdamW(hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"])
        pp_local_step(self.h, tokens_dev.data_ptr(), targets_dev.data_ptr(), B, S, opt, self.loss.data_ptr())
        return self.loss

    def counters(self):
        return pp_get_counters(self.h)

    def launch_counts(self):
        return pp_get_launch_counts(self.h)

    def set_option(self, key: str, value: int):
        pp_set_option(self.h, key, value)

    def set_jacobian_slices(self, mode: int, extra_lo: int = 0, extra_hi: int = 0):
        pp_set_jacobian_slices(self.h, mode, extra_lo, extra_hi)

    def gemm_timing(self):
        return pp_get_gemm_timing(self.h)

    def memory_report(self) -> dict:
        return dict(params=self.bytes_params, state=self.bytes_state, workspace=self.bytes_ws, shadow=self.bytes_shadow,
                    activations=self.bytes_act, total=self.bytes_params + self.bytes_state + self.bytes_ws)
