"""ctypes binding of liblemix_stage.so: argument marshalling only.

Function and method names follow include/lemix_stage.h and
include/lemix_kernels.h.  Tensors are torch tensors on the GPU (torch is used
for device memory and streams, nothing else); every compute step runs in the
library's kernels.  Loading fails loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblemix_stage.so")

LS_OK, LS_EINVAL, LS_ENOMEM, LS_EHIP, LS_ESTATE = 0, -1, -2, -3, -4
LS_BLOCK_GPT_PRELN, LS_BLOCK_LLAMA = 0, 1
LS_F32, LS_BF16, LS_F16 = 0, 1, 2
LS_ACT_GELU_TANH, LS_ACT_GELU_ERF, LS_ACT_SWIGLU = 0, 1, 2

DTYPE_CODE = {"f32": LS_F32, "bf16": LS_BF16, "f16": LS_F16}
TORCH_DTYPE = {LS_F32: torch.float32, LS_BF16: torch.bfloat16, LS_F16: torch.float16}
CODE_OF_TORCH = {v: k for k, v in TORCH_DTYPE.items()}
BLOCK_CODE = {"gpt": LS_BLOCK_GPT_PRELN, "llama": LS_BLOCK_LLAMA}
ACT_CODE = {"gelu_tanh": LS_ACT_GELU_TANH, "gelu_erf": LS_ACT_GELU_ERF, "swiglu": LS_ACT_SWIGLU}


class LsError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"lemix_stage status {status}: {msg}")
        self.status = status


class ls_config(C.Structure):
    _fields_ = [("block", C.c_int32), ("dtype", C.c_int32), ("io_dtype", C.c_int32),
                ("mma_dtype", C.c_int32), ("act", C.c_int32), ("n_layers", C.c_int32),
                ("d_model", C.c_int32), ("n_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ff", C.c_int32), ("norm_eps", C.c_float), ("rope_theta", C.c_float),
                ("page_size", C.c_int32), ("max_pos", C.c_int32)]


class ls_optim(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float), ("momentum", C.c_float),
                ("grad_scale", C.c_float), ("step", C.c_int32)]


LS_OPT_SGD, LS_OPT_ADAMW = 0, 1


class ls_kv(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("block_table", C.c_void_p),
                ("ctx_len", C.c_void_p), ("ctx_len_host", C.c_void_p),
                ("n_pages", C.c_int32), ("max_pages_per_req", C.c_int32)]


_lib: Optional[C.CDLL] = None

# name -> (restype, argtypes); every symbol the two headers declare
_VP, _I, _L, _SZ, _F = C.c_void_p, C.c_int, C.c_long, C.c_size_t, C.c_float
_D, _DP = C.c_double, C.POINTER(C.c_double)
SIGNATURES = {
    "ls_create": (_I, [C.POINTER(ls_config), C.POINTER(_VP)]),
    "ls_destroy": (None, [_VP]),
    "ls_param_count": (_SZ, [_VP]),
    "ls_get_config": (_I, [_VP, C.POINTER(ls_config)]),
    "ls_bind_params": (_I, [_VP, _VP, _VP]),
    "ls_workspace_bytes": (_SZ, [_VP, _I]),
    "ls_saved_bytes": (_SZ, [_VP, _I, _I]),
    "stage_prefill": (_I, [_VP, _VP, C.POINTER(C.c_int32), _I, C.POINTER(ls_kv), _VP, _VP, _VP]),
    "stage_decode": (_I, [_VP, _VP, _I, C.POINTER(ls_kv), _VP, _VP, _VP]),
    "stage_step": (_I, [_VP, _VP, _I, C.POINTER(C.c_int32), _I, C.POINTER(ls_kv), _VP, _VP, _VP]),
    "stage_train_fwd": (_I, [_VP, _VP, _I, _I, _VP, _VP, _VP, _VP]),
    "stage_train_bwd": (_I, [_VP, _VP, _I, _I, _VP, _VP, _VP, _I, _VP, _VP]),
    "stage_probe_interference": (_I, [_VP, _VP, _I, C.POINTER(ls_kv), _VP, _VP, _VP, _I, _I, _VP, _VP,
                                      _VP, _VP, _VP, _VP, _VP, _VP, _I, C.POINTER(C.c_float)]),
    "stage_optimizer_step": (_I, [_VP, C.POINTER(ls_optim), _VP, _VP, _VP, _VP, _VP, _VP]),
    "ls_last_error": (C.c_char_p, []),
    "lsk_timing_begin": (_I, []),
    "lsk_timing_end": (_I, [_DP, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "lsk_gemm": (_I, [_I, _I, _I, _I, _VP, _L, _I, _VP, _L, _I, _VP, _L, _I, _VP, _I, _VP, _L, _I, _VP]),
    "lsk_gemm_ws": (_I, [_I, _I, _I, _I, _VP, _L, _VP, _L, _VP, _L, _I, _VP, _I, _VP, _L, _VP, _SZ, _VP]),
    "lsk_kv_packed_bytes": (_SZ, [C.POINTER(ls_config), _I]),
    "lsk_kv_offload": (_I, [C.POINTER(ls_config), C.POINTER(ls_kv), _I, _I, _VP, _VP, _VP]),
    "lsk_kv_reload": (_I, [C.POINTER(ls_config), C.POINTER(ls_kv), _I, _I, _VP, _VP, _VP]),
    "lsk_memory_available": (_I, [_SZ, _SZ, C.POINTER(C.c_int), C.POINTER(_SZ)]),
    "lsk_optimizer": (_I, [_I, _F, _F, _F, _F, _F, _F, _F, _I, _SZ, _VP, _VP, _VP, _VP, _VP, _I, _VP, _I, _VP]),
    "lsk_convert": (_I, [_VP, _I, _VP, _I, _SZ, _VP]),
    "lsk_grad_scale": (_I, [_VP, _I, _SZ, _VP, _VP]),
    "lsk_gemm_scaled": (_I, [_I, _I, _I, _I, _VP, _L, _I, _VP, _L, _I, _VP, _L, _I, _VP, _I, _VP, _L, _I, _VP, _VP]),
    "lsk_convert_scaled": (_I, [_VP, _I, _VP, _I, _SZ, _VP, _VP]),
    "lsk_norm_bwd_scaled": (_I, [_I, _VP, _I, _VP, _VP, _VP, _VP, _I, _I, _I, _VP, _VP, _VP, _I, _VP, _VP, _I,
                                 _VP, _VP, _VP]),
    "lsk_colsum_scaled": (_I, [_VP, _I, _I, _I, _L, _VP, _I, _VP, _VP, _VP]),
    "lsk_norm_fwd": (_I, [_I, _VP, _I, _I, _VP, _VP, _I, _F, _VP, _I, _VP, _VP, _VP]),
    "lsk_norm_bwd_partial_floats": (_SZ, [_I, _I]),
    "lsk_norm_bwd": (_I, [_I, _VP, _I, _VP, _VP, _VP, _VP, _I, _I, _I, _VP, _VP, _VP, _I, _VP, _VP, _I,
                          _VP, _VP]),
    "lsk_rope": (_I, [_VP, _I, _I, _I, _I, _VP, _VP, _F, _VP]),
    "lsk_gelu_fwd": (_I, [_VP, _VP, _I, _SZ, _I, _VP]),
    "lsk_gelu_bwd": (_I, [_VP, _VP, _VP, _I, _SZ, _I, _VP]),
    "lsk_swiglu_fwd": (_I, [_VP, _VP, _I, _I, _I, _VP]),
    "lsk_swiglu_bwd": (_I, [_VP, _VP, _VP, _I, _I, _I, _VP]),
    "lsk_colsum_partial_floats": (_SZ, [_I, _I]),
    "lsk_colsum": (_I, [_VP, _I, _I, _I, _L, _VP, _I, _VP, _VP]),
    "lsk_attn_fwd": (_I, [_I, _VP, _I, _I, _I, _I, _I, _VP, _VP, _VP]),
    "lsk_attn_bwd": (_I, [_I, _VP, _VP, _VP, _VP, _I, _I, _I, _I, _I, _VP, _VP, _VP]),
    "lsk_attn_bwd_scratch_floats": (_SZ, [_I, _I, _I]),
    "lsk_attn_bwd_rope": (_I, [_I, _VP, _VP, _VP, _VP, _I, _I, _I, _I, _I, _VP, _VP, _VP, _VP, _VP]),
    "lsk_gemm_qkv_rope": (_I, [_I, _I, _I, _VP, _VP, _VP, _I, _I, _VP, _VP, _VP]),
    "lsk_gemm_swiglu_bwd": (_I, [_I, _I, _I, _I, _VP, _VP, _VP, _VP, _VP, _VP]),
    "lsk_kv_write": (_I, [_VP, _I, _I, _I, _I, _VP, _VP, _VP, _VP, _VP, _I, _I, _VP]),
    "lsk_rope_kv_write": (_I, [_VP, _I, _I, _I, _I, _VP, _VP, _VP, _VP, _VP, _VP, _I, _I, _VP]),
    "lsk_attn_paged": (_I, [_I, _VP, _I, _I, _I, _I, _VP, _VP, _VP, _VP, _VP, _I, _I, _I, _VP, _VP, _VP]),
    "lsk_attn_paged_scratch_floats": (_SZ, [_I, _I, _I, _I, _I]),
    "lsk_attn_paged_noalloc": (_I, [_VP, _I, _I, _I, _I, _VP, _VP, _VP, _VP, _VP, _I, _I, _I, _VP, _VP]),
    "lsk_gemm_partials": (_I, [_I, _I, _I, _I, _VP, _L, _VP, _L, _VP, _SZ, C.POINTER(_I), _VP]),
    "lsk_finish_resid_norm": (_I, [_VP, _I, _I, _I, _VP, _VP, _VP, _I, _VP, _VP, _I, _F, _VP, _I, _VP]),
    "lsk_finish_act": (_I, [_VP, _I, _I, _I, _I, _VP, _I, _VP, _I, _VP]),
    "lsk_finish_qkv": (_I, [_VP, _I, _I, _I, _I, _VP, _I, _VP, _VP, _VP, _VP, _I, _VP, _VP, _VP, _I, _I, _VP]),
    # lemix_sched.h (host bookkeeping; wrappers in sched.py)
    "ls_node_create": (_I, [_I, _D, _D, C.POINTER(_VP)]),
    "ls_node_destroy": (None, [_VP]),
    "ls_node_plan": (_I, [_VP, _VP, _I, _DP, _DP, _DP, C.POINTER(C.c_int64)]),
    "ls_node_queue_len": (_I, [_VP, _I]),
    "ls_node_prune": (_I, [_VP]),
    "ls_node_task_path": (_I, [_VP, C.c_int64, _DP]),
    "ls_node_calibrate": (_I, [_VP, C.c_int64, _I, _I, _D, _D]),
    "ls_node_score": (_I, [_VP, _VP, _D, _VP, _DP, _DP, _DP, _DP, _DP]),
    "ls_select_node": (_I, [C.POINTER(_VP), _I, _VP, _D, _VP, C.POINTER(_I), _DP]),
    "ls_deprioritize": (_I, [C.POINTER(_VP), _I, _VP, _D, C.POINTER(_I), _DP]),
    "ls_node_execute": (_I, [_VP, _D, _D, _VP, _VP]),
    "ls_batcher_create": (_I, [_I, _D, C.POINTER(_VP)]),
    "ls_batcher_destroy": (None, [_VP]),
    "ls_batcher_push": (_I, [_VP, C.c_int64, _I]),
    "ls_batcher_form": (_I, [_VP, _D, C.POINTER(C.c_int64), C.POINTER(_I), C.POINTER(_I), C.POINTER(_I)]),
    "ls_batcher_take_training": (_I, [_VP, C.POINTER(C.c_int64)]),
    "ls_batcher_finish": (_I, [_VP, C.POINTER(C.c_int64), _I]),
    "ls_batcher_queued": (_I, [_VP]),
    "ls_batcher_batch_size": (_I, [_VP]),
    # lemix_profile.h (wrappers and structures in profiler.py)
    "ls_profile_reduce": (_I, [_VP, _I, _VP]),
    "ls_profile_memory_threshold": (_I, [_D, _DP, _I, _DP, _DP]),
    "ls_profile_time_train": (_I, [_VP, _VP, _I, _I, _VP, _VP, _VP, _VP, _VP, _VP, _VP, _I, _DP, _DP]),
    "ls_profile_time_prefill": (_I, [_VP, _VP, C.POINTER(C.c_int32), _I, _VP, _VP, _VP, _VP, _I, _DP]),
    # lemix_serve.h (wrappers in sched.py)
    "ls_server_create": (_I, [_VP, _VP, _VP, _VP, C.POINTER(_VP)]),
    "ls_server_destroy": (None, [_VP]),
    "ls_server_submit": (_I, [_VP, C.c_int64, _VP, _VP, _I, _I]),
    "ls_server_pass": (_I, [_VP, _D, _VP, _VP, _VP, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
    "ls_server_in_flight": (_I, [_VP]),
}


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2507_21276_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != LS_OK:
        raise LsError(status, lib().ls_last_error().decode())


def _p(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return t.data_ptr()
    return int(t)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    return stream.cuda_stream if isinstance(stream, torch.cuda.Stream) else int(stream)


def make_config(cfg: dict, io_dtype: Optional[str] = None, mma_dtype: Optional[str] = None) -> ls_config:
    dt = DTYPE_CODE[cfg["dtype"]]
    io = DTYPE_CODE[io_dtype or cfg.get("io_dtype", cfg["dtype"])]
    mma = DTYPE_CODE[mma_dtype or cfg.get("mma_dtype", "f32" if cfg["dtype"] == "f32" else "f16")]
    return ls_config(BLOCK_CODE[cfg["block"]], dt, io, mma, ACT_CODE[cfg["act"]], cfg["n_layers"],
                     cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["d_ff"], cfg["norm_eps"],
                     cfg["rope_theta"], cfg["page_size"], cfg["max_pos"])


class KV:
    """Caller-owned paged KV cache (torch tensors) plus the ls_kv descriptor."""

    def __init__(self, stage: "Stage", n_pages: int, block_table, ctx_len, device="cuda"):
        c = stage.c
        self.stage = stage
        shape = (c.n_layers, n_pages, c.n_heads, c.page_size, c.head_dim)
        dt = TORCH_DTYPE[c.mma_dtype]
        self.k_pool = torch.zeros(shape, dtype=dt, device=device)
        self.v_pool = torch.zeros(shape, dtype=dt, device=device)
        self.block_table = torch.as_tensor(block_table, dtype=torch.int32).contiguous().to(device)
        self.n_pages = n_pages
        self.set_ctx(ctx_len, device)

    def set_ctx(self, ctx_len, device="cuda"):
        self.ctx_host = torch.as_tensor(ctx_len, dtype=torch.int32).contiguous().clone()
        self.ctx_len = self.ctx_host.to(device)

    def desc(self, with_host=True) -> ls_kv:
        return ls_kv(self.k_pool.data_ptr(), self.v_pool.data_ptr(), self.block_table.data_ptr(),
                     self.ctx_len.data_ptr(), self.ctx_host.data_ptr() if with_host else None,
                     self.n_pages, self.block_table.shape[1])


class Stage:
    """Thin owner of an ls_stage handle; methods are the C entry points."""

    def __init__(self, cfg: dict, io_dtype: Optional[str] = None, mma_dtype: Optional[str] = None):
        self.c = make_config(cfg, io_dtype, mma_dtype)
        self.h = C.c_void_p()
        _check(lib().ls_create(C.byref(self.c), C.byref(self.h)))
        self.io_torch = TORCH_DTYPE[self.c.io_dtype]
        self.param_torch = TORCH_DTYPE[self.c.dtype]
        self._params = None

    def close(self):
        if self.h:
            lib().ls_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def ls_param_count(self) -> int:
        return lib().ls_param_count(self.h)

    def ls_bind_params(self, params: torch.Tensor, stream=None):
        assert params.dtype == self.param_torch and params.numel() == self.ls_param_count()
        self._params = params
        _check(lib().ls_bind_params(self.h, _p(params), _stream(stream)))

    def ls_workspace_bytes(self, max_tokens: int) -> int:
        return lib().ls_workspace_bytes(self.h, max_tokens)

    def ls_saved_bytes(self, B: int, L: int) -> int:
        return lib().ls_saved_bytes(self.h, B, L)

    def new_workspace(self, max_tokens: int, device="cuda") -> torch.Tensor:
        return torch.empty(self.ls_workspace_bytes(max_tokens), dtype=torch.uint8, device=device)

    def new_saved(self, B: int, L: int, device="cuda") -> torch.Tensor:
        return torch.empty(self.ls_saved_bytes(B, L), dtype=torch.uint8, device=device)

    def stage_prefill(self, X, chunk_len, kv: KV, Y, workspace, stream=None, with_host=True):
        cl = (C.c_int32 * len(chunk_len))(*[int(v) for v in chunk_len])
        d = kv.desc(with_host)
        _check(lib().stage_prefill(self.h, _p(X), cl, len(chunk_len), C.byref(d), _p(Y), _p(workspace),
                                   _stream(stream)))

    def stage_step(self, X, n_decode, chunk_len, kv: KV, Y, workspace, stream=None, with_host=True):
        cl = (C.c_int32 * max(1, len(chunk_len)))(*[int(v) for v in chunk_len])
        d = kv.desc(with_host)
        _check(lib().stage_step(self.h, _p(X), n_decode, cl, len(chunk_len), C.byref(d), _p(Y), _p(workspace),
                                _stream(stream)))

    def stage_decode(self, X, B, kv: KV, Y, workspace, stream=None, with_host=True):
        d = kv.desc(with_host)
        _check(lib().stage_decode(self.h, _p(X), B, C.byref(d), _p(Y), _p(workspace), _stream(stream)))

    def stage_train_fwd(self, X, B, L, Y, saved, workspace, stream=None):
        _check(lib().stage_train_fwd(self.h, _p(X), B, L, _p(Y), _p(saved), _p(workspace), _stream(stream)))

    def stage_train_bwd(self, dY, B, L, saved, dX, dParams, accumulate, workspace, stream=None):
        assert dParams.dtype == torch.float32
        _check(lib().stage_train_bwd(self.h, _p(dY), B, L, _p(saved), _p(dX), _p(dParams),
                                     int(accumulate), _p(workspace), _stream(stream)))

    def stage_optimizer_step(self, params, master, m, v, dParams, *, kind, lr, step, beta1=0.9, beta2=0.999,
                             eps=1e-8, weight_decay=0.0, momentum=0.0, grad_scale=1.0, stream=None):
        o = ls_optim(kind, lr, beta1, beta2, eps, weight_decay, momentum, grad_scale, step)
        _check(lib().stage_optimizer_step(self.h, C.byref(o), _p(params), _p(master), _p(m),
                                          _p(v) if v is not None else None, _p(dParams), _stream(stream)))

    def stage_probe_interference(self, dec_X, dec_B, kv: KV, dec_Y, ws_a, trn_X, trn_B, trn_L, trn_Y,
                                 trn_saved, trn_dY, trn_dX, trn_dParams, ws_b, stream_a, stream_b,
                                 iters):
        out = (C.c_float * 6)()
        d = kv.desc(True)
        _check(lib().stage_probe_interference(
            self.h, _p(dec_X), dec_B, C.byref(d), _p(dec_Y), _p(ws_a), _p(trn_X), trn_B, trn_L,
            _p(trn_Y), _p(trn_saved), _p(trn_dY), _p(trn_dX), _p(trn_dParams), _p(ws_b),
            stream_a.cuda_stream, stream_b.cuda_stream, iters, out))
        return list(out)


# ---- kernel-level entry points (same names as the C symbols) -------------------------

def lsk_gemm(A, B, C_out, *, M, N, K, a_kmajor=True, b_kmajor=True, lda=None, ldb=None, ldc=None,
             bias=None, resid=None, ldr=None, accumulate=False, stream=None):
    op = CODE_OF_TORCH[A.dtype]
    _check(lib().lsk_gemm(op, M, N, K, _p(A), lda if lda is not None else (K if a_kmajor else M),
                          int(a_kmajor), _p(B), ldb if ldb is not None else (K if b_kmajor else N),
                          int(b_kmajor), _p(C_out), ldc if ldc is not None else N,
                          CODE_OF_TORCH[C_out.dtype], _p(bias),
                          CODE_OF_TORCH[bias.dtype] if bias is not None else 0, _p(resid),
                          ldr if ldr is not None else N, int(accumulate), _stream(stream)))


def lsk_grad_scale(x, out3, stream=None):
    _check(lib().lsk_grad_scale(_p(x), CODE_OF_TORCH[x.dtype], x.numel(), _p(out3), _stream(stream)))


def lsk_convert(src, dst, stream=None):
    _check(lib().lsk_convert(_p(src), CODE_OF_TORCH[src.dtype], _p(dst), CODE_OF_TORCH[dst.dtype],
                             src.numel(), _stream(stream)))


def lsk_norm_fwd(kind, x, gamma, beta, eps, h, mean, rstd, stream=None):
    T, d = x.shape
    _check(lib().lsk_norm_fwd(kind, _p(x), T, d, _p(gamma), _p(beta), CODE_OF_TORCH[gamma.dtype], eps,
                              _p(h), CODE_OF_TORCH[h.dtype], _p(mean), _p(rstd), _stream(stream)))


def lsk_norm_bwd(kind, dh, x, mean, rstd, gamma, dres, dx, dx16, dgamma, dbeta, accumulate, stream=None):
    T, d = x.shape
    partial = torch.empty(lib().lsk_norm_bwd_partial_floats(T, d), dtype=torch.float32, device=x.device)
    _check(lib().lsk_norm_bwd(kind, _p(dh), CODE_OF_TORCH[dh.dtype], _p(x), _p(mean), _p(rstd), _p(gamma),
                              CODE_OF_TORCH[gamma.dtype], T, d, _p(dres), _p(dx), _p(dx16),
                              CODE_OF_TORCH[dx16.dtype] if dx16 is not None else 0, _p(dgamma),
                              _p(dbeta), int(accumulate), _p(partial), _stream(stream)))


def lsk_rope(qkv, n_heads, head_dim, pos, table, sign, stream=None):
    _check(lib().lsk_rope(_p(qkv), CODE_OF_TORCH[qkv.dtype], qkv.shape[0], n_heads, head_dim, _p(pos),
                          _p(table), sign, _stream(stream)))


def lsk_gelu_fwd(u, g, kind, stream=None):
    _check(lib().lsk_gelu_fwd(_p(u), _p(g), CODE_OF_TORCH[u.dtype], u.numel(), kind, _stream(stream)))


def lsk_gelu_bwd(dg, u, du, kind, stream=None):
    _check(lib().lsk_gelu_bwd(_p(dg), _p(u), _p(du), CODE_OF_TORCH[u.dtype], u.numel(), kind,
                              _stream(stream)))


def lsk_swiglu_fwd(gu, a, stream=None):
    T, F = a.shape
    _check(lib().lsk_swiglu_fwd(_p(gu), _p(a), CODE_OF_TORCH[gu.dtype], T, F, _stream(stream)))


def lsk_swiglu_bwd(da, gu, dgu, stream=None):
    T, F = da.shape
    _check(lib().lsk_swiglu_bwd(_p(da), _p(gu), _p(dgu), CODE_OF_TORCH[gu.dtype], T, F, _stream(stream)))


def lsk_colsum(x, out, accumulate=False, stream=None):
    T, N = x.shape
    partial = torch.empty(lib().lsk_colsum_partial_floats(T, N), dtype=torch.float32, device=x.device)
    _check(lib().lsk_colsum(_p(x), CODE_OF_TORCH[x.dtype], T, N, N, _p(out), int(accumulate), _p(partial),
                            _stream(stream)))


def lsk_attn_fwd(impl, qkv, B, L, n_heads, head_dim, o, lse, stream=None):
    _check(lib().lsk_attn_fwd(impl, _p(qkv), CODE_OF_TORCH[qkv.dtype], B, L, n_heads, head_dim, _p(o),
                              _p(lse), _stream(stream)))


def lsk_attn_bwd(impl, qkv, o, dO, lse, B, L, n_heads, head_dim, dqkv, stream=None):
    dvec = torch.empty(lib().lsk_attn_bwd_scratch_floats(B, L, n_heads), dtype=torch.float32, device=qkv.device)
    _check(lib().lsk_attn_bwd(impl, _p(qkv), _p(o), _p(dO), _p(lse), CODE_OF_TORCH[qkv.dtype], B, L,
                              n_heads, head_dim, _p(dqkv), _p(dvec), _stream(stream)))


def lsk_kv_packed_bytes(stage, n_tokens):
    return lib().lsk_kv_packed_bytes(C.byref(stage.c), n_tokens)


def lsk_kv_offload(stage, kv, request, n_tokens, staging, host_buf, stream=None):
    d = kv.desc(True)
    _check(lib().lsk_kv_offload(C.byref(stage.c), C.byref(d), request, n_tokens, _p(staging), host_buf.data_ptr(),
                                _stream(stream)))


def lsk_kv_reload(stage, kv, request, n_tokens, host_buf, staging, stream=None):
    d = kv.desc(True)
    _check(lib().lsk_kv_reload(C.byref(stage.c), C.byref(d), request, n_tokens, host_buf.data_ptr(), _p(staging),
                               _stream(stream)))


def lsk_memory_available(need_bytes, threshold_bytes):
    ok, used = C.c_int(0), C.c_size_t(0)
    _check(lib().lsk_memory_available(need_bytes, threshold_bytes, C.byref(ok), C.byref(used)))
    return bool(ok.value), used.value


def lsk_optimizer(kind, grad, m, v, master, params, params_op, *, lr, step, beta1=0.9, beta2=0.999, eps=1e-8,
                  weight_decay=0.0, momentum=0.0, grad_scale=1.0, stream=None):
    _check(lib().lsk_optimizer(kind, lr, beta1, beta2, eps, weight_decay, momentum, grad_scale, step,
                               grad.numel(), _p(grad), _p(m), _p(v) if v is not None else None, _p(master),
                               _p(params), CODE_OF_TORCH[params.dtype],
                               _p(params_op) if params_op is not None else None,
                               CODE_OF_TORCH[params_op.dtype] if params_op is not None else 0,
                               _stream(stream)))


def lsk_gemm_ws(x, w, c, scratch, bias=None, resid=None, stream=None):
    """C[M, N] = X[M, K] W[N, K]^T (+ bias + resid) with an fp32 workspace for the split-K path."""
    M, K = x.shape
    N = w.shape[0]
    _check(lib().lsk_gemm_ws(CODE_OF_TORCH[x.dtype], M, N, K, _p(x), x.stride(0), _p(w), w.stride(0), _p(c),
                             c.stride(0), CODE_OF_TORCH[c.dtype], _p(bias) if bias is not None else None,
                             CODE_OF_TORCH[bias.dtype] if bias is not None else 0,
                             _p(resid) if resid is not None else None,
                             resid.stride(0) if resid is not None else 0, _p(scratch), scratch.numel(),
                             _stream(stream)))


def lsk_attn_bwd_rope(impl, qkv, o, dO, lse, B, L, n_heads, head_dim, dqkv, pos, table, stream=None):
    dvec = torch.empty(lib().lsk_attn_bwd_scratch_floats(B, L, n_heads), dtype=torch.float32, device=qkv.device)
    _check(lib().lsk_attn_bwd_rope(impl, _p(qkv), _p(o), _p(dO), _p(lse), CODE_OF_TORCH[qkv.dtype], B, L,
                                   n_heads, head_dim, _p(dqkv), _p(dvec), _p(pos), _p(table), _stream(stream)))


def lsk_gemm_qkv_rope(h, w, qkv, n_heads, head_dim, pos, table, stream=None):
    _check(lib().lsk_gemm_qkv_rope(CODE_OF_TORCH[h.dtype], h.shape[0], h.shape[1], _p(h), _p(w), _p(qkv),
                                   n_heads, head_dim, _p(pos), _p(table), _stream(stream)))


def lsk_gemm_swiglu_bwd(dY, Wd, pre, grad, da_scratch, stream=None):
    T, d = dY.shape
    F = Wd.shape[1]
    _check(lib().lsk_gemm_swiglu_bwd(CODE_OF_TORCH[dY.dtype], T, F, d, _p(dY), _p(Wd), _p(pre), _p(grad), _p(da_scratch),
                                     _stream(stream)))


def lsk_rope_kv_write(qkv, n_heads, head_dim, pos, req, table, k_pool, v_pool, block_table, page_size, stream=None):
    _check(lib().lsk_rope_kv_write(_p(qkv), CODE_OF_TORCH[qkv.dtype], qkv.shape[0], n_heads, head_dim, _p(pos),
                                   _p(req), _p(table), _p(k_pool), _p(v_pool), _p(block_table),
                                   block_table.shape[1], page_size, _stream(stream)))


def lsk_kv_write(qkv, n_heads, head_dim, pos, req, k_pool, v_pool, block_table, page_size, stream=None):
    _check(lib().lsk_kv_write(_p(qkv), CODE_OF_TORCH[qkv.dtype], qkv.shape[0], n_heads, head_dim, _p(pos),
                              _p(req), _p(k_pool), _p(v_pool), _p(block_table), block_table.shape[1],
                              page_size, _stream(stream)))


def lsk_attn_paged(impl, qkv, n_heads, head_dim, pos, req, k_pool, v_pool, block_table, page_size,
                   max_ctx, o, stream=None):
    T = qkv.shape[0]
    n = lib().lsk_attn_paged_scratch_floats(T, n_heads, head_dim, max_ctx, page_size)
    scratch = torch.empty(max(n, 1), dtype=torch.float32, device=qkv.device)
    _check(lib().lsk_attn_paged(impl, _p(qkv), CODE_OF_TORCH[qkv.dtype], T, n_heads, head_dim, _p(pos),
                                _p(req), _p(k_pool), _p(v_pool), _p(block_table), block_table.shape[1],
                                page_size, max_ctx, _p(o), _p(scratch), _stream(stream)))


def lsk_attn_paged_noalloc(qkv, n_heads, head_dim, pos, req, k_pool, v_pool, block_table, page_size, max_ctx, o,
                           stream=None):
    _check(lib().lsk_attn_paged_noalloc(_p(qkv), CODE_OF_TORCH[qkv.dtype], qkv.shape[0], n_heads, head_dim, _p(pos),
                                        _p(req), _p(k_pool), _p(v_pool), _p(block_table), block_table.shape[1],
                                        page_size, max_ctx, _p(o), _stream(stream)))


TIMED_KINDS = ("gemm", "attn_fwd", "attn_bwd", "decode_attn", "decode_gemm", "finish")


def lsk_timing_begin():
    _check(lib().lsk_timing_begin())


def lsk_timing_end():
    """{kind: (milliseconds, bracketed calls)} of the recording that lsk_timing_begin started, plus "dropped"."""
    ms, calls, dropped = (C.c_double * len(TIMED_KINDS))(), (C.c_int32 * len(TIMED_KINDS))(), C.c_int32(0)
    _check(lib().lsk_timing_end(ms, calls, C.byref(dropped)))
    out = {k: (ms[i], calls[i]) for i, k in enumerate(TIMED_KINDS)}
    out["dropped"] = dropped.value
    return out


def _opt(t):
    return _p(t) if t is not None else None


def lsk_gemm_partials(x, w, partial, stream=None):
    """Split-K partial products of a decode batch: returns the number of splits written to partial[s][M][N]."""
    M, K = x.shape
    N = w.shape[0]
    splits = C.c_int(0)
    _check(lib().lsk_gemm_partials(CODE_OF_TORCH[x.dtype], M, N, K, _p(x), x.stride(0), _p(w), w.stride(0),
                                   _p(partial), partial.numel(), C.byref(splits), _stream(stream)))
    return splits.value


def lsk_finish_resid_norm(partial, splits, T, d, x_out, *, bias=None, resid=None, kind=-1, gamma=None, beta=None,
                          eps=1e-5, h=None, stream=None):
    pdt = CODE_OF_TORCH[(gamma if gamma is not None else bias).dtype] if (gamma is not None or bias is not None) else 0
    _check(lib().lsk_finish_resid_norm(_p(partial), splits, T, d, _opt(bias), _opt(resid), _p(x_out), kind,
                                       _opt(gamma), _opt(beta), pdt, eps, _opt(h),
                                       CODE_OF_TORCH[h.dtype] if h is not None else 0, _stream(stream)))


def lsk_finish_act(partial, splits, T, F, act, out, bias=None, stream=None):
    _check(lib().lsk_finish_act(_p(partial), splits, T, F, act, _opt(bias),
                                CODE_OF_TORCH[bias.dtype] if bias is not None else 0, _p(out),
                                CODE_OF_TORCH[out.dtype], _stream(stream)))


def lsk_finish_qkv(partial, splits, n_heads, head_dim, pos, req, table, qkv, k_pool, v_pool, block_table, page_size,
                   bias=None, stream=None):
    _check(lib().lsk_finish_qkv(_p(partial), splits, qkv.shape[0], n_heads, head_dim, _opt(bias),
                                CODE_OF_TORCH[bias.dtype] if bias is not None else 0, _p(pos), _p(req), _opt(table),
                                _p(qkv), CODE_OF_TORCH[qkv.dtype], _p(k_pool), _p(v_pool), _p(block_table),
                                block_table.shape[1], page_size, _stream(stream)))
