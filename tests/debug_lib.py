"""Test-only loader of libmi355attn_debug.so: the product's sources compiled with
-DATTN_DEBUG_ENTRY_POINTS, which adds entry points that let a test pick the kernel
(attn_fwd_variant, attn_bwd_plain).  The package itself never loads this library."""
import ctypes
import os

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PATH = os.path.join(_ROOT, "paper_2512_18134_amd", "libmi355attn_debug.so")

FWD_AS_DISPATCHED, FWD_PROGRAM_ORDER, FWD_D128_ONE_WAVE_PER_SIMD, FWD_D64_8_WAVES, FWD_D64_4_WAVES = range(5)
FWD_D128_TWO_WAVES_PER_SIMD = 5
ATTN_ERR_UNSUPPORTED = -7

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(PATH):
            raise RuntimeError("libmi355attn_debug.so is not built: run `python -m paper_2512_18134_amd.build`")
        _lib = ctypes.CDLL(PATH)
        _lib.attn_fwd_variant.restype = ctypes.c_int
        _lib.attn_fwd_variant.argtypes = ([ctypes.c_void_p] * 5 + [ctypes.c_int] * 6
                                          + [ctypes.c_float, ctypes.c_void_p, ctypes.c_int])
        _lib.attn_bwd_plain.restype = ctypes.c_int
        _lib.attn_bwd_plain.argtypes = [ctypes.c_void_p] * 10 + [ctypes.c_int] * 6 + [ctypes.c_float, ctypes.c_void_p]
    return _lib


def attn_fwd_variant(q, k, v, causal, scale, variant):
    """attn_fwd_variant on torch bf16 device tensors; returns (o, lse) or raises on a non-zero status."""
    import torch
    B, H, S_q, D = q.shape
    S_kv = k.shape[2]
    o = torch.full(q.shape, float("nan"), dtype=q.dtype, device=q.device)
    lse = torch.full((B, H, S_q), float("nan"), dtype=torch.float32, device=q.device)
    rc = lib().attn_fwd_variant(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, S_q, S_kv,
                                D, int(bool(causal)), float(scale), torch.cuda.current_stream().cuda_stream,
                                int(variant))
    if rc != 0:
        raise RuntimeError("attn_fwd_variant(%d): status %d" % (variant, rc))
    return o, lse


def attn_bwd_plain(q, k, v, o, d_o, lse, causal, scale):
    """attn_bwd_plain (compiler-scheduled sweeps) on torch bf16 device tensors; returns (dq, dk, dv)."""
    import torch
    B, H, S_q, D = q.shape
    S_kv = k.shape[2]
    nan = float("nan")
    dq = torch.full(q.shape, nan, dtype=q.dtype, device=q.device)
    dk = torch.full(k.shape, nan, dtype=q.dtype, device=q.device)
    dv = torch.full(k.shape, nan, dtype=q.dtype, device=q.device)
    ws = torch.empty((2, B, H, S_q), dtype=torch.float32, device=q.device)
    rc = lib().attn_bwd_plain(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), d_o.data_ptr(), lse.data_ptr(),
                              dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), ws.data_ptr(), B, H, S_q, S_kv, D,
                              int(bool(causal)), float(scale), torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("attn_bwd_plain: status %d" % rc)
    return dq, dk, dv
