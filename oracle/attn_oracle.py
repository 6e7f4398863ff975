"""ctypes front end of the fp64 C oracle (oracle/attn_ref.c).

TEST INFRASTRUCTURE ONLY.  The oracle is the plain softmax-attention
definition behind the paper's Section 3 running example (Fig. 1a) with the
softmax bookkeeping that Section 6.2 mentions written out in full; see the
header of attn_ref.c for the formulas.  Nothing here imports, or is imported
by, the HIP package.

Inputs are numpy uint16 arrays holding bf16 (default) or IEEE binary16
bit patterns, shaped [B, H, S, D]; outputs are numpy float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "attn_ref.c"), os.path.join(_HERE, "attn_bwd_ref.c")]
_LIB = os.path.join(_HERE, "libattn_ref.so")
_lib = None


def build(force=False):
    """Compile attn_ref.c and attn_bwd_ref.c with gcc (-O2, OpenMP).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-o", tmp] + _SRCS + ["-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        for fn in (lib.attn_ref_f64, lib.attn_ref_f64_f16):
            fn.restype = ctypes.c_int
            fn.argtypes = [
                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                ctypes.c_int, ctypes.c_float,
                ctypes.c_int64, ctypes.c_void_p,
                ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.attn_bwd_ref_f64.restype = ctypes.c_int
        lib.attn_bwd_ref_f64.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_float, ctypes.c_int,
            ctypes.c_int64, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.attn_ref_max_threads.restype = ctypes.c_int
        lib.attn_ref_max_threads.argtypes = []
        _lib = lib
    return _lib


def max_threads():
    return int(_load().attn_ref_max_threads())


def attn_ref(q, k, v, causal, scale, rows=None, n_threads=0, dtype="bf16"):
    """Oracle attention.

    q: uint16 [B,H,S_q,D]; k, v: uint16 [B,H,S_kv,D]: bit patterns of `dtype`,
    "bf16" or "f16" (IEEE binary16).
    scale: rounded to fp32 first (the value the GPU entry point receives).
    rows: None -> every row, returns O [B,H,S_q,D], LSE [B,H,S_q];
          else a 1-D int64 array of flat row ids (b*H + h)*S_q + i,
          returns O [n,D], LSE [n].
    """
    lib = _load()
    q = np.ascontiguousarray(q)
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    for a in (q, k, v):
        if a.dtype != np.uint16 or a.ndim != 4:
            raise TypeError("q, k, v must be uint16 [B,H,S,D] arrays of 16-bit patterns")
    B, H, S_q, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[1] != H or k.shape[3] != D:
        raise ValueError("shape mismatch between q, k, v")
    S_kv = k.shape[2]
    if rows is None:
        n = B * H * S_q
        rows_p = None
        o = np.empty((B, H, S_q, D), dtype=np.float64)
        lse = np.empty((B, H, S_q), dtype=np.float64)
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n = rows.shape[0]
        rows_p = rows.ctypes.data
        o = np.empty((n, D), dtype=np.float64)
        lse = np.empty((n,), dtype=np.float64)
    if dtype not in ("bf16", "f16"):
        raise ValueError("dtype must be 'bf16' or 'f16'")
    fn = lib.attn_ref_f64 if dtype == "bf16" else lib.attn_ref_f64_f16
    rc = fn(q.ctypes.data, k.ctypes.data, v.ctypes.data,
            B, H, S_q, S_kv, D, int(bool(causal)),
            float(np.float32(scale)), n, rows_p,
            o.ctypes.data, lse.ctypes.data, int(n_threads))
    if rc != 0:
        raise RuntimeError("attn_ref_f64 failed (bad argument or out of memory)")
    return o, lse


def attn_bwd_ref(q, k, v, d_o, causal, scale, heads=None, n_threads=0, dtype="bf16"):
    """Oracle gradients of attention (attn_bwd_ref.c): (dq, dk, dv) in fp64.

    q, d_o: uint16 [B,H,S_q,D]; k, v: uint16 [B,H,S_kv,D]: bit patterns of `dtype`.
    d_o is the gradient of the loss with respect to the attention output.
    heads: None -> every head, returns dq [B,H,S_q,D], dk, dv [B,H,S_kv,D];
           else a 1-D int64 array of flat head ids b*H + h, returns [n,S,D] arrays.
    """
    lib = _load()
    q, k, v, d_o = (np.ascontiguousarray(a) for a in (q, k, v, d_o))
    for a in (q, k, v, d_o):
        if a.dtype != np.uint16 or a.ndim != 4:
            raise TypeError("q, k, v, d_o must be uint16 [B,H,S,D] arrays of 16-bit patterns")
    B, H, S_q, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[1] != H or k.shape[3] != D or d_o.shape != q.shape:
        raise ValueError("shape mismatch between q, k, v, d_o")
    if dtype not in ("bf16", "f16"):
        raise ValueError("dtype must be 'bf16' or 'f16'")
    S_kv = k.shape[2]
    if heads is None:
        n, heads_p = B * H, None
        lead = (B, H)
    else:
        heads = np.ascontiguousarray(heads, dtype=np.int64)
        n, heads_p = heads.shape[0], heads.ctypes.data
        lead = (n,)
    dq = np.empty(lead + (S_q, D), dtype=np.float64)
    dk = np.empty(lead + (S_kv, D), dtype=np.float64)
    dv = np.empty(lead + (S_kv, D), dtype=np.float64)
    rc = lib.attn_bwd_ref_f64(q.ctypes.data, k.ctypes.data, v.ctypes.data, d_o.ctypes.data,
                              B, H, S_q, S_kv, D, int(bool(causal)), float(np.float32(scale)),
                              int(dtype == "f16"), n, heads_p,
                              dq.ctypes.data, dk.ctypes.data, dv.ctypes.data, int(n_threads))
    if rc != 0:
        raise RuntimeError("attn_bwd_ref_f64 failed (bad argument or out of memory)")
    return dq, dk, dv
