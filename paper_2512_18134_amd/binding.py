"""ctypes binding of libmi355attn.so: argument marshalling only.

Same names as include/attn_fwd.h.  There is no fallback: importing this module
raises if the library has not been built (python -m paper_2512_18134_amd.build).
PyTorch appears only as the owner of device memory and of the stream.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# ATTN_FWD_LIB (debug only) loads another build of the same library, e.g. a schedule experiment
LIB_PATH = os.environ.get("ATTN_FWD_LIB", os.path.join(_HERE, "libmi355attn.so"))

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libmi355attn.so is not built: run `python -m paper_2512_18134_amd.build` "
        "(there is no CPU or PyTorch fallback for attn_fwd)")

_lib = ctypes.CDLL(LIB_PATH)
_lib.attn_fwd.restype = ctypes.c_int
_lib.attn_fwd.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int] * 6 + [ctypes.c_float, ctypes.c_void_p]
_lib.attn_fwd_f16.restype = ctypes.c_int
_lib.attn_fwd_f16.argtypes = _lib.attn_fwd.argtypes
_lib.attn_fwd_splitkv.restype = ctypes.c_int
_lib.attn_fwd_splitkv.argtypes = ([ctypes.c_void_p] * 6 + [ctypes.c_longlong, ctypes.c_int] + [ctypes.c_int] * 6
                                  + [ctypes.c_float, ctypes.c_void_p])
_lib.attn_fwd_splitkv_f16.restype = ctypes.c_int
_lib.attn_fwd_splitkv_f16.argtypes = _lib.attn_fwd_splitkv.argtypes
_lib.attn_fwd_splitkv_workspace_bytes.restype = ctypes.c_longlong
_lib.attn_fwd_splitkv_workspace_bytes.argtypes = [ctypes.c_int] * 5
_lib.attn_bwd.restype = ctypes.c_int
_lib.attn_bwd.argtypes = [ctypes.c_void_p] * 10 + [ctypes.c_int] * 6 + [ctypes.c_float, ctypes.c_void_p]
_lib.attn_bwd_f16.restype = ctypes.c_int
_lib.attn_bwd_f16.argtypes = _lib.attn_bwd.argtypes
_lib.attn_bwd_noalloc.restype = ctypes.c_int
_lib.attn_bwd_noalloc.argtypes = [ctypes.c_void_p] * 9 + [ctypes.c_int] * 6 + [ctypes.c_float, ctypes.c_void_p]
_lib.attn_strerror.restype = ctypes.c_char_p
_lib.attn_strerror.argtypes = [ctypes.c_int]
_lib.attn_version.restype = ctypes.c_int
_lib.attn_version.argtypes = []
_lib.attn_workgroup_tile.restype = ctypes.c_int
_lib.attn_workgroup_tile.argtypes = [ctypes.c_int] * 4 + [ctypes.c_longlong] + [ctypes.POINTER(ctypes.c_int)] * 2

ATTN_OK = 0
ATTN_ERR_NULL = -1
ATTN_ERR_SHAPE = -2
ATTN_ERR_UNSUPPORTED_D = -3
ATTN_ERR_ALIGN = -4
ATTN_ERR_SCALE = -5
ATTN_ERR_LAUNCH = -6
ATTN_ERR_UNSUPPORTED = -7
ATTN_ERR_WORKSPACE = -8


class AttnError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__("attn_fwd: %s (status %d)" % (attn_strerror(status), status))


def attn_strerror(status):
    return _lib.attn_strerror(int(status)).decode()


def attn_version():
    return int(_lib.attn_version())


_lib.attn_workgroup_queue_entry.restype = ctypes.c_int
_lib.attn_workgroup_queue_entry.argtypes = [ctypes.c_int] * 4 + [ctypes.POINTER(ctypes.c_int)]


def attn_workgroup_queue_entry(workgroup, n_workgroups, n_entries, pass_):
    """Host-side view of the persistent forward launch: the queue entry workgroup `workgroup` takes up in pass
    `pass_`, or -1."""
    entry = ctypes.c_int(-2)
    rc = int(_lib.attn_workgroup_queue_entry(int(workgroup), int(n_workgroups), int(n_entries), int(pass_),
                                             ctypes.byref(entry)))
    if rc != ATTN_OK:
        raise AttnError(rc)
    return entry.value


def attn_workgroup_tile(causal, workgroup, n_heads, n_tiles, head_bytes=0):
    """attn_workgroup_tile (host-only diagnostic): the (head, tile) that workgroup id works on."""
    head, tile = ctypes.c_int(-1), ctypes.c_int(-1)
    rc = int(_lib.attn_workgroup_tile(int(bool(causal)), int(workgroup), int(n_heads), int(n_tiles), int(head_bytes),
                                      ctypes.byref(head), ctypes.byref(tile)))
    if rc != ATTN_OK:
        raise AttnError(rc)
    return head.value, tile.value


def attn_fwd_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S_q, S_kv, D, causal, scale, stream_ptr):
    """The C entry point with raw integer addresses; returns the attn_status."""
    return int(_lib.attn_fwd(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S_q, S_kv, D,
                             int(bool(causal)), float(scale), stream_ptr))


def attn_fwd_f16_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S_q, S_kv, D, causal, scale, stream_ptr):
    """attn_fwd_f16 with raw integer addresses; returns the attn_status."""
    return int(_lib.attn_fwd_f16(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, H, S_q, S_kv, D,
                                 int(bool(causal)), float(scale), stream_ptr))


def attn_fwd(q, k, v, o=None, lse=None, causal=False, scale=None, stream=None):
    """attn_fwd on torch device tensors.

    q [B,H,S_q,D], k/v [B,H,S_kv,D]: contiguous bf16 on the GPU.  o (bf16) and
    lse (fp32 [B,H,S_q]) are allocated when not given.  The launch goes to
    `stream` (default: torch's current stream) and is asynchronous.
    Returns (o, lse).
    """
    import torch
    return _marshal(attn_fwd_raw, torch.bfloat16, q, k, v, o, lse, causal, scale, stream)


def attn_fwd_f16(q, k, v, o=None, lse=None, causal=False, scale=None, stream=None):
    """attn_fwd_f16 on torch device tensors: as attn_fwd, with fp16 q, k, v, o (D = 64 or 128)."""
    import torch
    return _marshal(attn_fwd_f16_raw, torch.float16, q, k, v, o, lse, causal, scale, stream)


def _marshal(entry, dt, q, k, v, o, lse, causal, scale, stream):
    import torch

    for t in (q, k, v):
        if t.dtype != dt or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise TypeError("q, k, v must be contiguous 4-D %s tensors on the GPU" % dt)
    B, H, S_q, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[1] != H or k.shape[3] != D:
        raise ValueError("q, k, v shapes do not agree")
    S_kv = k.shape[2]
    if o is None:
        o = torch.empty_like(q)
    if lse is None:
        lse = torch.empty((B, H, S_q), dtype=torch.float32, device=q.device)
    if o.dtype != dt or o.shape != q.shape or not o.is_contiguous() or not o.is_cuda:
        raise TypeError("o must be a contiguous GPU tensor shaped and typed like q")
    if lse.dtype != torch.float32 or tuple(lse.shape) != (B, H, S_q) or not lse.is_contiguous() or not lse.is_cuda:
        raise TypeError("lse must be a contiguous fp32 GPU tensor [B,H,S_q]")
    if scale is None:
        scale = 1.0 / float(D) ** 0.5
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    with torch.cuda.device(q.device):
        rc = entry(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                   B, H, S_q, S_kv, D, causal, scale, stream.cuda_stream)
    if rc != ATTN_OK:
        raise AttnError(rc)
    return o, lse


def attn_bwd_raw(q_ptr, k_ptr, v_ptr, o_ptr, do_ptr, lse_ptr, dq_ptr, dk_ptr, dv_ptr, ws_ptr,
                 B, H, S_q, S_kv, D, causal, scale, stream_ptr):
    """The C entry point attn_bwd with raw integer addresses; returns the attn_status."""
    return int(_lib.attn_bwd(q_ptr, k_ptr, v_ptr, o_ptr, do_ptr, lse_ptr, dq_ptr, dk_ptr, dv_ptr, ws_ptr,
                             B, H, S_q, S_kv, D, int(bool(causal)), float(scale), stream_ptr))


def attn_bwd_f16_raw(q_ptr, k_ptr, v_ptr, o_ptr, do_ptr, lse_ptr, dq_ptr, dk_ptr, dv_ptr, ws_ptr,
                     B, H, S_q, S_kv, D, causal, scale, stream_ptr):
    """The C entry point attn_bwd_f16 with raw integer addresses; returns the attn_status."""
    return int(_lib.attn_bwd_f16(q_ptr, k_ptr, v_ptr, o_ptr, do_ptr, lse_ptr, dq_ptr, dk_ptr, dv_ptr, ws_ptr,
                                 B, H, S_q, S_kv, D, int(bool(causal)), float(scale), stream_ptr))


def attn_bwd_noalloc_raw(q_ptr, k_ptr, v_ptr, o_ptr, do_ptr, lse_ptr, dq_ptr, dk_ptr, dv_ptr,
                         B, H, S_q, S_kv, D, causal, scale, stream_ptr):
    """The C entry point attn_bwd_noalloc with raw integer addresses; returns the attn_status."""
    return int(_lib.attn_bwd_noalloc(q_ptr, k_ptr, v_ptr, o_ptr, do_ptr, lse_ptr, dq_ptr, dk_ptr, dv_ptr,
                                     B, H, S_q, S_kv, D, int(bool(causal)), float(scale), stream_ptr))


def attn_bwd_noalloc(q, k, v, o, d_o, lse, dq, dk, dv, causal=False, scale=None, stream=None):
    """attn_bwd_noalloc on torch device tensors: attn_bwd with the library's own workspace.  The caller
    passes every output (this wrapper allocates nothing either).  Returns (dq, dk, dv)."""
    import torch
    entry = lambda *a: attn_bwd_noalloc_raw(*(a[:9] + a[10:]))   # drop the workspace address
    return _marshal_bwd(entry, torch.bfloat16, q, k, v, o, d_o, lse, dq, dk, dv, False, causal, scale, stream)


def attn_bwd_f16(q, k, v, o, d_o, lse, dq=None, dk=None, dv=None, delta_ws=None, causal=False, scale=None,
                 stream=None):
    """attn_bwd_f16 on torch device tensors: as attn_bwd, with fp16 tensors."""
    import torch
    return _marshal_bwd(attn_bwd_f16_raw, torch.float16, q, k, v, o, d_o, lse, dq, dk, dv, delta_ws, causal, scale,
                        stream)


def attn_bwd(q, k, v, o, d_o, lse, dq=None, dk=None, dv=None, delta_ws=None, causal=False, scale=None, stream=None):
    """attn_bwd on torch device tensors (include/attn_bwd.h).

    q, o, d_o [B,H,S_q,D], k, v [B,H,S_kv,D]: contiguous bf16 on the GPU; lse fp32 [B,H,S_q] as
    written by attn_fwd.  dq, dk, dv (bf16) and the fp32 workspace delta_ws (2*B*H*S_q floats) are
    allocated when not given.  Asynchronous on `stream`.  Returns (dq, dk, dv).
    """
    import torch
    return _marshal_bwd(attn_bwd_raw, torch.bfloat16, q, k, v, o, d_o, lse, dq, dk, dv, delta_ws, causal, scale, stream)


def _marshal_bwd(entry, dt, q, k, v, o, d_o, lse, dq, dk, dv, delta_ws, causal, scale, stream):
    import torch

    for t in (q, k, v, o, d_o):
        if t.dtype != dt or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise TypeError("q, k, v, o, d_o must be contiguous 4-D %s tensors on the GPU" % dt)
    B, H, S_q, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[1] != H or k.shape[3] != D:
        raise ValueError("q, k, v shapes do not agree")
    if o.shape != q.shape or d_o.shape != q.shape:
        raise ValueError("o and d_o must be shaped like q")
    S_kv = k.shape[2]
    if lse.dtype != torch.float32 or tuple(lse.shape) != (B, H, S_q) or not lse.is_contiguous() or not lse.is_cuda:
        raise TypeError("lse must be a contiguous fp32 GPU tensor [B,H,S_q]")
    no_ws = delta_ws is False          # attn_bwd_noalloc: the library's own workspace, outputs from the caller
    if no_ws and (dq is None or dk is None or dv is None):
        raise TypeError("attn_bwd_noalloc: the caller passes dq, dk, dv")
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    if delta_ws is None:
        delta_ws = torch.empty((2, B, H, S_q), dtype=torch.float32, device=q.device)
    for t, like in ((dq, q), (dk, k), (dv, v)):
        if t.dtype != dt or t.shape != like.shape or not t.is_contiguous() or not t.is_cuda:
            raise TypeError("dq, dk, dv must be contiguous GPU tensors shaped and typed like q, k, v")
    if not no_ws and (delta_ws.dtype != torch.float32 or delta_ws.numel() < 2 * B * H * S_q
                      or not delta_ws.is_contiguous() or not delta_ws.is_cuda):
        raise TypeError("delta_ws must be a contiguous fp32 GPU tensor with at least 2*B*H*S_q elements")
    if scale is None:
        scale = 1.0 / float(D) ** 0.5
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    with torch.cuda.device(q.device):
        rc = entry(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), d_o.data_ptr(), lse.data_ptr(),
                   dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), 0 if no_ws else delta_ws.data_ptr(),
                   B, H, S_q, S_kv, D, causal, scale, stream.cuda_stream)
    if rc != ATTN_OK:
        raise AttnError(rc)
    return dq, dk, dv


def attn_fwd_splitkv_workspace_bytes(B, H, S_q, D, n_split):
    return int(_lib.attn_fwd_splitkv_workspace_bytes(B, H, S_q, D, n_split))


def attn_fwd_splitkv_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, ws_ptr, ws_bytes, n_split,
                         B, H, S_q, S_kv, D, causal, scale, stream_ptr):
    """The C entry point attn_fwd_splitkv with raw integer addresses; returns the attn_status."""
    return int(_lib.attn_fwd_splitkv(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, ws_ptr, ws_bytes, n_split,
                                     B, H, S_q, S_kv, D, int(bool(causal)), float(scale), stream_ptr))


def attn_fwd_splitkv_f16_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, ws_ptr, ws_bytes, n_split,
                             B, H, S_q, S_kv, D, causal, scale, stream_ptr):
    """The C entry point attn_fwd_splitkv_f16 with raw integer addresses; returns the attn_status."""
    return int(_lib.attn_fwd_splitkv_f16(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, ws_ptr, ws_bytes, n_split,
                                         B, H, S_q, S_kv, D, int(bool(causal)), float(scale), stream_ptr))


def attn_fwd_splitkv(q, k, v, n_split, o=None, lse=None, workspace=None, causal=False, scale=None, stream=None):
    """attn_fwd_splitkv on torch device tensors (bf16).  `workspace`: a contiguous GPU tensor of at least
    attn_fwd_splitkv_workspace_bytes(...) bytes (allocated when not given).  Returns (o, lse)."""
    import torch
    return _marshal_splitkv(attn_fwd_splitkv_raw, torch.bfloat16, q, k, v, n_split, o, lse, workspace, causal, scale,
                            stream)


def attn_fwd_splitkv_f16(q, k, v, n_split, o=None, lse=None, workspace=None, causal=False, scale=None, stream=None):
    """attn_fwd_splitkv_f16 on torch device tensors: as attn_fwd_splitkv, with fp16 tensors."""
    import torch
    return _marshal_splitkv(attn_fwd_splitkv_f16_raw, torch.float16, q, k, v, n_split, o, lse, workspace, causal, scale,
                            stream)


def _marshal_splitkv(entry, dt, q, k, v, n_split, o, lse, workspace, causal, scale, stream):
    import torch

    for t in (q, k, v):
        if t.dtype != dt or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise TypeError("q, k, v must be contiguous 4-D %s tensors on the GPU" % dt)
    B, H, S_q, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[1] != H or k.shape[3] != D:
        raise ValueError("q, k, v shapes do not agree")
    S_kv = k.shape[2]
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty((B, H, S_q), dtype=torch.float32, device=q.device) if lse is None else lse
    if o.dtype != dt or o.shape != q.shape or not o.is_contiguous() or not o.is_cuda:
        raise TypeError("o must be a contiguous GPU tensor shaped and typed like q")
    if lse.dtype != torch.float32 or tuple(lse.shape) != (B, H, S_q) or not lse.is_contiguous() or not lse.is_cuda:
        raise TypeError("lse must be a contiguous fp32 GPU tensor [B,H,S_q]")
    need = attn_fwd_splitkv_workspace_bytes(B, H, S_q, D, n_split)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=q.device)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous GPU tensor")
    if scale is None:
        scale = 1.0 / float(D) ** 0.5
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    with torch.cuda.device(q.device):
        rc = entry(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                   workspace.data_ptr(), workspace.numel() * workspace.element_size(), n_split,
                   B, H, S_q, S_kv, D, causal, scale, stream.cuda_stream)
    if rc != ATTN_OK:
        raise AttnError(rc)
    return o, lse
