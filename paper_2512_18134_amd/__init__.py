"""MI355X (gfx950) Flash-Attention forward: the loop of the paper's Section 3
running example (Fig. 1a / 1f), hand-written in HIP behind a C-ABI library.

`synth` (input generation) imports without the HIP library; everything that
computes lives in `binding`, which raises at import time if the library has
not been built (there is no CPU fallback).
"""
import importlib

__all__ = ["synth", "binding", "attn_fwd", "attn_fwd_f16", "attn_fwd_splitkv", "attn_fwd_splitkv_f16", "attn_fwd_splitkv_workspace_bytes", "attn_bwd", "attn_bwd_f16", "attn_strerror", "attn_version", "attn_workgroup_tile", "attn_workgroup_queue_entry"]


def __getattr__(name):
    if name in ("attn_fwd", "attn_fwd_f16", "attn_fwd_splitkv", "attn_fwd_splitkv_f16", "attn_fwd_splitkv_workspace_bytes", "attn_bwd", "attn_bwd_f16", "attn_strerror", "attn_version", "attn_workgroup_tile", "attn_workgroup_queue_entry"):
        return getattr(importlib.import_module(__name__ + ".binding"), name)
    raise AttributeError(name)
