"""C-ABI checks that need no GPU: the library loads, exports every symbol that
include/attn_fwd.h declares, and validates arguments on the host before any
HIP call (so a validation error launches nothing)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")


@pytest.fixture(scope="module")
def binding():
    from paper_2512_18134_amd import binding as b
    return b


def declared_symbols():
    names = set()
    for fn in sorted(os.listdir(INCLUDE)):
        if fn.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(INCLUDE, fn)).read(), flags=re.S)
            names.update(re.findall(r"\b(attn_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported(binding):
    names = declared_symbols()
    assert {"attn_fwd", "attn_fwd_f16", "attn_fwd_splitkv", "attn_fwd_splitkv_f16", "attn_bwd", "attn_bwd_f16", "attn_strerror",
            "attn_version"} <= set(names)
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "symbol %s missing from libmi355attn.so" % n


def test_version_and_strerror(binding):
    assert binding.attn_version() >= 100
    for code in range(0, -9, -1):
        msg = binding.attn_strerror(code)
        assert isinstance(msg, str) and msg and "unknown" not in msg
    assert "unknown" in binding.attn_strerror(-99)


def test_validation_happens_before_any_launch(binding):
    b = binding
    ok = 0x1000  # aligned, non-NULL fake addresses: never dereferenced on a validation error
    f = lambda **kw: b.attn_fwd_raw(*[kw.get(n, d) for n, d in (
        ("q", ok), ("k", ok), ("v", ok), ("o", ok), ("lse", ok), ("B", 1), ("H", 1), ("S_q", 8), ("S_kv", 8),
        ("D", 64), ("causal", 0), ("scale", 0.125), ("stream", 0))])
    for name in ("q", "k", "v", "o", "lse"):
        assert f(**{name: 0}) == b.ATTN_ERR_NULL
    for name in ("B", "H", "S_q", "S_kv"):
        assert f(**{name: 0}) == b.ATTN_ERR_SHAPE
        assert f(**{name: -3}) == b.ATTN_ERR_SHAPE
    assert f(B=1 << 20, H=1 << 20) == b.ATTN_ERR_SHAPE
    for D in (0, 32, 96, 127, 512):
        assert f(D=D) == b.ATTN_ERR_UNSUPPORTED_D
    for name in ("q", "k", "v", "o"):
        assert f(**{name: ok + 8}) == b.ATTN_ERR_ALIGN
    assert f(lse=ok + 2) == b.ATTN_ERR_ALIGN
    for s in (float("nan"), float("inf"), -1.0):
        assert f(scale=s) == b.ATTN_ERR_SCALE


def test_f16_entry_validates_like_the_bf16_one_and_narrows_scale_and_size(binding):
    b = binding
    ok = 0x1000
    f = lambda **kw: b.attn_fwd_f16_raw(*[kw.get(n, d) for n, d in (
        ("q", ok), ("k", ok), ("v", ok), ("o", ok), ("lse", ok), ("B", 1), ("H", 1), ("S_q", 8), ("S_kv", 8),
        ("D", 64), ("causal", 0), ("scale", 0.125), ("stream", 0))])
    for name in ("q", "k", "v", "o", "lse"):
        assert f(**{name: 0}) == b.ATTN_ERR_NULL
    for name in ("B", "H", "S_q", "S_kv"):
        assert f(**{name: 0}) == b.ATTN_ERR_SHAPE
    for D in (0, 32, 96, 512):
        assert f(D=D) == b.ATTN_ERR_UNSUPPORTED_D
    assert f(q=ok + 8) == b.ATTN_ERR_ALIGN
    for s in (float("nan"), float("inf"), -1.0, 0.0):
        assert f(scale=s) == b.ATTN_ERR_SCALE
    assert f(S_kv=1 << 24, D=128) == b.ATTN_ERR_SHAPE  # one head of K beyond 32-bit byte offsets


@pytest.mark.parametrize("entry", ["attn_fwd_splitkv_raw", "attn_fwd_splitkv_f16_raw"])
def test_splitkv_entry_validates_before_any_launch(binding, entry):
    b = binding
    ok = 0x1000
    names = ("q", "k", "v", "o", "lse", "ws")
    def f(**kw):
        ptrs = [kw.get(n, ok) for n in names]
        ws_bytes = kw.get("ws_bytes", 1 << 40)
        rest = [kw.get(n, d) for n, d in (("n_split", 4), ("B", 1), ("H", 1), ("S_q", 8), ("S_kv", 8), ("D", 64),
                                           ("causal", 0), ("scale", 0.125), ("stream", 0))]
        return getattr(b, entry)(*(ptrs + [ws_bytes] + rest))
    for n in names:
        assert f(**{n: 0}) == b.ATTN_ERR_NULL
    for n in ("B", "H", "S_q", "S_kv"):
        assert f(**{n: 0}) == b.ATTN_ERR_SHAPE
    for ns in (0, -1, 257):
        assert f(n_split=ns) == b.ATTN_ERR_SHAPE
    for D in (0, 32, 256):
        assert f(D=D) == b.ATTN_ERR_UNSUPPORTED_D
    assert f(causal=1) == b.ATTN_ERR_UNSUPPORTED
    assert f(scale=0.0) == b.ATTN_ERR_SCALE
    assert f(ws=ok + 8) == b.ATTN_ERR_ALIGN
    need = b.attn_fwd_splitkv_workspace_bytes(1, 1, 8, 64, 4)
    assert need == 4 * 8 * 65 * 4
    assert f(ws_bytes=need - 1) == b.ATTN_ERR_WORKSPACE
    assert b.attn_fwd_splitkv_workspace_bytes(1, 1, 8, 256, 4) == -1
    assert b.attn_fwd_splitkv_workspace_bytes(1, 1, 8, 64, 0) == -1


def test_bwd_entry_validates_before_any_launch(binding):
    b = binding
    ok = 0x1000
    names = ("q", "k", "v", "o", "d_o", "lse", "dq", "dk", "dv", "ws")
    def f(**kw):
        ptrs = [kw.get(n, ok) for n in names]
        rest = [kw.get(n, d) for n, d in (("B", 1), ("H", 1), ("S_q", 8), ("S_kv", 8), ("D", 64), ("causal", 0),
                                           ("scale", 0.125), ("stream", 0))]
        return b.attn_bwd_raw(*(ptrs + rest))
    for n in names:
        assert f(**{n: 0}) == b.ATTN_ERR_NULL
    for n in ("B", "H", "S_q", "S_kv"):
        assert f(**{n: 0}) == b.ATTN_ERR_SHAPE
    for D in (0, 32, 96, 256):
        assert f(D=D) == b.ATTN_ERR_UNSUPPORTED_D
    for n in ("q", "k", "v", "o", "d_o", "dq", "dk", "dv"):
        assert f(**{n: ok + 8}) == b.ATTN_ERR_ALIGN
    assert f(lse=ok + 2) == b.ATTN_ERR_ALIGN and f(ws=ok + 2) == b.ATTN_ERR_ALIGN
    for s in (float("nan"), float("inf"), -1.0):
        assert f(scale=s) == b.ATTN_ERR_SCALE
    assert f(S_q=1 << 24, D=128) == b.ATTN_ERR_SHAPE
    # the entry point with the library's own workspace: same checks, and a limit on the rows
    def g(**kw):
        ptrs = [kw.get(n, ok) for n in names[:-1]]
        rest = [kw.get(n, d) for n, d in (("B", 1), ("H", 1), ("S_q", 8), ("S_kv", 8), ("D", 64), ("causal", 0),
                                           ("scale", 0.125), ("stream", 0))]
        return b.attn_bwd_noalloc_raw(*(ptrs + rest))
    assert g(q=0) == b.ATTN_ERR_NULL and g(B=0) == b.ATTN_ERR_SHAPE and g(dk=ok + 8) == b.ATTN_ERR_ALIGN
    assert g(D=256) == b.ATTN_ERR_UNSUPPORTED_D
    assert g(S_q=(1 << 21) + 1) == b.ATTN_ERR_WORKSPACE and g(B=2, H=1 << 10, S_q=1 << 10 | 1) == b.ATTN_ERR_WORKSPACE
    # the fp16 entry: same checks, and scale > 0 only
    def h(**kw):
        ptrs = [kw.get(n, ok) for n in names]
        rest = [kw.get(n, d) for n, d in (("B", 1), ("H", 1), ("S_q", 8), ("S_kv", 8), ("D", 128), ("causal", 0),
                                           ("scale", 0.125), ("stream", 0))]
        return b.attn_bwd_f16_raw(*(ptrs + rest))
    assert h(q=0) == b.ATTN_ERR_NULL and h(B=0) == b.ATTN_ERR_SHAPE and h(dq=ok + 8) == b.ATTN_ERR_ALIGN
    assert h(D=256) == b.ATTN_ERR_UNSUPPORTED_D and h(D=96) == b.ATTN_ERR_UNSUPPORTED_D
    assert h(scale=0.0) == b.ATTN_ERR_SCALE


def test_product_package_does_not_import_the_oracle():
    # the HIP path and the oracle share nothing and neither imports the other
    pkg = os.path.join(ROOT, "paper_2512_18134_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".hpp", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|attn_ref|attn_bwd_ref|libattn_ref", text, flags=re.M), fn
    for fn in os.listdir(os.path.join(ROOT, "oracle")):
        if fn.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", fn)).read()
            assert "paper_2512_18134_amd" not in text and "attn_fwd.h" not in text and "attn_bwd.h" not in text, fn
