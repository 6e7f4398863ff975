"""attn_bwd_noalloc (the entry point for callers that cannot allocate device memory) against attn_bwd:
same kernels, the library's own workspace instead of the caller's, so the results must agree bit for bit.
Two calls in a row on one stream, the second on a smaller input (the workspace keeps the first call's
contents), then the first shape again."""
import numpy as np
import pytest
import torch

from paper_2512_18134_amd import synth

pytestmark = pytest.mark.gpu


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def one_case(B, shape, causal, seed):
    b, h, sq, skv, d = shape
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=seed)
    d_o = synth.make_do(b, h, sq, d, seed=seed)
    scale = synth.default_scale(d)
    qd, kd, vd, dod = to_dev(q), to_dev(k), to_dev(v), to_dev(d_o)
    o, lse = B.attn_fwd(qd, kd, vd, causal=causal, scale=scale)
    want = B.attn_bwd(qd, kd, vd, o, dod, lse, causal=causal, scale=scale)
    nan = float("nan")
    got = [torch.full(t.shape, nan, dtype=torch.bfloat16, device="cuda") for t in (qd, kd, vd)]
    # through the C ABI with raw addresses: no wrapper logic between the test and the entry point
    rc = B.attn_bwd_noalloc_raw(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(), dod.data_ptr(),
                                lse.data_ptr(), got[0].data_ptr(), got[1].data_ptr(), got[2].data_ptr(),
                                b, h, sq, skv, d, causal, scale, torch.cuda.current_stream().cuda_stream)
    assert rc == B.ATTN_OK, B.attn_strerror(rc)
    torch.cuda.synchronize()
    for name, g, w in zip(("dq", "dk", "dv"), got, want):
        assert torch.equal(g.view(torch.int16), w.view(torch.int16)), (shape, causal, name)
        assert bool(torch.isfinite(g.float()).all()), (shape, causal, name)


def test_noalloc_backward_equals_backward_with_caller_workspace():
    from paper_2512_18134_amd import binding as B
    assert torch.cuda.is_available(), "these tests need the MI355X"
    big, small = (2, 3, 700, 650, 128), (1, 2, 130, 97, 128)
    one_case(B, big, True, 81)
    one_case(B, small, True, 82)       # smaller input right after: stale workspace contents beyond its rows
    one_case(B, big, False, 83)
    one_case(B, (1, 2, 333, 333, 64), False, 84)


def test_noalloc_backward_rejects_shapes_beyond_its_workspace():
    from paper_2512_18134_amd import binding as B
    ok = 0x1000   # aligned, non-NULL fake addresses: a rejected call launches nothing
    rc = B.attn_bwd_noalloc_raw(ok, ok, ok, ok, ok, ok, ok, ok, ok, 1, 1, (1 << 21) + 1, 8, 64, 0, 0.125, 0)
    assert rc == B.ATTN_ERR_WORKSPACE
    assert B.attn_bwd_noalloc_raw(0, ok, ok, ok, ok, ok, ok, ok, ok, 1, 1, 8, 8, 64, 0, 0.125, 0) == B.ATTN_ERR_NULL
