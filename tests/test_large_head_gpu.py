"""A head whose K (and V) tensor is larger than 2 GiB: the shape class the pipelined kernels do not
take (they address one head's keys with 32-bit byte offsets), so attn_fwd must route it to the
generic kernel, whose offsets are 64-bit.  Checked element by element against the oracle.

The keys are a seeded block of 65537 rows repeated cyclically (the period does not divide 2^23
rows, so an address that wrapped at 2^31 or 2^32 bytes would land on different data), and the
keys past the 2 GiB mark are planted so that each query row's softmax concentrates on one of them:
reading those rows from a wrapped address changes O by O(1), far above the tolerance.
"""
import numpy as np
import pytest
import torch

from oracle.attn_oracle import attn_ref
from paper_2512_18134_amd import synth

pytestmark = pytest.mark.gpu

O_TOL = 2e-2
LSE_TOL = 1e-3


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def f32_to_bf16_bits(x):
    # round to nearest even, finite inputs only
    w = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((w + 0x7FFF + ((w >> 16) & 1)) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (b.astype(np.uint32) << 16).view(np.float32)


def test_head_larger_than_2gib_uses_64bit_addressing():
    from paper_2512_18134_amd import binding as B
    assert torch.cuda.is_available(), "this test needs the MI355X"
    D, S_q, period = 128, 70, 65537
    S_kv = (1 << 23) + S_q                      # K of one head: 2 GiB + 17.5 KiB
    print("large head: S_q=%d S_kv=%d D=%d" % (S_q, S_kv, D), flush=True)
    q, kb, vb = synth.make_qkv(1, 1, S_q, period, D, seed=77)
    k = np.resize(kb.reshape(period, D), (S_kv, D))
    v = np.resize(vb.reshape(period, D), (S_kv, D))
    # key 2^23 + i is 3 q_i: its score, 3 |q_i|^2 scale ~ 34, stands far above the ~ N(0,1) rest
    k[1 << 23:] = f32_to_bf16_bits(3.0 * bf16_bits_to_f32(q.reshape(S_q, D)))
    k = k.reshape(1, 1, S_kv, D)
    v = v.reshape(1, 1, S_kv, D)
    scale = synth.default_scale(D)

    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full(qd.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    B.attn_fwd(qd, kd, vd, o, lse, causal=False, scale=scale)
    torch.cuda.synchronize()
    og = o.float().cpu().numpy().astype(np.float64).reshape(S_q, D)
    lg = lse.cpu().numpy().astype(np.float64).reshape(S_q)
    del kd, vd
    print("large head: kernel done, oracle running", flush=True)

    # the oracle takes ~1 s per row at this length: sampled rows, both workgroup tiles and the ragged tail
    rows = np.array([0, 1, 17, 31, 32, 47, 62, 63, 64, 65, 68, 69], dtype=np.int64)
    orf, lrf = attn_ref(q, k, v, False, scale, rows=rows)
    eo, el = np.max(np.abs(og[rows] - orf)), np.max(np.abs(lg[rows] - lrf))
    print("large head: rows=%d max|dO|=%.3e max|dLSE|=%.3e" % (len(rows), eo, el), flush=True)
    assert eo <= O_TOL and el <= LSE_TOL
    # every row: the planted key dominates, so the output is the value row paired with it, to bf16 rounding
    vt = bf16_bits_to_f32(v.reshape(S_kv, D)[1 << 23:]).astype(np.float64)
    assert np.max(np.abs(orf - vt[rows])) < 1e-3
    assert np.max(np.abs(og - vt)) <= O_TOL
