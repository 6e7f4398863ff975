"""Seeded random shapes through every entry point of the C ABI, each checked against the fp64 oracle.

The hand-picked shapes of the other GPU tests cover the tile boundaries that were thought of; these
cover the ones that were not: 48 shapes with B in 1..3, H in 1..4, S_q and S_kv in 1..700
(a quarter of them forced to a multiple of 32 plus or minus one), D in {64, 128, 256}, causal or not,
and 12 with many heads (B in 1..8, H in 1..16) on sequences of at most 330, mostly causal.
Bars as in the per-entry tests.
"""
import numpy as np
import pytest
import torch

from oracle.attn_oracle import attn_bwd_ref, attn_ref
from paper_2512_18134_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2512_18134_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        def length():
            s = int(rng.integers(1, 701))
            if rng.random() < 0.25:
                s = max(1, 32 * int(rng.integers(1, 22)) + int(rng.integers(-1, 2)))
            return s
        out.append((int(rng.integers(1, 4)), int(rng.integers(1, 5)), length(), length(),
                    int(rng.choice([64, 128, 128, 256])), bool(rng.integers(0, 2)), 1000 + i))
    return out


def many_heads(n, seed):
    # B*H up to 128 on short sequences: every XCD owns several heads (the causal dispatch order
    # then works through them in groups; left-over heads are shared out tile by tile)
    rng = np.random.default_rng(seed)
    out = []
    for i, s in enumerate(shapes(n, seed)):
        out.append((int(rng.integers(1, 9)), int(rng.integers(1, 17)), min(s[2], 330), min(s[3], 330), s[4],
                    i % 4 != 3, 2000 + i))
    return out


SHAPES = shapes(48, seed=2024) + many_heads(12, seed=2025)


def dev(bits, dt):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(dt)


def host(t, dtype):
    if dtype == "f16":
        return t.cpu().numpy().astype(np.float64)
    return synth.bf16_bits_to_f32(t.cpu().view(torch.int16).numpy().view(np.uint16)).astype(np.float64)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "B%d_H%d_Sq%d_Skv%d_D%d_%s_seed%d" % (s[0], s[1], s[2], s[3], s[4], "causal" if s[5] else "full", s[6]))
def test_random_shape_all_entry_points(B, shape):
    b, h, sq, skv, d, causal, seed = shape
    print("fuzz", shape, flush=True)
    scale = synth.default_scale(d)
    for dtype in ("bf16", "f16"):
        dt = torch.bfloat16 if dtype == "bf16" else torch.float16
        fwd = B.attn_fwd if dtype == "bf16" else B.attn_fwd_f16
        q, k, v = synth.make_qkv(b, h, sq, skv, d, seed, dtype=dtype)
        qd, kd, vd = dev(q, dt), dev(k, dt), dev(v, dt)
        o, lse = fwd(qd, kd, vd, causal=causal, scale=scale)
        torch.cuda.synchronize()
        orf, lrf = attn_ref(q, k, v, causal, scale, dtype=dtype)
        o_tol = 2e-2 if dtype == "bf16" else 4e-3
        og, lg = host(o, dtype), lse.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
        assert np.max(np.abs(og - orf)) <= o_tol, ("fwd", dtype)
        assert np.max(np.abs(lg - lrf)) <= 1e-3, ("lse", dtype)
        # backward: D in {64, 128}
        if d <= 128:
            bwd = B.attn_bwd if dtype == "bf16" else B.attn_bwd_f16
            d_o = synth.make_do(b, h, sq, d, seed, dtype=dtype)
            grads = bwd(qd, kd, vd, o, dev(d_o, dt), lse, causal=causal, scale=scale)
            torch.cuda.synchronize()
            rel = 2e-2 if dtype == "bf16" else 2.5e-3
            for name, g, w in zip(("dq", "dk", "dv"), grads, attn_bwd_ref(q, k, v, d_o, causal, scale, dtype=dtype)):
                gh = host(g, dtype)
                assert np.all(np.isfinite(gh)), (name, dtype)
                assert np.max(np.abs(gh - w)) <= rel * np.max(np.abs(w)) + 2e-5, (name, dtype)
        # split-KV: not causal, D in {64, 128}
        if d <= 128:
            n_split = 1 + seed % 7
            split = B.attn_fwd_splitkv if dtype == "bf16" else B.attn_fwd_splitkv_f16
            o2, lse2 = split(qd, kd, vd, n_split, scale=scale)
            torch.cuda.synchronize()
            if causal:
                orf, lrf = attn_ref(q, k, v, False, scale, dtype=dtype)
            assert np.max(np.abs(host(o2, dtype) - orf)) <= o_tol, "splitkv"
            assert np.max(np.abs(lse2.cpu().numpy() - lrf)) <= 1e-3, "splitkv lse"
