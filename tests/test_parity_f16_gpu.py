"""Parity of attn_fwd_f16 (through the C ABI) against the fp64 oracle on IEEE fp16 tensors,
the element type of the paper's Section 6 evaluation.

Tolerances: fp16 carries 11 significand bits where bf16 carries 8, so both the rounding of P
before the second contraction and the rounding of O are 8x finer than on the bf16 path:
max |O_gpu - O_ref| <= 4e-3 (|O| < 8 here: half an ulp of fp16 is 2^-9 ~ 2e-3, plus the P
rounding), max |LSE_gpu - LSE_ref| <= 1e-3 (fp32 bookkeeping, identical to the bf16 path).
"""
import numpy as np
import pytest
import torch

from oracle.attn_oracle import attn_bwd_ref, attn_ref
from paper_2512_18134_amd import synth

pytestmark = pytest.mark.gpu

O_TOL = 4e-3
LSE_TOL = 1e-3


@pytest.fixture(scope="module")
def B():
    from paper_2512_18134_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.float16)


def run_gpu(B, q, k, v, causal, scale):
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full(qd.shape, float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full(qd.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    B.attn_fwd_f16(qd, kd, vd, o, lse, causal=causal, scale=scale)
    torch.cuda.synchronize()
    return o.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


SMALL = [
    (1, 1, 128, 128, 64, False),
    (1, 2, 1, 1, 64, False),
    (1, 1, 1, 300, 128, False),
    (2, 3, 257, 257, 64, True),
    (2, 2, 300, 431, 128, False),
    (1, 3, 515, 515, 128, True),
    (1, 2, 700, 100, 128, True),
    (1, 2, 100, 700, 128, True),
    (1, 1, 1023, 1025, 64, False),
    (3, 5, 64, 64, 128, True),
    (1, 2, 300, 431, 256, False),
    (2, 2, 515, 515, 256, True),
    (1, 1, 1, 300, 256, False),
    (1, 3, 129, 1000, 256, True),
]


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "B%d_H%d_Sq%d_Skv%d_D%d_%s" % (s[0], s[1], s[2], s[3], s[4], "causal" if s[5] else "full"))
def test_small_shapes_elementwise(B, shape):
    b, h, sq, skv, d, causal = shape
    print("f16 case", shape, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=300 + sq + d, dtype="f16")
    scale = synth.default_scale(d)
    og, lg = run_gpu(B, q, k, v, causal, scale)
    orf, lrf = attn_ref(q, k, v, causal, scale, dtype="f16")
    assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
    eo, el = np.max(np.abs(og - orf)), np.max(np.abs(lg - lrf))
    print("%s max|dO|=%.3e max|dLSE|=%.3e" % (shape, eo, el), flush=True)
    assert eo <= O_TOL and el <= LSE_TOL


@pytest.mark.parametrize("d", [64, 128, 256])
def test_sharp_softmax(B, d):
    # per-row offsets on Q and K: a few keys dominate every row and the running maximum moves often
    b, h, s = 1, 2, 777
    print("f16 sharp D", d, flush=True)
    q, k, v = synth.make_qkv(b, h, s, s, d, seed=41, sharp=True, dtype="f16")
    scale = synth.default_scale(d)
    for causal in (False, True):
        og, lg = run_gpu(B, q, k, v, causal, scale)
        orf, lrf = attn_ref(q, k, v, causal, scale, dtype="f16")
        assert np.max(np.abs(og - orf)) <= O_TOL and np.max(np.abs(lg - lrf)) <= LSE_TOL


def test_values_that_bf16_cannot_hold_pass_through(B):
    # one key: O must reproduce V bit for bit, including significands with 10 fraction bits
    d = 128
    v = (np.arange(d, dtype=np.uint16) * 7 + 0x3C01).reshape(1, 1, 1, d)   # 1 + odd multiples of 2^-10 ...
    q, k, _ = synth.make_qkv(1, 1, 5, 1, d, seed=3, dtype="f16")
    og, lg = run_gpu(B, q, k, v, False, 0.25)
    want = v.view(np.float16).astype(np.float64)
    assert np.array_equal(og, np.broadcast_to(want, og.shape))
    _, lrf = attn_ref(q, k, v, False, 0.25, dtype="f16")
    assert np.max(np.abs(lg - lrf)) <= LSE_TOL


def test_paper_shape_sampled_rows(B):
    # the paper's sweep shape (BATCH=4, NUM_HEADS=32, HEAD_DIM=128, non-causal) at seq 2048,
    # in the launch configuration the bench times; the oracle computes sampled rows one by one
    cfg = synth.paper_workload(2048, causal=False)
    print("f16", cfg["name"], flush=True)
    q, k, v = synth.make_qkv(cfg["B"], cfg["H"], cfg["S_q"], cfg["S_kv"], cfg["D"], cfg["seed"], dtype="f16")
    scale = synth.default_scale(cfg["D"])
    og, lg = run_gpu(B, q, k, v, False, scale)
    assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
    rng = np.random.default_rng(9)
    S = cfg["S_q"]
    rows = set(rng.integers(0, cfg["B"] * cfg["H"] * S, size=3000).tolist())
    for bh in (0, 31, 127):
        rows.update(bh * S + i for i in (0, 1, 255, 256, 257, S - 2, S - 1))
    rows = np.array(sorted(rows), dtype=np.int64)
    orf, lrf = attn_ref(q, k, v, False, scale, rows=rows, dtype="f16")
    eo = np.max(np.abs(og.reshape(-1, cfg["D"])[rows] - orf))
    el = np.max(np.abs(lg.reshape(-1)[rows] - lrf))
    print("%s rows=%d max|dO|=%.3e max|dLSE|=%.3e" % (cfg["name"], len(rows), eo, el), flush=True)
    assert eo <= O_TOL and el <= LSE_TOL
    vf = v.view(np.float16).astype(np.float64)
    assert np.all(og >= vf.min(axis=2, keepdims=True) - 2.0 ** -9)
    assert np.all(og <= vf.max(axis=2, keepdims=True) + 2.0 ** -9)


def test_f16_rejects_what_it_does_not_cover(B):
    q = torch.zeros((1, 1, 8, 96), dtype=torch.float16, device="cuda")
    with pytest.raises(B.AttnError) as e:
        B.attn_fwd_f16(q, q, q)
    assert e.value.status == B.ATTN_ERR_UNSUPPORTED_D
    q = torch.zeros((1, 1, 8, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(B.AttnError) as e:
        B.attn_fwd_f16(q, q, q, scale=0.0)
    assert e.value.status == B.ATTN_ERR_SCALE
    with pytest.raises(TypeError):
        B.attn_fwd(q, q, q)            # the bf16 entry does not take fp16 tensors


# ------------------------------------------------------------------ backward (attn_bwd_f16)
BWD_TOL = 2.5e-3   # the bf16 bar (2e-2 of the tensor's largest element, + 2e-5) / 8: three more significand bits
BWD_FLOOR = 2e-5


def run_bwd(B, q, k, v, d_o, causal, scale):
    qd, kd, vd, dod = to_dev(q), to_dev(k), to_dev(v), to_dev(d_o)
    o, lse = B.attn_fwd_f16(qd, kd, vd, causal=causal, scale=scale)
    nan = float("nan")
    dq = torch.full(qd.shape, nan, dtype=torch.float16, device="cuda")
    dk = torch.full(kd.shape, nan, dtype=torch.float16, device="cuda")
    dv = torch.full(kd.shape, nan, dtype=torch.float16, device="cuda")
    B.attn_bwd_f16(qd, kd, vd, o, dod, lse, dq, dk, dv, causal=causal, scale=scale)
    torch.cuda.synchronize()
    return [t.cpu().numpy().astype(np.float64) for t in (dq, dk, dv)]


BWD_SMALL = [
    (1, 1, 128, 128, 64, False),
    (2, 3, 257, 257, 64, True),
    (1, 1, 1023, 1025, 64, False),
    (1, 2, 700, 100, 64, True),
    (1, 1, 1, 300, 128, False),
    (2, 2, 300, 431, 128, False),
    (1, 3, 515, 515, 128, True),
    (1, 2, 700, 100, 128, True),
    (1, 2, 100, 700, 128, True),
    (3, 5, 64, 64, 128, True),
]


@pytest.mark.parametrize("shape", BWD_SMALL, ids=lambda s: "bwd_B%d_H%d_Sq%d_Skv%d_D%d_%s" % (s[0], s[1], s[2], s[3], s[4], "causal" if s[5] else "full"))
def test_bwd_small_shapes_elementwise(B, shape):
    b, h, sq, skv, d, causal = shape
    print("f16 bwd case", shape, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=900 + sq, dtype="f16")
    d_o = synth.make_do(b, h, sq, d, seed=900 + sq, dtype="f16")
    scale = synth.default_scale(d)
    got = run_bwd(B, q, k, v, d_o, causal, scale)
    want = attn_bwd_ref(q, k, v, d_o, causal, scale, dtype="f16")
    for name, g, w in zip(("dq", "dk", "dv"), got, want):
        assert np.all(np.isfinite(g)), name
        err, bar = np.max(np.abs(g - w)), BWD_TOL * np.max(np.abs(w)) + BWD_FLOOR
        print("%s %s max error %.3e (bar %.3e)" % (shape, name, err, bar), flush=True)
        assert err <= bar, (name, err, bar)


def test_bwd_paper_shape_heads_in_full(B):
    # the shape of the paper's backward figures (BATCH=4, NUM_HEADS=32, HEAD_DIM=128, fp16, non-causal) at seq 2048
    cfg = synth.paper_workload(2048, causal=False)
    print("f16 bwd", cfg["name"], flush=True)
    q, k, v = synth.make_qkv(cfg["B"], cfg["H"], cfg["S_q"], cfg["S_kv"], cfg["D"], cfg["seed"], dtype="f16")
    d_o = synth.make_do(cfg["B"], cfg["H"], cfg["S_q"], cfg["D"], cfg["seed"], dtype="f16")
    scale = synth.default_scale(cfg["D"])
    got = run_bwd(B, q, k, v, d_o, False, scale)
    heads = np.array([5, 126], dtype=np.int64)
    want = attn_bwd_ref(q, k, v, d_o, False, scale, heads=heads, dtype="f16")
    for name, g, w in zip(("dq", "dk", "dv"), got, want):
        assert np.all(np.isfinite(g))
        sub = g.reshape((-1,) + g.shape[2:])[heads]
        err, bar = np.max(np.abs(sub - w)), BWD_TOL * np.max(np.abs(w)) + BWD_FLOOR
        print("%s %s max error %.3e (bar %.3e)" % (cfg["name"], name, err, bar), flush=True)
        assert err <= bar


def test_bwd_f16_rejects_what_it_does_not_cover(B):
    z = torch.zeros((1, 1, 8, 256), dtype=torch.float16, device="cuda")
    lse = torch.zeros((1, 1, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(B.AttnError) as e:
        B.attn_bwd_f16(z, z, z, z, z, lse)
    assert e.value.status == B.ATTN_ERR_UNSUPPORTED_D
    z = torch.zeros((1, 1, 8, 64), dtype=torch.float16, device="cuda")
    with pytest.raises(B.AttnError) as e:
        B.attn_bwd_f16(z, z, z, z, z, lse, scale=0.0)
    assert e.value.status == B.ATTN_ERR_SCALE


@pytest.mark.parametrize("shape", [(1, 3, 25600 + 9, 48, 128, True), (1, 2, 40000, 70, 64, False), (1, 1, 76800 + 3, 40, 256, False)],
                         ids=lambda s: "B%d_H%d_Sq%d_Skv%d_D%d_%s" % (s[0], s[1], s[2], s[3], s[4], "causal" if s[5] else "full"))
def test_more_tiles_than_cu_slots(B, shape):
    # more query tiles than the chip has CU slots: the persistent workgroups of the fp16 kernels walk their
    # queues through several passes, the last one short; few keys keep the oracle cheap
    b, h, sq, skv, d, causal = shape
    print("f16 case", shape, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=11 + d, dtype="f16")
    scale = synth.default_scale(d)
    og, lg = run_gpu(B, q, k, v, causal, scale)
    orf, lrf = attn_ref(q, k, v, causal, scale, dtype="f16")
    assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
    assert np.max(np.abs(og - orf)) <= O_TOL and np.max(np.abs(lg - lrf)) <= LSE_TOL
