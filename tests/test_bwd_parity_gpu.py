"""Parity of attn_bwd (through the C ABI) against the fp64 backward oracle.

The GPU backward consumes what the GPU forward wrote (o in bf16, lse in fp32); the oracle
differentiates the definition from q, k, v, d_o alone.

Tolerances.  Every gradient element is a sum of products whose factors p and ds were rounded
to bf16 (relative 2^-9) and whose result is rounded to bf16 once more; Delta is computed from
the bf16-rounded o.  With N(0,1) inputs the gradients have magnitude O(1) at most, and the
accumulated error is dominated by the final rounding, half an ulp of the largest element.
The bar used here: max |d - d_ref| <= 2e-2 * max |d_ref| + 2e-5 for each of dq, dk, dv: the forward bar of
2e-2 on O (whose elements are O(1)) made relative to the size of the tensor, since gradients range from 1e-2
(long sequences) to 50 (dV of a key every query attends to); the floor covers tensors that are exactly zero
(one visible key: Delta is computed from the bf16-rounded o, so dq and dk come out ~1e-6 instead of 0).
"""
import numpy as np
import pytest
import torch

from oracle.attn_oracle import attn_bwd_ref
from paper_2512_18134_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-2
ABS_FLOOR = 2e-5


@pytest.fixture(scope="module")
def B():
    from paper_2512_18134_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_f64(t):
    return synth.bf16_bits_to_f32(t.cpu().view(torch.int16).numpy().view(np.uint16)).astype(np.float64)


def run_gpu(B, q, k, v, d_o, causal, scale):
    qd, kd, vd, dod = to_dev(q), to_dev(k), to_dev(v), to_dev(d_o)
    o, lse = B.attn_fwd(qd, kd, vd, causal=causal, scale=scale)
    nan = float("nan")
    dq = torch.full(qd.shape, nan, dtype=torch.bfloat16, device="cuda")
    dk = torch.full(kd.shape, nan, dtype=torch.bfloat16, device="cuda")
    dv = torch.full(kd.shape, nan, dtype=torch.bfloat16, device="cuda")
    B.attn_bwd(qd, kd, vd, o, dod, lse, dq, dk, dv, causal=causal, scale=scale)
    torch.cuda.synchronize()
    return to_f64(dq), to_f64(dk), to_f64(dv)


def compare(got, want, tag):
    worst = 0.0
    for name, g, w in zip(("dq", "dk", "dv"), got, want):
        assert np.all(np.isfinite(g)), (tag, name)
        err = np.max(np.abs(g - w))
        bar = TOL * np.max(np.abs(w)) + ABS_FLOOR
        print("%s %s max|d|=%.3e (|ref|max=%.3f, bar %.3e)" % (tag, name, err, np.max(np.abs(w)), bar), flush=True)
        assert err <= bar, (tag, name, err, bar)
        worst = max(worst, err / bar)
    return worst


SMALL = [
    # B, H, S_q, S_kv, D, causal
    (1, 1, 128, 128, 64, False),
    (1, 2, 1, 1, 64, False),
    (1, 1, 1, 300, 128, False),
    (1, 1, 300, 1, 128, False),
    (2, 3, 257, 257, 64, True),
    (2, 2, 300, 431, 128, False),
    (1, 3, 515, 515, 128, True),
    (1, 2, 700, 100, 128, True),
    (1, 2, 100, 700, 128, True),
    (1, 1, 1023, 1025, 64, False),
    (3, 5, 64, 64, 128, True),
    (1, 8, 384, 384, 128, True),
]


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "B%d_H%d_Sq%d_Skv%d_D%d_%s" % (s[0], s[1], s[2], s[3], s[4], "causal" if s[5] else "full"))
def test_small_shapes_elementwise(B, shape):
    b, h, sq, skv, d, causal = shape
    print("bwd case", shape, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=500 + sq + d)
    d_o = synth.make_do(b, h, sq, d, seed=500 + sq + d)
    scale = synth.default_scale(d)
    got = run_gpu(B, q, k, v, d_o, causal, scale)
    want = attn_bwd_ref(q, k, v, d_o, causal, scale)
    compare(got, want, str(shape))


@pytest.mark.parametrize("shape", [(1, 3, 100, 128 * 101 + 5, 128, False), (1, 3, 128 * 90 + 3, 64, 128, True),
                                   (1, 5, 150, 128 * 120 + 77, 64, False), (2, 2, 128 * 150 + 1, 96, 64, True)],
                         ids=lambda s: "B%d_H%d_Sq%d_Skv%d_D%d_%s" % (s[0], s[1], s[2], s[3], s[4], "causal" if s[5] else "full"))
def test_more_owner_tiles_than_cu_slots(B, shape):
    # one of the two sweeps has more owner tiles than the chip has workgroup slots (and the other only a few):
    # its persistent workgroups walk their queues through several passes, the last one short
    b, h, sq, skv, d, causal = shape
    print("bwd case", shape, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=900 + d)
    d_o = synth.make_do(b, h, sq, d, seed=900 + d)
    scale = synth.default_scale(d)
    got = run_gpu(B, q, k, v, d_o, causal, scale)
    want = attn_bwd_ref(q, k, v, d_o, causal, scale)
    compare(got, want, str(shape))


@pytest.mark.parametrize("d", [64, 128])
def test_sharp_softmax(B, d):
    b, h, s = 1, 2, 600
    print("bwd sharp D", d, flush=True)
    q, k, v = synth.make_qkv(b, h, s, s, d, seed=43, sharp=True)
    d_o = synth.make_do(b, h, s, d, seed=43)
    scale = synth.default_scale(d)
    for causal in (False, True):
        compare(run_gpu(B, q, k, v, d_o, causal, scale), attn_bwd_ref(q, k, v, d_o, causal, scale), "sharp D%d" % d)


def test_invariants_and_invisible_keys(B):
    # causal with S_kv > S_q: keys no query sees get exact zeros; dK rows sum to ~0, dV rows to sum of dO
    b, h, sq, skv, d = 1, 2, 200, 333, 128
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=11)
    d_o = synth.make_do(b, h, sq, d, seed=11)
    dq, dk, dv = run_gpu(B, q, k, v, d_o, True, synth.default_scale(d))
    assert np.all(dk[:, :, sq:] == 0) and np.all(dv[:, :, sq:] == 0)
    assert np.max(np.abs(dq[:, :, 0])) < 1e-6  # row 0 sees one key: dp - Delta cancels up to the rounding of o
    do64 = synth.bf16_bits_to_f32(d_o).astype(np.float64)
    assert np.max(np.abs(dv.sum(axis=2) - do64.sum(axis=2))) < 0.5   # 200 bf16-rounded rows
    assert np.max(np.abs(dk.sum(axis=2))) < 0.2


def test_deterministic_and_stream(B):
    b, h, s, d = 2, 4, 512, 128
    q, k, v = synth.make_qkv(b, h, s, s, d, seed=12)
    d_o = synth.make_do(b, h, s, d, seed=12)
    qd, kd, vd, dod = to_dev(q), to_dev(k), to_dev(v), to_dev(d_o)
    o, lse = B.attn_fwd(qd, kd, vd, causal=True)
    a = B.attn_bwd(qd, kd, vd, o, dod, lse, causal=True)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        b2 = B.attn_bwd(qd, kd, vd, o, dod, lse, causal=True, stream=st)
    torch.cuda.synchronize()
    for x, y in zip(a, b2):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


def test_paper_shape_heads_in_full(B):
    # the paper's backward figure shape (BATCH=4, NUM_HEADS=32, HEAD_DIM=128, non-causal) at seq 2048,
    # in the launch configuration the bench times; the oracle computes three heads in full
    cfg = synth.paper_workload(2048, causal=False)
    print("bwd", cfg["name"], flush=True)
    q, k, v = synth.make_qkv(cfg["B"], cfg["H"], cfg["S_q"], cfg["S_kv"], cfg["D"], cfg["seed"])
    d_o = synth.make_do(cfg["B"], cfg["H"], cfg["S_q"], cfg["D"], cfg["seed"])
    scale = synth.default_scale(cfg["D"])
    got = run_gpu(B, q, k, v, d_o, False, scale)
    heads = np.array([0, 77, 127], dtype=np.int64)
    want = attn_bwd_ref(q, k, v, d_o, False, scale, heads=heads)
    sub = [g.reshape((-1,) + g.shape[2:])[heads] for g in got]
    compare(sub, want, cfg["name"])
    for g in got:
        assert np.all(np.isfinite(g))


def test_scale_zero_runs_the_compiler_scheduled_sweeps(B):
    # scale == 0: uniform softmax; the hand-scheduled loops need scale > 0, so this takes the other kernels
    b, h, sq, skv, d = 1, 2, 150, 210, 128
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=13)
    d_o = synth.make_do(b, h, sq, d, seed=13)
    for causal in (False, True):
        compare(run_gpu(B, q, k, v, d_o, causal, 0.0), attn_bwd_ref(q, k, v, d_o, causal, 0.0), "scale0")


def test_hand_scheduled_sweeps_equal_compiler_scheduled_sweeps(B):
    # the generated (hand-scheduled) sweeps against the same sweeps with instruction scheduling left to the
    # compiler, which run through the debug build's attn_bwd_plain entry point on the same inputs
    import debug_lib
    for D, causal in ((128, False), (128, True), (64, True)):
        q, k, v = synth.make_qkv(1, 2, 700, 650, D, seed=23)
        d_o = synth.make_do(1, 2, 700, D, seed=23)
        scale = synth.default_scale(D)
        got = run_gpu(B, q, k, v, d_o, causal, scale)
        qd, kd, vd, dod = to_dev(q), to_dev(k), to_dev(v), to_dev(d_o)
        o, lse = B.attn_fwd(qd, kd, vd, causal=causal, scale=scale)
        ref = debug_lib.attn_bwd_plain(qd, kd, vd, o, dod, lse, causal, scale)
        torch.cuda.synchronize()
        for n, gt, rt in zip(("dq", "dk", "dv"), got, ref):
            plain = to_f64(rt)
            # same arithmetic up to fp32 re-association: within bf16 rounding of the gradients
            assert np.max(np.abs(gt - plain)) <= 2.0 ** -6 * np.max(np.abs(plain)), (n, causal, D)


def test_headline_shape_one_head_in_full(B):
    # the forward headline workload's shape (B1 H16 S16384 D128, non-causal) in the launch configuration
    # `bench.py --config 4 --bwd` times; the oracle computes one head in full (all 16384 rows of dq, dk, dv)
    cfg, q, k, v, scale = synth.make_config(synth.HEADLINE_CONFIG)
    print("bwd", cfg["name"], flush=True)
    d_o = synth.make_do(cfg["B"], cfg["H"], cfg["S_q"], cfg["D"], cfg["seed"])
    got = run_gpu(B, q, k, v, d_o, cfg["causal"], scale)
    heads = np.array([11], dtype=np.int64)
    want = attn_bwd_ref(q, k, v, d_o, cfg["causal"], scale, heads=heads)
    sub = [g.reshape((-1,) + g.shape[2:])[heads] for g in got]
    compare(sub, want, cfg["name"])
    for g in got:
        assert np.all(np.isfinite(g))


def test_causal_heads_dispatched_in_groups(B):
    # a causal launch whose XCDs each own three heads and take them in groups (two heads, then one):
    # both sweeps must still cover every owner tile of every head; two heads against the oracle in full
    b, h, s, d = 1, 24, 4200, 128
    print("bwd grouped causal", (b, h, s, d), flush=True)
    q, k, v = synth.make_qkv(b, h, s, s, d, seed=71)
    d_o = synth.make_do(b, h, s, d, seed=71)
    scale = synth.default_scale(d)
    got = run_gpu(B, q, k, v, d_o, True, scale)
    for g in got:
        assert np.all(np.isfinite(g))
    heads = np.array([1, 23], dtype=np.int64)       # first group of XCD 0, short last group of XCD 7
    want = attn_bwd_ref(q, k, v, d_o, True, scale, heads=heads)
    compare([g.reshape((-1,) + g.shape[2:])[heads] for g in got], want, "grouped causal")


def test_rejected_arguments(B):
    z = torch.zeros((1, 1, 8, 256), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((1, 1, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(B.AttnError) as e:
        B.attn_bwd(z, z, z, z, z, lse)
    assert e.value.status == B.ATTN_ERR_UNSUPPORTED_D


def test_dq_atomics_probe_counts_the_key_tiles_each_query_meets():
    # the measurement kernel behind `bench.py --probe-dq-atomics` (debug build): after one launch every element
    # of dq holds the number of 128-key tiles its query row meets -- exact in fp32 -- and bad shapes are refused
    import ctypes
    import debug_lib
    lib = debug_lib.lib()
    lib.attn_probe_dq_atomics.restype = ctypes.c_int
    lib.attn_probe_dq_atomics.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 4 + [ctypes.c_void_p]
    st = torch.cuda.current_stream().cuda_stream
    heads, s_q, s_kv = 3, 320, 384
    for causal in (0, 1):
        dq = torch.zeros((heads, s_q, 128), dtype=torch.float32, device="cuda:0")
        assert lib.attn_probe_dq_atomics(dq.data_ptr(), heads, s_q, s_kv, causal, st) == 0
        torch.cuda.synchronize()
        rows = np.arange(s_q)
        want = np.minimum(rows // 128 + 1, s_kv // 128) if causal else np.full(s_q, s_kv // 128)
        assert np.array_equal(dq.cpu().numpy(), np.broadcast_to(want[None, :, None].astype(np.float32), (heads, s_q, 128)))
    dq = torch.zeros((1, 64, 128), dtype=torch.float32, device="cuda:0")
    for bad in ((1, 65, 128), (1, 64, 100), (0, 64, 128)):
        assert lib.attn_probe_dq_atomics(dq.data_ptr(), bad[0], bad[1], bad[2], 0, st) != 0
    assert lib.attn_probe_dq_atomics(None, 1, 64, 128, 0, st) != 0
