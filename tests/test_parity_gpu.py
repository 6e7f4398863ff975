"""Parity of the HIP path (through the C ABI) against the fp64 oracle.

Tolerances: max |O_gpu - O_ref| <= 2e-2 (O is bf16),
max |LSE_gpu - LSE_ref| <= 1e-3 (fp32, natural log).
"""
import math

import numpy as np
import pytest
import torch

from oracle.attn_oracle import attn_ref
from paper_2512_18134_amd import synth

pytestmark = pytest.mark.gpu

O_TOL = 2e-2
LSE_TOL = 1e-3


@pytest.fixture(scope="module")
def B():
    from paper_2512_18134_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return binding


def to_dev(bits):
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def o_to_f64(o):
    return synth.bf16_bits_to_f32(o.cpu().view(torch.int16).numpy().view(np.uint16)).astype(np.float64)


def run_gpu(B, q, k, v, causal, scale):
    # poison the outputs so an unwritten element cannot pass by accident
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full(qd.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    B.attn_fwd(qd, kd, vd, o, lse, causal=causal, scale=scale)
    torch.cuda.synchronize()
    return o_to_f64(o), lse.cpu().numpy().astype(np.float64)


def check_full(B, q, k, v, causal, scale, tag=""):
    og, lg = run_gpu(B, q, k, v, causal, scale)
    orf, lrf = attn_ref(q, k, v, causal, scale)
    assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg)), tag
    eo = np.max(np.abs(og - orf))
    el = np.max(np.abs(lg - lrf))
    print("%s max|dO|=%.3e max|dLSE|=%.3e" % (tag, eo, el), flush=True)
    assert eo <= O_TOL, (tag, eo)
    assert el <= LSE_TOL, (tag, el)
    return og, lg


SMALL = [
    # B, H, S_q, S_kv, D, causal  -- several tiles, ragged tails, S_q != S_kv
    (1, 1, 128, 128, 64, False),
    (1, 2, 1, 1, 64, False),
    (1, 1, 1, 300, 128, False),
    (2, 3, 257, 257, 64, True),
    (2, 2, 300, 431, 128, False),
    (1, 3, 515, 515, 128, True),
    (1, 2, 700, 100, 128, True),
    (1, 2, 100, 700, 128, True),
    (1, 2, 333, 265, 256, False),
    (2, 1, 290, 290, 256, True),
    (1, 1, 1023, 1025, 64, False),
    (3, 5, 64, 64, 128, True),
    (1, 1, 31, 33, 256, True),
]


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "B%d_H%d_Sq%d_Skv%d_D%d_%s" % (s[0], s[1], s[2], s[3], s[4], "causal" if s[5] else "full"))
def test_small_shapes_elementwise(B, shape):
    b, h, sq, skv, d, causal = shape
    print("case", shape, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=100 + sq + d)
    check_full(B, q, k, v, causal, synth.default_scale(d), str(shape))


@pytest.mark.parametrize("index", [1, 2])
def test_baseline_configs_full(B, index):
    cfg, q, k, v, scale = synth.make_config(index)
    print("config", cfg["name"], flush=True)
    check_full(B, q, k, v, cfg["causal"], scale, cfg["name"])


def sample_rows(cfg, n_random, seed, tile=256):
    """Flat row ids: first/last tile rows, rows around tile boundaries, random rows."""
    Bb, H, S = cfg["B"], cfg["H"], cfg["S_q"]
    rng = np.random.default_rng(seed)
    per_head = set([0, 1, S - 1, S - 2])
    for t in range(tile, S, tile * max(1, S // tile // 8)):
        per_head.update([t - 1, t, t + 1])
    per_head.update(range(0, 40))
    per_head.update(range(S - 40, S))
    rows = []
    for bh in range(Bb * H):
        rows.extend(bh * S + i for i in sorted(per_head) if 0 <= i < S)
    rows.extend(rng.integers(0, Bb * H * S, size=n_random).tolist())
    return np.array(sorted(set(rows)), dtype=np.int64)


@pytest.mark.parametrize("index,n_random", [(3, 4096), (4, 4096), (5, 4096)])
def test_baseline_configs_sampled_rows(B, index, n_random):
    # full-size workloads in the launch configuration the bench times; the oracle computes a sample of
    # rows one by one: every (b, h): the first and last 40 rows and the rows around tile boundaries;
    # plus 4096 seeded-random rows over the whole workload
    cfg, q, k, v, scale = synth.make_config(index)
    print("config", cfg["name"], flush=True)
    og, lg = run_gpu(B, q, k, v, cfg["causal"], scale)
    assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
    rows = sample_rows(cfg, n_random, seed=index)
    orf, lrf = attn_ref(q, k, v, cfg["causal"], scale, rows=rows)
    eo = np.max(np.abs(og.reshape(-1, cfg["D"])[rows] - orf))
    el = np.max(np.abs(lg.reshape(-1)[rows] - lrf))
    print("%s rows=%d (%d seeded-random) max|dO|=%.3e max|dLSE|=%.3e" % (cfg["name"], len(rows), n_random, eo, el),
          flush=True)
    assert len(rows) >= n_random and eo <= O_TOL and el <= LSE_TOL
    # properties that hold for every row at any size
    vf = synth.bf16_bits_to_f32(v).astype(np.float64)
    if not cfg["causal"]:
        lo = vf.min(axis=2, keepdims=True) - 2.0 ** -6
        hi = vf.max(axis=2, keepdims=True) + 2.0 ** -6
        assert np.all(og >= lo) and np.all(og <= hi)
    else:
        assert np.array_equal(og[:, :, 0, :], vf[:, :, 0, :])  # row 0 sees only key 0


def test_config5_one_head_in_full(B):
    # the sharp-softmax workload (config 5) at full size: every row of one head against the oracle
    cfg, q, k, v, scale = synth.make_config(5)
    og, lg = run_gpu(B, q, k, v, cfg["causal"], scale)
    head = 5
    rows = np.arange(head * cfg["S_q"], (head + 1) * cfg["S_q"], dtype=np.int64)
    orf, lrf = attn_ref(q, k, v, cfg["causal"], scale, rows=rows)
    eo = np.max(np.abs(og.reshape(-1, cfg["D"])[rows] - orf))
    el = np.max(np.abs(lg.reshape(-1)[rows] - lrf))
    print("%s head %d in full (%d rows) max|dO|=%.3e max|dLSE|=%.3e" % (cfg["name"], head, len(rows), eo, el), flush=True)
    assert eo <= O_TOL and el <= LSE_TOL


@pytest.mark.parametrize("shape", [(1, 24, 8300, 128), (1, 40, 4000, 64), (1, 24, 4200, 256)],
                         ids=lambda s: "B%d_H%d_S%d_D%d" % s)
def test_causal_heads_dispatched_in_groups(B, shape):
    # Causal launches whose XCDs each own several heads and work through them in groups of heads
    # (the last group of every XCD one head short here): every row of every head must still be
    # written, once, by the right workgroup.  Sampled rows of all heads against the oracle.
    b, h, s, d = shape
    cfg = {"B": b, "H": h, "S_q": s, "S_kv": s, "D": d}
    print("grouped causal", shape, flush=True)
    q, k, v = synth.make_qkv(b, h, s, s, d, seed=60 + d)
    scale = synth.default_scale(d)
    og, lg = run_gpu(B, q, k, v, True, scale)
    assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
    rows = sample_rows(cfg, 1500, seed=d)
    orf, lrf = attn_ref(q, k, v, True, scale, rows=rows)
    eo = np.max(np.abs(og.reshape(-1, d)[rows] - orf))
    el = np.max(np.abs(lg.reshape(-1)[rows] - lrf))
    print("%s rows=%d max|dO|=%.3e max|dLSE|=%.3e" % (shape, len(rows), eo, el), flush=True)
    assert eo <= O_TOL and el <= LSE_TOL
    vf = synth.bf16_bits_to_f32(v).astype(np.float64)
    assert np.array_equal(og[:, :, 0, :], vf[:, :, 0, :])


# ------------------------------------------------------ closed forms on the GPU
def bf16(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


@pytest.mark.parametrize("causal", [False, True])
def test_identical_keys_mean_of_values(B, causal):
    b, h, s, d = 1, 2, 400, 128
    q, _, v = synth.make_qkv(b, h, s, s, d, seed=7)
    krow = bf16(np.linspace(-1, 1, d))
    k = np.broadcast_to(krow, (b, h, s, d)).copy()
    og, lg = run_gpu(B, q, k, v, causal, 0.25)
    vf = synth.bf16_bits_to_f32(v).astype(np.float64)
    n = np.arange(1, s + 1, dtype=np.float64) if causal else np.full(s, float(s))
    mean = np.cumsum(vf, axis=2) / n[None, None, :, None] if causal else np.broadcast_to(vf.mean(2, keepdims=True), vf.shape)
    sc = 0.25 * (synth.bf16_bits_to_f32(q).astype(np.float64) @ synth.bf16_bits_to_f32(krow).astype(np.float64))
    assert np.max(np.abs(og - mean)) <= O_TOL
    assert np.max(np.abs(lg - (sc + np.log(n)))) <= LSE_TOL


def test_causal_row0_is_v0_exactly(B):
    q, k, v = synth.make_qkv(2, 2, 300, 300, 64, seed=8)
    og, lg = run_gpu(B, q, k, v, True, synth.default_scale(64))
    assert np.array_equal(og[:, :, 0], synth.bf16_bits_to_f32(v).astype(np.float64)[:, :, 0])


def test_one_hot_scores_select_value_row(B):
    s, d = 192, 256
    rng = np.random.default_rng(3)
    a = rng.integers(0, s, size=s)
    q = np.zeros((1, 1, s, d), np.float32)
    k = np.zeros((1, 1, s, d), np.float32)
    for i in range(s):
        q[0, 0, i, a[i]] = 64.0
        k[0, 0, i, i] = 1.0
    _, _, v = synth.make_qkv(1, 1, s, s, d, seed=9)
    og, lg = run_gpu(B, bf16(q), bf16(k), v, False, 1.0)
    want = synth.bf16_bits_to_f32(v).astype(np.float64)[0, 0, a]
    assert np.array_equal(og[0, 0], want)  # the selected row is exactly representable
    assert np.max(np.abs(lg - 64.0)) <= LSE_TOL


def test_scale_zero_is_uniform(B):
    q, k, v = synth.make_qkv(1, 2, 150, 200, 128, seed=10)
    og, lg = run_gpu(B, q, k, v, False, 0.0)
    mean = synth.bf16_bits_to_f32(v).astype(np.float64).mean(axis=2, keepdims=True)
    assert np.max(np.abs(og - mean)) <= O_TOL
    assert np.max(np.abs(lg - math.log(200))) <= LSE_TOL


def test_joint_permutation_invariance_and_determinism(B):
    q, k, v = synth.make_qkv(1, 2, 320, 384, 128, seed=11)
    scale = synth.default_scale(128)
    o1, l1 = run_gpu(B, q, k, v, False, scale)
    o1b, l1b = run_gpu(B, q, k, v, False, scale)
    assert np.array_equal(o1, o1b) and np.array_equal(l1, l1b)  # bitwise run-to-run
    perm = np.random.default_rng(2).permutation(384)
    o2, l2 = run_gpu(B, q, k[:, :, perm].copy(), v[:, :, perm].copy(), False, scale)
    assert np.max(np.abs(o1 - o2)) <= 2 * 2.0 ** -7  # two bf16 roundings apart at most (|O| < 1 here)
    assert np.max(np.abs(l1 - l2)) <= 1e-4


@pytest.mark.parametrize("D", [64, 128, 256])
def test_sharp_softmax_small(B, D):
    # the rescale path: scores of several hundred, near one-hot rows; a row maximum
    # that is wrong by even one key overflows exp2 here
    q, k, v = synth.make_qkv(1, 2, 513, 513, D, seed=12, sharp=True)
    for causal in (False, True):
        check_full(B, q, k, v, causal, synth.default_scale(D), "sharp D=%d causal=%s" % (D, causal))


@pytest.mark.parametrize("D", [64, 128])
def test_row_max_in_either_lane_half(B, D):
    # one key per 64-key tile carries a huge score; its position walks through all 64
    # slots of a tile, i.e. through both lane halves and every accumulator register
    s = 64 * 64
    q = np.zeros((1, 1, 64, D), np.float32)
    q[..., 0] = 16.0
    k = np.zeros((1, 1, s, D), np.float32)
    for t in range(64):
        k[0, 0, 64 * t + t, 0] = 4.0 + 0.25 * t      # scaled score 64..127, growing tile by tile
    _, _, v = synth.make_qkv(1, 1, 64, s, D, seed=15)
    check_full(B, bf16(q), bf16(k), v, False, 1.0, "max walks D=%d" % D)


def test_increasing_scores_force_rescale_every_tile(B):
    # keys sorted so that every later tile raises the row max: alpha < 1 each time
    s, d = 512, 128
    q = np.zeros((1, 1, s, d), np.float32)
    q[..., 0] = 1.0
    k = np.zeros((1, 1, s, d), np.float32)
    k[0, 0, :, 0] = np.arange(s) * 0.125
    _, _, v = synth.make_qkv(1, 1, s, s, d, seed=13)
    check_full(B, bf16(q), bf16(k), v, False, 1.0, "increasing scores")


def test_error_status_raises(B):
    q = torch.zeros((1, 1, 8, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.AttnError):
        B.attn_fwd(q, q, q)


def test_non_default_stream(B):
    q, k, v = synth.make_qkv(1, 2, 256, 256, 128, seed=14)
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    o0, l0 = B.attn_fwd(qd, kd, vd)
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        o1, l1 = B.attn_fwd(qd, kd, vd)
    st.synchronize()
    assert torch.equal(o0, o1) and torch.equal(l0, l1)


def test_pipelined_schedule_equals_program_order_kernel(B):
    # The software-pipelined loop must compute what the loop in program order computes (the paper's
    # Fig. 1f against Fig. 1a): the generic, non-pipelined kernel runs through the debug build's
    # attn_fwd_variant entry point on the same inputs.
    import debug_lib
    for D, causal in ((64, False), (128, True), (256, True)):
        q, k, v = synth.make_qkv(1, 2, 700, 700, D, seed=21)
        scale = synth.default_scale(D)
        og, lg = run_gpu(B, q, k, v, causal, scale)
        o_s, l_s = debug_lib.attn_fwd_variant(to_dev(q), to_dev(k), to_dev(v), causal, scale,
                                              debug_lib.FWD_PROGRAM_ORDER)
        torch.cuda.synchronize()
        # same arithmetic up to fp32 re-association and the lazily moved softmax reference: within bf16 rounding of O
        assert np.max(np.abs(og - o_to_f64(o_s))) <= 2.0 ** -6, D
        assert np.max(np.abs(lg - l_s.cpu().numpy().astype(np.float64))) <= 1e-4, D


def test_tiling_variants_agree_with_the_oracle(B):
    # every tiling the library holds for D = 64 and D = 128, each forced through the debug build (also on
    # shapes the dispatcher would give to another one)
    import debug_lib
    for D, causal, variant in ((64, True, debug_lib.FWD_D64_8_WAVES), (64, False, debug_lib.FWD_D64_4_WAVES),
                               (128, True, debug_lib.FWD_D128_ONE_WAVE_PER_SIMD),
                               (128, False, debug_lib.FWD_D128_ONE_WAVE_PER_SIMD),
                               (128, True, debug_lib.FWD_D128_TWO_WAVES_PER_SIMD),
                               (128, False, debug_lib.FWD_D128_TWO_WAVES_PER_SIMD)):
        q, k, v = synth.make_qkv(2, 2, 530, 610, D, seed=37)
        scale = synth.default_scale(D)
        o, lse = debug_lib.attn_fwd_variant(to_dev(q), to_dev(k), to_dev(v), causal, scale, variant)
        torch.cuda.synchronize()
        orf, lrf = attn_ref(q, k, v, causal, scale)
        assert np.max(np.abs(o_to_f64(o) - orf)) <= O_TOL, (D, causal, variant)
        assert np.max(np.abs(lse.cpu().numpy().astype(np.float64) - lrf)) <= LSE_TOL, (D, causal, variant)


MANY_TILES = [
    # more query tiles than the chip has CU slots, so that the persistent workgroups walk their queues through
    # several passes, the last one short; few keys keep the oracle cheap.  B, H, S_q, S_kv, D, causal
    (1, 3, 25600 + 17, 64, 128, False),    # 303 tiles of 256 rows: one full pass, a short second one
    (1, 5, 33000, 96, 128, True),          # 645 tiles: two full passes and a short third
    (2, 2, 40000, 70, 64, False),          # 628 tiles of 256 rows
    (1, 1, 76800 + 5, 40, 256, True),      # 601 tiles of 128 rows
    (1, 9, 7500, 150, 64, True),           # 4-wave D = 64 workgroups (two per CU): 531 tiles of 128 rows
]


@pytest.mark.parametrize("shape", MANY_TILES, ids=lambda s: "B%d_H%d_Sq%d_Skv%d_D%d_%s" % (s[0], s[1], s[2], s[3], s[4], "causal" if s[5] else "full"))
def test_more_tiles_than_cu_slots(B, shape):
    b, h, sq, skv, d, causal = shape
    print("case", shape, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=7 + d)
    og, lg = check_full(B, q, k, v, causal, synth.default_scale(d), str(shape))
    # a second launch on the same buffers gives the same bits (the walk is static)
    og2, lg2 = run_gpu(B, q, k, v, causal, synth.default_scale(d))
    assert np.array_equal(og, og2) and np.array_equal(lg, lg2)
