"""Pins for the fp64 oracle: closed forms, invariants, special cases that reduce
to library routines, and brute force on tiny inputs.  None of these re-types the
oracle's own two-pass formula; each would fail for a plausible oracle mistake
(dropped scale, wrong mask bound, transposed operand, missing max shift, wrong
log base, O normalised by the wrong sum ...).

The paper prints no worked numeric attention example (its Fig. 1a is a
simplified loop without numbers), so there is no golden file from the paper;
the small fixture under tests/golden/ is hand-derived and cited there.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle.attn_oracle import attn_ref
from paper_2512_18134_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bf16(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def f64(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def rand_qkv(seed, B, H, Sq, Skv, D):
    return synth.make_qkv(B, H, Sq, Skv, D, seed)


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("causal", [False, True])
def test_identical_keys_give_mean_of_values(causal):
    # all keys equal -> uniform weights: O = (prefix) mean of V, LSE = s + ln n_i
    B, H, S, D = 2, 3, 37, 16
    q, _, v = rand_qkv(11, B, H, S, S, D)
    krow = bf16(np.linspace(-1.0, 1.0, D))
    k = np.broadcast_to(krow, (B, H, S, D)).copy()
    scale = 0.37
    o, lse = attn_ref(q, k, v, causal, scale)
    vf, qf = f64(v), f64(q)
    s = float(np.float32(scale)) * (qf @ f64(krow))             # [B,H,S]
    if causal:
        n = np.arange(1, S + 1, dtype=np.float64)
        mean = np.cumsum(vf, axis=2) / n[None, None, :, None]
    else:
        n = np.full(S, float(S))
        mean = np.broadcast_to(vf.mean(axis=2, keepdims=True), vf.shape)
    assert np.max(np.abs(o - mean)) < 1e-12
    assert np.max(np.abs(lse - (s + np.log(n)))) < 1e-11


def test_causal_row0_is_v0():
    q, k, v = rand_qkv(12, 2, 2, 33, 33, 32)
    scale = synth.default_scale(32)
    o, lse = attn_ref(q, k, v, True, scale)
    assert np.array_equal(o[:, :, 0, :], f64(v)[:, :, 0, :])
    s00 = scale * np.einsum("bhd,bhd->bh", f64(q)[:, :, 0], f64(k)[:, :, 0])
    assert np.max(np.abs(lse[:, :, 0] - s00)) < 1e-12


def test_one_hot_scores_select_a_value_row():
    # q_i = beta * e_{a(i)}, k_j = e_{pi(j)}: s_ij = scale*beta*[pi(j) == a(i)]
    S, D = 16, 16
    rng = np.random.default_rng(5)
    pi = rng.permutation(D)[:S]           # distinct columns per key
    a = rng.integers(0, S, size=S)        # query i wants key a(i)
    beta, scale = 64.0, 1.0
    q = np.zeros((1, 1, S, D), np.float32)
    k = np.zeros((1, 1, S, D), np.float32)
    for i in range(S):
        q[0, 0, i, pi[a[i]]] = beta
    for j in range(S):
        k[0, 0, j, pi[j]] = 1.0
    _, _, v = rand_qkv(13, 1, 1, S, S, D)
    o, lse = attn_ref(bf16(q), bf16(k), v, False, scale)
    want = f64(v)[0, 0, a, :]
    # the other S-1 keys carry weight exp(-64) each
    assert np.max(np.abs(o[0, 0] - want)) < 1e-20 * 1e-5 + 16 * math.exp(-64.0) * 12
    assert np.max(np.abs(lse[0, 0] - (beta * scale + np.log1p((S - 1) * math.exp(-64.0))))) < 1e-12


def test_two_key_logistic():
    # D = 1, two keys: O = sigma(s0-s1) v0 + sigma(s1-s0) v1 ; LSE = logaddexp(s0, s1)
    q = bf16([[[[1.5]]]])
    k = bf16([[[[0.75], [-2.0]]]])
    v = bf16([[[[3.0], [-1.0]]]])
    scale = 0.5
    o, lse = attn_ref(q, k, v, False, scale)
    s0, s1 = 0.5 * 1.5 * 0.75, 0.5 * 1.5 * -2.0
    sig = 1.0 / (1.0 + math.exp(-(s0 - s1)))
    assert abs(o[0, 0, 0, 0] - (sig * 3.0 + (1 - sig) * -1.0)) < 1e-14
    assert abs(lse[0, 0, 0] - math.log(math.exp(s0) + math.exp(s1))) < 1e-14


def test_hand_derived_golden():
    # tests/golden/attn_2x3.txt: a 2-query, 3-key, D=2 case worked by hand
    # (scores are multiples of ln 2, so every weight is a power of two).
    rows = [l for l in open(os.path.join(GOLD, "attn_2x3.txt")) if l.strip() and not l.startswith("#")]
    vals = {r.split(":")[0].strip(): np.array([float(t) for t in r.split(":")[1].split()]) for r in rows}
    ln2 = math.log(2.0)
    q = bf16(vals["q"].reshape(1, 1, 2, 2))
    k = bf16(vals["k"].reshape(1, 1, 3, 2))
    v = bf16(vals["v"].reshape(1, 1, 3, 2))
    # the oracle receives scale rounded to fp32, so the expected values carry the same factor
    scale = float(np.float32(ln2))
    r = scale / ln2
    for causal, tag in ((False, "full"), (True, "causal")):
        o, lse = attn_ref(q, k, v, causal, scale)
        # expected values in the file are exact for scale == ln 2; allow the fp32 rounding of ln 2
        assert np.max(np.abs(o.reshape(-1) - vals["o_" + tag])) < 5e-7
        assert np.max(np.abs(lse.reshape(-1) - vals["lse_over_ln2_" + tag] * ln2)) < 5e-7 * max(1.0, r)


def test_scale_zero_is_uniform():
    q, k, v = rand_qkv(14, 1, 2, 19, 23, 8)
    o, lse = attn_ref(q, k, v, False, 0.0)
    assert np.max(np.abs(o - f64(v).mean(axis=2, keepdims=True))) < 1e-13
    assert np.max(np.abs(lse - math.log(23))) < 1e-13
    o, lse = attn_ref(q, k, v, True, 0.0)
    n = np.minimum(np.arange(1, 20), 23).astype(np.float64)
    assert np.max(np.abs(lse - np.log(n)[None, None, :])) < 1e-13


# ------------------------------------------------------------------ invariants
def test_joint_permutation_of_keys_and_values():
    q, k, v = rand_qkv(15, 2, 2, 24, 40, 16)
    perm = np.random.default_rng(1).permutation(40)
    scale = synth.default_scale(16)
    o1, l1 = attn_ref(q, k, v, False, scale)
    o2, l2 = attn_ref(q, k[:, :, perm], v[:, :, perm], False, scale)
    assert np.max(np.abs(o1 - o2)) < 1e-13
    assert np.max(np.abs(l1 - l2)) < 1e-13
    # permuting K alone must change the result (guards against V being ignored)
    o3, _ = attn_ref(q, k[:, :, perm], v, False, scale)
    assert np.max(np.abs(o1 - o3)) > 1e-3


def test_convex_combination_and_constant_values():
    q, k, v = rand_qkv(16, 1, 3, 31, 29, 8)
    scale = 0.9
    for causal in (False, True):
        o, _ = attn_ref(q, k, v, causal, scale)
        vf = f64(v)
        lo, hi = vf.min(axis=2, keepdims=True), vf.max(axis=2, keepdims=True)
        assert np.all(o >= lo - 1e-12) and np.all(o <= hi + 1e-12)
    vc = np.broadcast_to(bf16(np.arange(8) * 0.25 - 1.0), v.shape).copy()
    o, _ = attn_ref(q, k, vc, True, scale)
    assert np.max(np.abs(o - f64(vc)[:, :, :1, :])) < 1e-13


def test_causal_row_equals_truncated_full_attention():
    B, H, S, D = 1, 2, 21, 8
    q, k, v = rand_qkv(17, B, H, S, S, D)
    scale = synth.default_scale(D)
    oc, lc = attn_ref(q, k, v, True, scale)
    for i in (0, 1, 7, 20):
        of, lf = attn_ref(q[:, :, i:i + 1], k[:, :, :i + 1], v[:, :, :i + 1], False, scale)
        assert np.max(np.abs(oc[:, :, i] - of[:, :, 0])) < 1e-13
        assert np.max(np.abs(lc[:, :, i] - lf[:, :, 0])) < 1e-13
    # last causal row sees every key
    of, lf = attn_ref(q, k, v, False, scale)
    assert np.max(np.abs(oc[:, :, -1] - of[:, :, -1])) < 1e-13


def test_causal_is_top_left_aligned_when_lengths_differ():
    # S_q > S_kv: rows i >= S_kv see all keys; S_q < S_kv: row i sees keys 0..i only
    q, k, v = rand_qkv(18, 1, 1, 12, 5, 4)
    scale = 0.7
    oc, lc = attn_ref(q, k, v, True, scale)
    of, lf = attn_ref(q, k, v, False, scale)
    assert np.max(np.abs(oc[:, :, 4:] - of[:, :, 4:])) < 1e-13
    assert np.max(np.abs(oc[:, :, 0] - f64(v)[:, :, 0])) == 0.0
    q, k, v = rand_qkv(19, 1, 1, 5, 12, 4)
    oc, lc = attn_ref(q, k, v, True, scale)
    o5, l5 = attn_ref(q, k[:, :, :5], v[:, :, :5], True, scale)
    assert np.max(np.abs(oc - o5)) < 1e-13 and np.max(np.abs(lc - l5)) < 1e-13


def test_split_kv_merge():
    # attention over K = K1 || K2 equals the LSE-weighted merge of the halves
    q, k, v = rand_qkv(20, 1, 2, 9, 30, 8)
    scale = 1.1
    o, l = attn_ref(q, k, v, False, scale)
    o1, l1 = attn_ref(q, k[:, :, :13], v[:, :, :13], False, scale)
    o2, l2 = attn_ref(q, k[:, :, 13:], v[:, :, 13:], False, scale)
    lm = np.logaddexp(l1, l2)
    om = np.exp(l1 - lm)[..., None] * o1 + np.exp(l2 - lm)[..., None] * o2
    assert np.max(np.abs(l - lm)) < 1e-13
    assert np.max(np.abs(o - om)) < 1e-13


def test_value_scaling_is_linear_and_leaves_lse():
    # O is linear in V and LSE does not depend on V
    q, k, v = rand_qkv(21, 1, 1, 10, 17, 8)
    o1, l1 = attn_ref(q, k, v, False, 0.5)
    v2 = bf16(synth.bf16_bits_to_f32(v) * 2.0)
    o2, l2 = attn_ref(q, k, v2, False, 0.5)
    assert np.max(np.abs(o2 - 2 * o1)) < 1e-13 and np.array_equal(l1, l2)


# ------------------------------------------- library routines and brute force
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(2, 3, 40, 40, 64), (1, 2, 64, 200, 128), (1, 1, 130, 70, 256)])
def test_against_torch_cpu_fp64(shape, causal):
    B, H, Sq, Skv, D = shape
    q, k, v = rand_qkv(22 + D, B, H, Sq, Skv, D)
    scale = synth.default_scale(D)
    o, lse = attn_ref(q, k, v, causal, scale)
    qt, kt, vt = (torch.from_numpy(f64(x)) for x in (q, k, v))
    s = torch.matmul(qt, kt.transpose(-1, -2)) * scale
    if causal:
        keep = torch.arange(Skv)[None, :] <= torch.arange(Sq)[:, None]
        s = s.masked_fill(~keep, float("-inf"))
    want_o = torch.matmul(torch.softmax(s, dim=-1), vt).numpy()
    want_l = torch.logsumexp(s, dim=-1).numpy()
    assert np.max(np.abs(o - want_o)) < 1e-12
    assert np.max(np.abs(lse - want_l)) < 1e-12


# ------------------------------------------------------------ fp16 inputs (Section 6's element type)
def test_f16_decoding_of_every_finite_pattern():
    # one key: the softmax weight is 1, so O is the value row itself and LSE = scale * q.k;
    # numpy's float16 is the independent IEEE binary16 decoder (subnormals included)
    bits = np.arange(65536, dtype=np.uint16)
    bits = bits[np.isfinite(bits.view(np.float16))]
    n = bits.size
    assert n == 63488
    want = bits.view(np.float16).astype(np.float64)
    one = np.array([0x3C00], dtype=np.uint16)  # 1.0
    # V: [n heads][1 key][1]; Q = K = 1
    v = bits.reshape(1, n, 1, 1)
    qk = np.broadcast_to(one, (1, n, 1, 1)).copy()
    o, lse = attn_ref(qk, qk, v, False, 1.0, dtype="f16")
    assert np.array_equal(o.reshape(-1), want)   # (-0 compares equal to the accumulated +0)
    assert np.array_equal(lse.reshape(-1), np.ones(n))
    # Q, then K, run over every pattern against a unit partner: LSE = the decoded value
    for which in (0, 1):
        q = bits.reshape(1, n, 1, 1) if which == 0 else qk
        k = qk if which == 0 else bits.reshape(1, n, 1, 1)
        _, lse = attn_ref(q, k, qk, False, 1.0, dtype="f16")
        assert np.array_equal(lse.reshape(-1), want + 0.0)
    # the same bits read as bf16 give other numbers: the dtype switch is live
    _, lse_b = attn_ref(bits.reshape(1, n, 1, 1), qk, qk, False, 1.0, dtype="bf16")
    assert not np.array_equal(lse_b.reshape(-1), want)


def test_f16_two_key_logistic_with_a_value_bf16_cannot_hold():
    x = 1.0 + 2.0 ** -10          # exact in fp16, not in bf16
    f16 = lambda a: np.asarray(a, dtype=np.float16).view(np.uint16)
    q = f16([[[[x, 0.0]]]])
    k = f16([[[[1.0, 0.0], [0.0, 0.0]]]])
    v = f16([[[[1.0, 0.0], [0.0, 1.0]]]])
    o, lse = attn_ref(q, k, v, False, 1.0, dtype="f16")
    w = 1.0 / (1.0 + math.exp(-x))
    assert abs(o[0, 0, 0, 0] - w) < 1e-15 and abs(o[0, 0, 0, 1] - (1 - w)) < 1e-15
    assert abs(lse[0, 0, 0] - math.log(math.exp(x) + 1.0)) < 1e-15


@pytest.mark.parametrize("causal", [False, True])
def test_f16_against_torch_cpu_fp64(causal):
    B, H, Sq, Skv, D = 1, 2, 50, 90, 128
    q, k, v = synth.make_qkv(B, H, Sq, Skv, D, 77, dtype="f16")
    scale = synth.default_scale(D)
    o, lse = attn_ref(q, k, v, causal, scale, dtype="f16")
    qt, kt, vt = (torch.from_numpy(x.view(np.float16).astype(np.float64)) for x in (q, k, v))
    s = torch.matmul(qt, kt.transpose(-1, -2)) * scale
    if causal:
        keep = torch.arange(Skv)[None, :] <= torch.arange(Sq)[:, None]
        s = s.masked_fill(~keep, float("-inf"))
    assert np.max(np.abs(o - torch.matmul(torch.softmax(s, dim=-1), vt).numpy())) < 1e-12
    assert np.max(np.abs(lse - torch.logsumexp(s, dim=-1).numpy())) < 1e-12


def test_lse_brute_force_long_double():
    # small scores: log(sum(exp(s))) needs no max shift; do it in long double
    q, k, v = rand_qkv(30, 1, 1, 6, 11, 4)
    scale = 0.25
    _, lse = attn_ref(q, k, v, False, scale)
    qf, kf = f64(q)[0, 0], f64(k)[0, 0]
    for i in range(6):
        acc = np.longdouble(0)
        for j in range(11):
            dot = sum(np.longdouble(qf[i, d]) * np.longdouble(kf[j, d]) for d in range(4))
            acc += np.exp(np.longdouble(np.float32(scale)) * dot)
        assert abs(float(np.log(acc)) - lse[0, 0, i]) < 1e-14


def test_large_scores_do_not_overflow():
    # |s| ~ 1e3: exp(s) overflows fp64's naive form only past 709; the max shift must handle it
    q = bf16(np.full((1, 1, 2, 4), 16.0))
    k = bf16(np.array([[[[16.0] * 4, [15.0] * 4, [-16.0] * 4]]]))
    v = bf16(np.array([[[[1.0, 0, 0, 0], [0, 1.0, 0, 0], [0, 0, 1.0, 0]]]]))
    o, lse = attn_ref(q, k, v, False, 1.0)
    s = np.array([1024.0, 960.0, -1024.0])
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(lse))
    assert abs(lse[0, 0, 0] - (1024.0 + math.log1p(math.exp(-64.0)))) < 1e-12
    assert abs(o[0, 0, 0, 0] - 1.0 / (1.0 + math.exp(-64.0))) < 1e-15
    assert o[0, 0, 0, 2] < 1e-300 or o[0, 0, 0, 2] == 0.0


def test_row_subset_matches_full():
    q, k, v = rand_qkv(31, 2, 3, 17, 17, 8)
    o, lse = attn_ref(q, k, v, True, 0.6)
    rows = np.array([0, 5, 16, 17, 50, 2 * 3 * 17 - 1], dtype=np.int64)
    os_, ls_ = attn_ref(q, k, v, True, 0.6, rows=rows)
    assert np.array_equal(os_, o.reshape(-1, 8)[rows])
    assert np.array_equal(ls_, lse.reshape(-1)[rows])
    o1, _ = attn_ref(q, k, v, True, 0.6, n_threads=1)
    assert np.array_equal(o, o1)


def test_bad_arguments_raise():
    q, k, v = rand_qkv(32, 1, 1, 4, 4, 4)
    with pytest.raises(RuntimeError):
        attn_ref(q, k, v, False, 1.0, rows=np.array([4], dtype=np.int64))
    with pytest.raises(ValueError):
        attn_ref(q, k[:, :, :, :2], v, False, 1.0)
    with pytest.raises(TypeError):
        attn_ref(q.astype(np.float32), k, v, False, 1.0)
