"""Pins for the backward oracle (oracle/attn_bwd_ref.c), all on the CPU.

The backward oracle is the chain rule written out; it is pinned to things it does not
compute itself: finite differences of the (separately pinned) forward oracle, torch's
autograd in fp64, closed forms and invariants of the softmax Jacobian.
"""
import math

import numpy as np
import pytest
import torch

from oracle.attn_oracle import attn_bwd_ref, attn_ref
from paper_2512_18134_amd import synth


def bf16(x):
    return synth.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def f16(x):
    return np.asarray(x, dtype=np.float16).view(np.uint16)


def widen(bits, dtype):
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def coarse(rng, shape):
    """multiples of 1/8 in [-1.5, 1.5]: x +- 2^-7 (bf16) and x +- 2^-9 (fp16) stay representable"""
    return rng.integers(-12, 13, size=shape).astype(np.float64) / 8.0


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype,h", [("bf16", 2.0 ** -7), ("f16", 2.0 ** -9)])
def test_central_differences_of_the_forward_oracle(dtype, h, causal):
    # L = sum(dO * O(q, k, v)); every coordinate of q, k, v is moved by +-h (exactly representable)
    rng = np.random.default_rng(5)
    pack = bf16 if dtype == "bf16" else f16
    B, H, Sq, Skv, D = 1, 2, 5, 6, 4
    scale = 0.5
    x = {"q": coarse(rng, (B, H, Sq, D)), "k": coarse(rng, (B, H, Skv, D)), "v": coarse(rng, (B, H, Skv, D))}
    d_o = coarse(rng, (B, H, Sq, D))

    def loss(vals):
        o, _ = attn_ref(pack(vals["q"]), pack(vals["k"]), pack(vals["v"]), causal, scale, dtype=dtype)
        return float(np.sum(o * d_o))

    for name in x:
        assert np.array_equal(widen(pack(x[name]), dtype), x[name])
    dq, dk, dv = attn_bwd_ref(pack(x["q"]), pack(x["k"]), pack(x["v"]), pack(d_o), causal, scale, dtype=dtype)
    got = {"q": dq, "k": dk, "v": dv}
    worst = 0.0
    for name in ("q", "k", "v"):
        for idx in np.ndindex(x[name].shape):
            up = {n: a.copy() for n, a in x.items()}
            dn = {n: a.copy() for n, a in x.items()}
            up[name][idx] += h
            dn[name][idx] -= h
            fd = (loss(up) - loss(dn)) / (2 * h)
            worst = max(worst, abs(fd - got[name][idx]))
    # truncation error of the central difference: h^2/6 * |third derivative| (O(1) here)
    assert worst < 40 * h * h, worst


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(2, 2, 33, 33, 64), (1, 2, 40, 70, 128), (1, 1, 70, 40, 128), (1, 1, 50, 50, 256)])
def test_against_torch_autograd_fp64(shape, causal):
    B, H, Sq, Skv, D = shape
    q, k, v = synth.make_qkv(B, H, Sq, Skv, D, 50 + D)
    d_o = synth.make_do(B, H, Sq, D, 50 + D)
    scale = synth.default_scale(D)
    dq, dk, dv = attn_bwd_ref(q, k, v, d_o, causal, scale)
    qt, kt, vt = (torch.from_numpy(widen(a, "bf16")).requires_grad_(True) for a in (q, k, v))
    s = torch.matmul(qt, kt.transpose(-1, -2)) * scale
    if causal:
        keep = torch.arange(Skv)[None, :] <= torch.arange(Sq)[:, None]
        s = s.masked_fill(~keep, float("-inf"))
    o = torch.matmul(torch.softmax(s, dim=-1), vt)
    o.backward(torch.from_numpy(widen(d_o, "bf16")))
    for got, want in ((dq, qt.grad), (dk, kt.grad), (dv, vt.grad)):
        assert np.max(np.abs(got - want.numpy())) < 1e-12


def test_f16_inputs_decode_like_numpy_float16():
    # one query, one key: dV = dO exactly, for every finite fp16 pattern of dO
    bits = np.arange(65536, dtype=np.uint16)
    bits = bits[np.isfinite(bits.view(np.float16))]
    n = bits.size
    one = np.full((1, n, 1, 1), 0x3C00, dtype=np.uint16)
    dq, dk, dv = attn_bwd_ref(one, one, one, bits.reshape(1, n, 1, 1), False, 1.0, dtype="f16")
    assert np.array_equal(dv.reshape(-1), bits.view(np.float16).astype(np.float64) + 0.0)
    assert np.all(dq == 0) and np.all(dk == 0)
    # q, k, v: values spread over normal and subnormal fp16 range, against autograd on numpy's decoding
    rng = np.random.default_rng(2)
    B, H, Sq, Skv, D = 1, 2, 12, 15, 8
    def draw(shape):
        x = rng.standard_normal(shape) * np.where(rng.random(shape) < 0.5, 1.0, 2.0 ** -15)
        return f16(x)
    q, k, v, d_o = draw((B, H, Sq, D)), draw((B, H, Skv, D)), draw((B, H, Skv, D)), draw((B, H, Sq, D))
    assert np.any((q & 0x7C00) == 0) and np.any((v & 0x7C00) == 0)      # subnormals are present
    dq, dk, dv = attn_bwd_ref(q, k, v, d_o, True, 1.0, dtype="f16")
    qt, kt, vt = (torch.from_numpy(widen(a, "f16")).requires_grad_(True) for a in (q, k, v))
    s = torch.matmul(qt, kt.transpose(-1, -2))
    keep = torch.arange(Skv)[None, :] <= torch.arange(Sq)[:, None]
    o = torch.matmul(torch.softmax(s.masked_fill(~keep, float("-inf")), dim=-1), vt)
    o.backward(torch.from_numpy(widen(d_o, "f16")))
    for got, want in ((dq, qt.grad), (dk, kt.grad), (dv, vt.grad)):
        w = want.numpy()
        assert np.max(np.abs(got - w)) <= 1e-13 * max(1.0, np.max(np.abs(w)))
        assert np.allclose(got, w, rtol=1e-9, atol=1e-30)               # tiny entries too


def test_one_key_passes_gradient_to_v_only():
    # a single visible key: p = 1 whatever q and k are, so dQ = dK = 0 and dV = sum of dO rows
    q, k, v = synth.make_qkv(1, 2, 9, 1, 8, 3)
    d_o = synth.make_do(1, 2, 9, 8, 3)
    dq, dk, dv = attn_bwd_ref(q, k, v, d_o, False, 0.7)
    assert np.all(dq == 0) and np.all(dk == 0)
    assert np.max(np.abs(dv[:, :, 0, :] - widen(d_o, "bf16").sum(axis=2))) < 1e-13


def test_two_key_logistic_closed_form():
    # q = (x), k = (1), (0): p0 = sigma(x); O = p0 v0 + (1 - p0) v1; with dO = 1:
    # dL/dx = sigma'(x) (v0 - v1), dV0 = p0, dV1 = 1 - p0, dK0 = sigma'(x) (v0 - v1) x = -dK1
    x, v0, v1 = 0.75, 1.5, -0.5
    q = bf16([[[[x]]]])
    k = bf16([[[[1.0], [0.0]]]])
    v = bf16([[[[v0], [v1]]]])
    d_o = bf16([[[[1.0]]]])
    dq, dk, dv = attn_bwd_ref(q, k, v, d_o, False, 1.0)
    sg = 1.0 / (1.0 + math.exp(-x))
    slope = sg * (1 - sg) * (v0 - v1)
    assert abs(dq[0, 0, 0, 0] - slope) < 1e-15
    assert abs(dk[0, 0, 0, 0] - slope * x) < 1e-15 and abs(dk[0, 0, 1, 0] + slope * x) < 1e-15
    assert abs(dv[0, 0, 0, 0] - sg) < 1e-15 and abs(dv[0, 0, 1, 0] - (1 - sg)) < 1e-15


@pytest.mark.parametrize("causal", [False, True])
def test_invariants_of_the_softmax_jacobian(causal):
    B, H, Sq, Skv, D = 1, 3, 37, 29, 16
    q, k, v = synth.make_qkv(B, H, Sq, Skv, D, 8)
    d_o = synth.make_do(B, H, Sq, D, 8)
    dq, dk, dv = attn_bwd_ref(q, k, v, d_o, causal, 0.3)
    # shifting every key by one vector leaves the softmax unchanged: the dK rows sum to zero
    assert np.max(np.abs(dk.sum(axis=2))) < 1e-12
    # every row of P sums to one: the dV rows sum to the dO rows
    assert np.max(np.abs(dv.sum(axis=2) - widen(d_o, "bf16").sum(axis=2))) < 1e-12
    # a constant V makes O constant: no gradient reaches q or k
    vc = np.broadcast_to(bf16(np.linspace(-1, 1, D)), v.shape).copy()
    dq2, dk2, _ = attn_bwd_ref(q, k, vc, d_o, causal, 0.3)
    assert np.max(np.abs(dq2)) < 1e-13 and np.max(np.abs(dk2)) < 1e-13


def test_causal_keys_nobody_sees_get_no_gradient():
    # S_kv > S_q, top-left aligned: keys j >= S_q are invisible to every row
    q, k, v = synth.make_qkv(1, 1, 6, 11, 8, 4)
    d_o = synth.make_do(1, 1, 6, 8, 4)
    dq, dk, dv = attn_bwd_ref(q, k, v, d_o, True, 0.5)
    assert np.all(dk[:, :, 6:] == 0) and np.all(dv[:, :, 6:] == 0)
    assert np.any(dk[:, :, :6] != 0)
    # row 0 sees only key 0 -> no gradient to q_0; the last key only gets row 5's term
    assert np.all(dq[0, 0, 0] == 0)
    # causal gradients of the first n rows = non-causal gradients with dO zeroed below row n, keys cut at n
    n = 4
    d_cut = d_o.copy()
    d_cut[:, :, n:] = 0
    dq_c, dk_c, dv_c = attn_bwd_ref(q, k, v, d_cut, True, 0.5)
    dq_t, dk_t, dv_t = attn_bwd_ref(q[:, :, :n], k[:, :, :n], v[:, :, :n], d_o[:, :, :n], True, 0.5)
    assert np.max(np.abs(dq_c[:, :, :n] - dq_t)) < 1e-14
    assert np.max(np.abs(dk_c[:, :, :n] - dk_t)) < 1e-14 and np.max(np.abs(dv_c[:, :, :n] - dv_t)) < 1e-14


def test_linear_in_d_o_and_head_subset_and_threads():
    q, k, v = synth.make_qkv(2, 2, 19, 23, 8, 6)
    d1 = synth.make_do(2, 2, 19, 8, 6)
    g1 = attn_bwd_ref(q, k, v, d1, False, 0.4)
    d2 = bf16(2.0 * synth.bf16_bits_to_f32(d1))
    g2 = attn_bwd_ref(q, k, v, d2, False, 0.4)
    for a, b in zip(g1, g2):
        assert np.max(np.abs(2 * a - b)) < 1e-13
    heads = np.array([3, 0], dtype=np.int64)
    gs = attn_bwd_ref(q, k, v, d1, False, 0.4, heads=heads)
    for full, sub in zip(g1, gs):
        flat = full.reshape((4,) + full.shape[2:])
        assert np.max(np.abs(sub - flat[heads])) < 1e-14
    gt = attn_bwd_ref(q, k, v, d1, False, 0.4, n_threads=1)
    for a, b in zip(g1, gt):
        assert np.max(np.abs(a - b)) < 1e-13


def test_bad_arguments_raise():
    q, k, v = synth.make_qkv(1, 1, 4, 4, 8, 1)
    d_o = synth.make_do(1, 1, 4, 8, 1)
    with pytest.raises(ValueError):
        attn_bwd_ref(q, k, v, d_o[:, :, :3], False, 1.0)
    with pytest.raises(RuntimeError):
        attn_bwd_ref(q, k, v, d_o, False, 1.0, heads=np.array([1], dtype=np.int64))
    with pytest.raises(TypeError):
        attn_bwd_ref(q.astype(np.float32), k, v, d_o, False, 1.0)
