"""Parity of attn_fwd_splitkv (through the C ABI) against the fp64 oracle, and agreement with attn_fwd.

Same tolerances as the unsplit path: max |dO| <= 2e-2 (bf16 O), max |dLSE| <= 1e-3.  The partial
results are fp32, so the merge adds rounding of order 1e-7 only.
"""
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


def run_split(B, q, k, v, n_split, scale):
    qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    o = torch.full(qd.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full(qd.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    need = B.attn_fwd_splitkv_workspace_bytes(qd.shape[0], qd.shape[1], qd.shape[2], qd.shape[3], n_split)
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device="cuda")   # exactly the stated size
    B.attn_fwd_splitkv(qd, kd, vd, n_split, o, lse, ws, scale=scale)
    torch.cuda.synchronize()
    return o_to_f64(o), lse.cpu().numpy().astype(np.float64)


CASES = [
    # B, H, S_q, S_kv, D, n_split
    (1, 2, 100, 1000, 128, 1),
    (1, 2, 100, 1000, 128, 2),
    (1, 2, 100, 1000, 128, 3),
    (1, 2, 100, 1000, 128, 7),
    (2, 1, 300, 4097, 64, 4),
    (1, 3, 1, 777, 128, 5),
    (1, 1, 257, 100, 64, 8),      # more ranges asked for than 64-key tiles exist
    (1, 1, 64, 64, 128, 2),       # a single tile: falls back to one range
    (2, 2, 513, 2048, 128, 16),
    (1, 1, 40, 16384, 64, 256),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "B%d_H%d_Sq%d_Skv%d_D%d_split%d" % c)
def test_split_matches_oracle(B, case):
    b, h, sq, skv, d, n_split = case
    print("splitkv case", case, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=700 + skv + n_split)
    scale = synth.default_scale(d)
    og, lg = run_split(B, q, k, v, n_split, scale)
    orf, lrf = attn_ref(q, k, v, False, scale)
    assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
    eo, el = np.max(np.abs(og - orf)), np.max(np.abs(lg - lrf))
    print("%s max|dO|=%.3e max|dLSE|=%.3e" % (case, eo, el), flush=True)
    assert eo <= O_TOL and el <= LSE_TOL


@pytest.mark.parametrize("case", [(1, 2, 100, 1000, 128, 3), (2, 1, 300, 4097, 64, 4), (1, 3, 1, 777, 128, 5),
                                  (1, 1, 64, 64, 128, 2), (1, 1, 40, 16384, 64, 256)],
                         ids=lambda c: "f16_B%d_H%d_Sq%d_Skv%d_D%d_split%d" % c)
def test_split_f16_matches_oracle(B, case):
    # attn_fwd_splitkv_f16: same launch, fp16 tensors; the O bar of the fp16 forward tests (4e-3)
    b, h, sq, skv, d, n_split = case
    print("splitkv f16 case", case, flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=800 + skv + n_split, dtype="f16")
    scale = synth.default_scale(d)
    dev = lambda bits: torch.from_numpy(bits.view(np.int16)).cuda().view(torch.float16)
    o = torch.full((b, h, sq, d), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((b, h, sq), float("nan"), dtype=torch.float32, device="cuda")
    B.attn_fwd_splitkv_f16(dev(q), dev(k), dev(v), n_split, o, lse, scale=scale)
    torch.cuda.synchronize()
    og, lg = o.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    orf, lrf = attn_ref(q, k, v, False, scale, dtype="f16")
    assert np.all(np.isfinite(og)) and np.all(np.isfinite(lg))
    eo, el = np.max(np.abs(og - orf)), np.max(np.abs(lg - lrf))
    print("%s max|dO|=%.3e max|dLSE|=%.3e" % (case, eo, el), flush=True)
    assert eo <= 4e-3 and el <= LSE_TOL


def test_sharp_softmax_and_agreement_with_unsplit(B):
    # per-row offsets: the ranges have very different maxima, so the merge weights span many decades
    b, h, sq, skv, d = 1, 4, 200, 3000, 128
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=9, sharp=True)
    scale = synth.default_scale(d)
    og, lg = run_split(B, q, k, v, 6, scale)
    orf, lrf = attn_ref(q, k, v, False, scale)
    assert np.max(np.abs(og - orf)) <= O_TOL and np.max(np.abs(lg - lrf)) <= LSE_TOL
    o1, l1 = B.attn_fwd(to_dev(q), to_dev(k), to_dev(v), scale=scale)
    torch.cuda.synchronize()
    assert np.max(np.abs(og - o_to_f64(o1))) <= 2.0 ** -5          # a few bf16 ulps of |O| <= 4
    assert np.max(np.abs(lg - l1.cpu().numpy())) <= 1e-4
    # deterministic for a given n_split
    og2, lg2 = run_split(B, q, k, v, 6, scale)
    assert np.array_equal(og, og2) and np.array_equal(lg, lg2)


def test_long_context_shape_all_rows(B):
    # the shape the bench times (few query tiles, long S_kv), every row against the oracle
    b, h, sq, skv, d, n_split = 1, 8, 256, 32768, 128, 32
    print("splitkv long context", flush=True)
    q, k, v = synth.make_qkv(b, h, sq, skv, d, seed=21)
    scale = synth.default_scale(d)
    og, lg = run_split(B, q, k, v, n_split, scale)
    orf, lrf = attn_ref(q, k, v, False, scale)
    eo, el = np.max(np.abs(og - orf)), np.max(np.abs(lg - lrf))
    print("long context max|dO|=%.3e max|dLSE|=%.3e" % (eo, el), flush=True)
    assert eo <= O_TOL and el <= LSE_TOL


def test_rejected_arguments(B):
    q = torch.zeros((1, 1, 8, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.AttnError) as e:
        B.attn_fwd_splitkv(q, q, q, 2, causal=True)
    assert e.value.status == B.ATTN_ERR_UNSUPPORTED
    small = torch.zeros((64,), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.AttnError) as e:
        B.attn_fwd_splitkv(q, q, q, 2, workspace=small)
    assert e.value.status == B.ATTN_ERR_WORKSPACE
