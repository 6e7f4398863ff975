"""Input generator: determinism, order independence, bf16 rounding, moments."""
import numpy as np

from paper_2512_18134_amd import synth


def test_counter_based_is_chunk_independent():
    a = synth.normal_bf16(7, synth.TENSOR_Q, (3, 5, 64), chunk=64)
    b = synth.normal_bf16(7, synth.TENSOR_Q, (3, 5, 64), chunk=1 << 20)
    assert np.array_equal(a, b)
    x = synth.normal_f64(7, synth.TENSOR_Q, 100, 50)
    y = synth.normal_f64(7, synth.TENSOR_Q, 0, 200)[100:150]
    assert np.array_equal(x, y)


def test_streams_differ_by_seed_and_tensor():
    a = synth.normal_f64(1, synth.TENSOR_Q, 0, 1000)
    b = synth.normal_f64(2, synth.TENSOR_Q, 0, 1000)
    c = synth.normal_f64(1, synth.TENSOR_K, 0, 1000)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.15
    assert abs(np.corrcoef(a, c)[0, 1]) < 0.15


def test_moments():
    x = synth.normal_f64(3, synth.TENSOR_V, 0, 1 << 20)
    assert abs(x.mean()) < 5e-3
    assert abs(x.std() - 1.0) < 5e-3
    assert abs(((x ** 4).mean()) - 3.0) < 0.05


def test_bf16_rne():
    # 1 + 2^-8 is exactly half way between bf16 neighbours 1 and 1 + 2^-7: ties to even (1.0)
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(x)
    back = synth.bf16_bits_to_f32(bits)
    assert back.tolist() == [1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -2.5, 0.0]
    # round trip of every finite bf16 pattern is the identity
    allbits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    f = synth.bf16_bits_to_f32(allbits)
    fin = np.isfinite(f)
    assert np.array_equal(synth.f32_to_bf16_bits(f[fin]), allbits[fin])


def test_f16_generation_is_the_same_normals_rounded_to_half():
    shape = (1, 2, 33, 64)
    b = synth.make_qkv(1, 2, 33, 33, 64, 5)[0]
    h = synth.make_qkv(1, 2, 33, 33, 64, 5, dtype="f16")[0]
    assert h.dtype == np.uint16 and h.shape == shape
    x = synth.normal_f64(5, synth.TENSOR_Q, 0, int(np.prod(shape))).astype(np.float32).reshape(shape)
    assert np.array_equal(h.view(np.float16), x.astype(np.float16))
    # fp16 keeps 3 more fraction bits than bf16 for |x| in normal range
    eb = np.abs(synth.bf16_bits_to_f32(b) - x).max()
    eh = np.abs(synth.f16_bits_to_f32(h) - x).max()
    assert eh < eb / 4
    assert np.array_equal(synth.f32_to_f16_bits(synth.f16_bits_to_f32(h)), h)
    w = synth.paper_workload(16384, False)
    assert (w["B"], w["H"], w["S_q"], w["S_kv"], w["D"], w["causal"], w["dtype"]) == (4, 32, 16384, 16384, 128, False, "f16")


def test_sharp_rows_have_offsets():
    q, k, v = synth.make_qkv(1, 2, 64, 64, 256, seed=4, sharp=True)
    qf = synth.bf16_bits_to_f32(q)
    row_means = qf.mean(axis=-1)
    assert 1.5 < row_means.std() < 2.5      # N(0, sigma=2) per row
    vf = synth.bf16_bits_to_f32(v)
    assert abs(vf.mean(axis=-1).std()) < 0.2  # V has none


def test_flop_count():
    assert synth.attention_flops(1, 1, 128, 128, 64, False) == 4194304
    assert synth.attention_flops(2, 16, 4096, 4096, 128, True) == 137472507904
    assert synth.attention_flops(1, 16, 16384, 16384, 128, False) == 2199023255552
    assert synth.attention_flops(1, 1, 5, 3, 2, True) == 4 * 2 * (1 + 2 + 3 + 3 + 3)
