"""Seeded synthetic Q/K/V for the attention forward path.

This module is shared by the tests, the oracle's callers and the bench.  It
holds none of the attention arithmetic: it only produces 16-bit float bit patterns
(bf16, or IEEE fp16 with dtype="f16").

The generator is counter based, so every element depends only on
(seed, tensor id, flat index): generation order, chunking and threading do not
change the bits.

    key   = splitmix64(splitmix64(seed) ^ (0x9E3779B97F4A7C15 * (tensor_id + 1)))
    u1,u2 = two splitmix64 outputs of counters key + 2*idx, key + 2*idx + 1,
            mapped to (0,1) with 53 bits:  ((z >> 11) + 0.5) / 2**53
    z     = sqrt(-2 ln u1) * cos(2 pi u2)            (Box-Muller, fp64)
    value = RNE_bf16( fp32(z) [+ fp32(row offset)] )

The paper's evaluation (Section 6.2) uses random FP16 inputs of shape
(BATCH, NUM_HEADS, seq, HEAD_DIM); the five workloads here have the shapes and
distributions of this library's benchmark set (bf16, iid N(0,1); the last one
adds a per-row N(0, sigma=2) offset to Q and K, which makes the softmax sharp).
"""
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)

TENSOR_Q, TENSOR_K, TENSOR_V, TENSOR_OFFQ, TENSOR_OFFK, TENSOR_DO = 0, 1, 2, 3, 4, 5


def _splitmix64(x):
    """splitmix64 output function on a uint64 array (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = x + _GOLD
        z = (z ^ (z >> np.uint64(30))) * _C1
        z = (z ^ (z >> np.uint64(27))) * _C2
        return z ^ (z >> np.uint64(31))


def _key(seed, tensor_id):
    s = _splitmix64(np.array([seed], dtype=np.uint64))
    with np.errstate(over="ignore"):
        t = _GOLD * np.uint64(tensor_id + 1)
    return _splitmix64(s ^ t)[0]


def normal_f64(seed, tensor_id, start, count):
    """`count` standard normals (fp64) for flat indices start .. start+count-1."""
    key = _key(seed, tensor_id)
    idx = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        c0 = key + idx * np.uint64(2)
        c1 = c0 + np.uint64(1)
    inv = 1.0 / float(1 << 53)
    u1 = ((_splitmix64(c0) >> np.uint64(11)).astype(np.float64) + 0.5) * inv
    u2 = ((_splitmix64(c1) >> np.uint64(11)).astype(np.float64) + 0.5) * inv
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16).  Finite input."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return ((b + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_f16_bits(x):
    """Round-to-nearest-even fp32 -> IEEE fp16 bit patterns (uint16)."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(bits):
    """Exact widening of fp16 bit patterns (uint16) to fp32."""
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float32)


def normal_bf16(seed, tensor_id, shape, row_offset_id=None, row_offset_sigma=0.0, chunk=1 << 22, dtype="bf16"):
    """16-bit patterns (bf16, or fp16 with dtype="f16") of iid N(0,1) values of `shape`
    ([..., D]); optionally every row (last axis) gets one extra scalar
    N(0, row_offset_sigma^2) added in fp32 before the rounding to 16 bits."""
    pack = {"bf16": f32_to_bf16_bits, "f16": f32_to_f16_bits}[dtype]
    n = int(np.prod(shape))
    d = int(shape[-1])
    out = np.empty(n, dtype=np.uint16)
    if row_offset_id is not None:
        off = (normal_f64(seed, row_offset_id, 0, n // d) * row_offset_sigma).astype(np.float32)
    chunk = max(d, (chunk // d) * d)
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        x = normal_f64(seed, tensor_id, s, c).astype(np.float32)
        if row_offset_id is not None:
            x = (x.reshape(-1, d) + off[s // d:(s + c) // d, None]).reshape(-1)
        out[s:s + c] = pack(x)
    return out.reshape(shape)


# The five benchmark workloads, numbered 1..5 as in the build's baseline statement (bench.py --config N;
# config 4 is the headline); the seed of config N is N - 1.
CONFIGS = {
    1: dict(name="config1_B1_H1_S128_D64_full", B=1, H=1, S_q=128, S_kv=128, D=64, causal=False, seed=0, sharp=False),
    2: dict(name="config2_B4_H16_S1024_D64_full", B=4, H=16, S_q=1024, S_kv=1024, D=64, causal=False, seed=1, sharp=False),
    3: dict(name="config3_B2_H16_S4096_D128_causal", B=2, H=16, S_q=4096, S_kv=4096, D=128, causal=True, seed=2, sharp=False),
    4: dict(name="config4_B1_H16_S16384_D128_full", B=1, H=16, S_q=16384, S_kv=16384, D=128, causal=False, seed=3, sharp=False),
    5: dict(name="config5_B1_H8_S8192_D256_causal_sharp", B=1, H=8, S_q=8192, S_kv=8192, D=256, causal=True, seed=4, sharp=True),
}
HEADLINE_CONFIG = 4


def default_scale(D):
    """1/sqrt(D) rounded to fp32: the value handed to both sides."""
    return float(np.float32(1.0 / np.sqrt(np.float64(D))))


def make_qkv(B, H, S_q, S_kv, D, seed, sharp=False, dtype="bf16"):
    """(q, k, v) as uint16 arrays of `dtype` bits ("bf16" or "f16"), shapes [B,H,S_q,D], [B,H,S_kv,D] x2."""
    if sharp:
        q = normal_bf16(seed, TENSOR_Q, (B, H, S_q, D), TENSOR_OFFQ, 2.0, dtype=dtype)
        k = normal_bf16(seed, TENSOR_K, (B, H, S_kv, D), TENSOR_OFFK, 2.0, dtype=dtype)
    else:
        q = normal_bf16(seed, TENSOR_Q, (B, H, S_q, D), dtype=dtype)
        k = normal_bf16(seed, TENSOR_K, (B, H, S_kv, D), dtype=dtype)
    v = normal_bf16(seed, TENSOR_V, (B, H, S_kv, D), dtype=dtype)
    return q, k, v


def make_do(B, H, S_q, D, seed, dtype="bf16"):
    """Upstream gradient dO for the backward pass: iid N(0,1), same generator, its own tensor id."""
    return normal_bf16(seed, TENSOR_DO, (B, H, S_q, D), dtype=dtype)


def paper_workload(seq, causal, D=128, BH=128):
    """Shape of the paper's Section 6.2 sweep: BATCH * NUM_HEADS = BH heads of HEAD_DIM = 128, fp16
    N(0,1) inputs, `seq` queries and keys; the figure's x axis is `seq` (1k .. 16k)."""
    return dict(name="paper_B%d_H32_S%d_D%d_%s_f16" % (BH // 32, seq, D, "causal" if causal else "full"),
                B=BH // 32, H=32, S_q=seq, S_kv=seq, D=D, causal=bool(causal), seed=100 + seq // 1024,
                sharp=False, dtype="f16")


def make_config(number):
    """Inputs of workload `number` (1..5): (cfg dict, q, k, v, scale)."""
    cfg = CONFIGS[number]
    q, k, v = make_qkv(cfg["B"], cfg["H"], cfg["S_q"], cfg["S_kv"], cfg["D"], cfg["seed"], cfg["sharp"])
    return cfg, q, k, v, default_scale(cfg["D"])


def attention_flops(B, H, S_q, S_kv, D, causal):
    """Algorithmic FLOP: 4*D per unmasked (i, j) pair (2*D for QK^T, 2*D for PV)."""
    if causal:
        pairs = sum(min(i + 1, S_kv) for i in range(S_q)) if S_q != S_kv else S_q * (S_q + 1) // 2
    else:
        pairs = S_q * S_kv
    return 4 * B * H * D * pairs
