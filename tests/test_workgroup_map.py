"""The work decomposition (workgroup id -> head, tile) as host logic, through the library's
attn_workgroup_tile diagnostic: every (head, tile) pair is handed out exactly once, and the order has
the locality and balance properties the kernels rely on.  Workgroup ids reach the 8 XCDs round-robin,
so the ids with the same value mod 8 are one XCD's queue, in dispatch order.
"""
import ctypes

import pytest

N_XCD = 8
GROUP_WGS = 64      # workgroups of one causal group per XCD: two per CU


@pytest.fixture(scope="module")
def B():
    from paper_2512_18134_amd import binding
    return binding


def table(B, causal, n_heads, n_tiles):
    return [B.attn_workgroup_tile(causal, w, n_heads, n_tiles) for w in range(n_heads * n_tiles)]


SHAPES = [(1, 1), (1, 7), (3, 5), (8, 1), (8, 64), (16, 64), (24, 33), (32, 16), (40, 4), (128, 8), (13, 9),
          (7, 128), (64, 3), (24, 65), (8, 200)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "heads%d_tiles%d" % s)
def test_every_pair_exactly_once(B, causal, shape):
    n_heads, n_tiles = shape
    t = table(B, causal, n_heads, n_tiles)
    assert sorted(t) == [(h, q) for h in range(n_heads) for q in range(n_tiles)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "heads%d_tiles%d" % s)
def test_full_attention_gives_each_xcd_a_contiguous_range(B, shape):
    # all tiles of a head (and neighbouring heads) stream the same K/V through one L2
    n_heads, n_tiles = shape
    t = table(B, False, n_heads, n_tiles)
    flat = [h * n_tiles + q for h, q in t]
    bounds = []
    for x in range(N_XCD):
        ids = flat[x::N_XCD]
        if ids:
            assert ids == list(range(ids[0], ids[0] + len(ids)))     # in order, no gaps
            bounds.append((ids[0], ids[-1]))
    assert all(a[1] + 1 == b[0] for a, b in zip(bounds, bounds[1:]))


@pytest.mark.parametrize("shape", [s for s in SHAPES if s[0] % N_XCD == 0], ids=lambda s: "heads%d_tiles%d" % s)
def test_causal_with_whole_heads_per_xcd(B, shape):
    n_heads, n_tiles = shape
    nh = n_heads // N_XCD
    gsz = min(nh, -(-GROUP_WGS // n_tiles))
    t = table(B, True, n_heads, n_tiles)
    for x in range(N_XCD):
        queue = t[x::N_XCD]
        assert {h for h, _ in queue} == set(range(x * nh, (x + 1) * nh))      # whole heads, K/V in one L2
        pos = 0
        for first in range(0, nh, gsz):                                       # group after group
            heads = list(range(x * nh + first, x * nh + min(first + gsz, nh)))
            group = queue[pos:pos + len(heads) * n_tiles]
            pos += len(group)
            assert sorted(group) == [(h, q) for h in heads for q in range(n_tiles)]
            tiles = [q for _, q in group]
            assert tiles == sorted(tiles, reverse=True)                       # heaviest (last) tiles first
            # ... and across the heads of the group, not head after head
            assert [h for h, _ in group[:len(heads)]] == heads
        assert pos == len(queue)
        # the workgroups in flight on an XCD (32 CUs) belong to few heads
        for i in range(0, len(queue) - 31):
            assert len({h for h, _ in queue[i:i + 32]}) <= 2 * gsz


@pytest.mark.parametrize("shape", [s for s in SHAPES if s[0] % N_XCD != 0], ids=lambda s: "heads%d_tiles%d" % s)
def test_causal_otherwise_is_heaviest_first_over_the_grid(B, shape):
    n_heads, n_tiles = shape
    tiles = [q for _, q in table(B, True, n_heads, n_tiles)]
    assert tiles == sorted(tiles, reverse=True)


def test_arguments_are_checked(B):
    for bad in [(0, 0, 4), (0, 4, 0), (-1, 4, 4), (16, 4, 4), (0, 1 << 16, 1 << 16)]:
        with pytest.raises(B.AttnError) as e:
            B.attn_workgroup_tile(False, *bad)
        assert e.value.status == B.ATTN_ERR_SHAPE
    lib = ctypes.CDLL(B._lib._name)
    lib.attn_workgroup_tile.argtypes = [ctypes.c_int] * 4 + [ctypes.c_void_p] * 2
    assert lib.attn_workgroup_tile(0, 0, 1, 1, None, None) == B.ATTN_ERR_NULL
