"""The work decomposition (workgroup id -> head, tile) as host logic, through the library's
attn_workgroup_tile diagnostic: every (head, tile) pair is handed out exactly once, and the order has
the locality and balance properties the kernels rely on.  Workgroup ids reach the 8 XCDs round-robin,
so the ids with the same value mod 8 are one XCD's queue, in dispatch order.
"""
import ctypes

import pytest

N_XCD = 8
L2_BYTES = 4 << 20                  # one XCD's L2
HEAD_BYTES = [0, 256 << 10, 1 << 20, 3 << 20, 64 << 20]


def group_heads(n_tiles, head_bytes):
    """Heads per causal group: between 32 and 128 workgroups, as many heads as stream no more than one L2
    of operands between them; heads that do not fit an L2 twice over get the large groups."""
    lo, hi = -(-32 // n_tiles), -(-128 // n_tiles)
    fit = L2_BYTES // head_bytes if head_bytes else hi
    return hi if fit < 2 else min(max(fit, lo), hi)


@pytest.fixture(scope="module")
def B():
    from paper_2512_18134_amd import binding
    return binding


def table(B, causal, n_heads, n_tiles, head_bytes=0):
    return [B.attn_workgroup_tile(causal, w, n_heads, n_tiles, head_bytes) for w in range(n_heads * n_tiles)]


SHAPES = [(1, 1), (1, 7), (3, 5), (8, 1), (8, 64), (16, 64), (24, 33), (32, 16), (40, 4), (128, 8), (13, 9),
          (7, 128), (64, 3), (24, 65), (8, 200)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "heads%d_tiles%d" % s)
def test_every_pair_exactly_once(B, causal, shape):
    n_heads, n_tiles = shape
    for head_bytes in HEAD_BYTES:
        t = table(B, causal, n_heads, n_tiles, head_bytes)
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


@pytest.mark.parametrize("head_bytes", HEAD_BYTES, ids=lambda b: "%dKiB" % (b >> 10))
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "heads%d_tiles%d" % s)
def test_causal_queues(B, shape, head_bytes):
    # XCD x owns the whole heads x*a .. x*a + a - 1; the n_heads % 8 heads left over are shared out
    # tile by tile and come first in every queue
    n_heads, n_tiles = shape
    a, r = divmod(n_heads, N_XCD)
    want = group_heads(n_tiles, head_bytes)
    ng = a // want if a > want else 1
    sizes = [a // ng + 1] * (a % ng) + [a // ng] * (ng - a % ng) if a else []
    assert sum(sizes) == a and all(z >= min(want, a) for z in sizes)
    t = table(B, True, n_heads, n_tiles, head_bytes)
    left_weight = []
    for x in range(N_XCD):
        queue = t[x::N_XCD]
        m = -(-(r * n_tiles - x) // N_XCD) if r * n_tiles > x else 0
        head_part, queue = queue[:m], queue[m:]
        assert all(h >= N_XCD * a for h, _ in head_part)                      # left-over heads only
        tiles = [q for _, q in head_part]
        assert tiles == sorted(tiles, reverse=True)                           # heaviest first
        left_weight.append(sum(q + 1 for q in tiles))
        assert {h for h, _ in queue} == set(range(x * a, (x + 1) * a))        # whole heads, K/V in one L2
        pos, first = 0, 0
        for z in sizes:                                                       # group after group
            heads = list(range(x * a + first, x * a + first + z))
            first += z
            group = queue[pos:pos + z * n_tiles]
            pos += len(group)
            assert sorted(group) == [(h, q) for h in heads for q in range(n_tiles)]
            tiles = [q for _, q in group]
            assert tiles == sorted(tiles, reverse=True)                       # heaviest (last) tiles first
            # ... and across the heads of the group, not head after head
            assert [h for h, _ in group[:z]] == heads
        assert pos == len(queue)
        # the workgroups in flight on an XCD (32 CUs) belong to few heads
        for i in range(0, len(queue) - 31):
            assert len({h for h, _ in queue[i:i + 32]}) <= 2 * max(sizes)
    # the left-over tiles weigh about the same on every XCD (tile q streams ~ q + 1 units)
    assert max(left_weight) - min(left_weight) <= 16


def test_arguments_are_checked(B):
    for bad in [(0, 0, 4), (0, 4, 0), (-1, 4, 4), (16, 4, 4), (0, 1 << 16, 1 << 16), (0, 4, 4, -1)]:
        with pytest.raises(B.AttnError) as e:
            B.attn_workgroup_tile(False, *bad)
        assert e.value.status == B.ATTN_ERR_SHAPE
    lib = ctypes.CDLL(B._lib._name)
    lib.attn_workgroup_tile.argtypes = [ctypes.c_int] * 4 + [ctypes.c_longlong] + [ctypes.c_void_p] * 2
    assert lib.attn_workgroup_tile(0, 0, 1, 1, 0, None, None) == B.ATTN_ERR_NULL


def test_group_sizes_follow_the_l2(B):
    # 16 heads per XCD, 4 tiles each (D = 128, S = 1024 forward): K and V of a head are 512 KiB, eight
    # heads fill the 4 MiB L2 -> groups of 8 heads (32 workgroups); at 4 KiB per head the cap of 128
    # workgroups decides (32 heads asked, 16 there); heads of 8 MiB cannot share an L2 by fitting and get
    # the large groups as well
    for head_bytes, heads in ((512 << 10, 8), (4 << 10, 16), (8 << 20, 16), (1 << 20, 8), (2 << 20, 8)):
        queue = table(B, True, 128, 4, head_bytes)[0::N_XCD]
        first_group = {h for h, _ in queue[:heads * 4]}
        assert len(first_group) == heads and len({h for h, _ in queue[:heads * 4 + 1]}) == heads + (heads < 16)


def queue_walk(B, n_wg, n_entries):
    """{workgroup: [entries in pass order]} of a persistent launch, walked until a pass is empty for everybody."""
    walk = {w: [] for w in range(n_wg)}
    k = 0
    while True:
        got = [B.attn_workgroup_queue_entry(w, n_wg, n_entries, k) for w in range(n_wg)]
        if all(e < 0 for e in got):
            return walk
        for w, e in enumerate(got):
            if e >= 0:
                walk[w].append(e)
        k += 1
        assert k < 10000


def test_persistent_workgroups_take_every_queue_entry_once(B):
    for n_wg, n_entries in ((256, 512), (256, 1024), (256, 257), (256, 300), (512, 513), (512, 2048), (8, 9), (8, 1000),
                            (16, 23), (256, 256), (300, 200), (7, 7), (256, 1), (264, 1000)):
        walk = queue_walk(B, n_wg, n_entries)
        seen = sorted(e for es in walk.values() for e in es)
        assert seen == list(range(n_entries)), (n_wg, n_entries)
        if n_wg < n_entries:
            for w, es in walk.items():
                # a workgroup stays on its XCD's entries, never skips a pass before its last, and the numbers of
                # entries of two workgroups differ by one at most
                assert all(e % 8 == w % 8 for e in es)
                assert len(es) >= 1
            sizes = [len(es) for es in walk.values()]
            assert max(sizes) - min(sizes) <= 1


def test_persistent_walk_pairs_heavy_with_light(B):
    # entries queued heaviest first (a causal launch): weight of entry e falls with e.  Two passes over 256
    # slots: every slot's load is the same up to one step of the weight
    n_wg, n_entries = 256, 512
    walk = queue_walk(B, n_wg, n_entries)
    weight = lambda e: n_entries // 8 - e // 8          # an XCD's queue position decides the weight
    loads = [sum(weight(e) for e in es) for es in walk.values()]
    assert max(loads) - min(loads) == 0
    # four passes: still even
    walk = queue_walk(B, 256, 1024)
    weight = lambda e: 1024 // 8 - e // 8
    loads = [sum(weight(e) for e in es) for es in walk.values()]
    assert max(loads) - min(loads) == 0
    # a third, short pass goes to the slots that got the lighter pairs... at least nobody gets two more than another
    walk = queue_walk(B, 256, 600)
    assert max(len(es) for es in walk.values()) - min(len(es) for es in walk.values()) <= 1


def test_queue_entry_arguments_are_checked(B):
    for bad in [(0, 0, 4, 0), (0, 4, 0, 0), (-1, 8, 16, 0), (8, 8, 16, 0), (0, 8, 16, -1), (0, 12, 16, 0)]:
        with pytest.raises(B.AttnError) as e:
            B.attn_workgroup_queue_entry(*bad)
        assert e.value.status == B.ATTN_ERR_SHAPE
    lib = ctypes.CDLL(B._lib._name)
    lib.attn_workgroup_queue_entry.argtypes = [ctypes.c_int] * 4 + [ctypes.c_void_p]
    assert lib.attn_workgroup_queue_entry(0, 8, 16, 0, None) == B.ATTN_ERR_NULL
