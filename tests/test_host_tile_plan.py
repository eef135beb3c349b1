"""The host-side tile plan (which tile of which segment every workgroup handles) checked on
the CPU with random segment tables: a wrong plan would mean out-of-bounds accesses on the GPU.
No GPU needed."""
import random

import pytest
from hypothesis import given, settings, strategies as st


@pytest.fixture(scope="module")
def B():
    from paper_2504_17672_amd import binding
    return binding


def random_table(rng, n_total, S, K):
    cuts = sorted(rng.sample(range(n_total + 1), min(2 * S, n_total + 1)))
    segs = []
    for a, b in zip(cuts[0::2], cuts[1::2]):
        segs.append((a, b - a, rng.randrange(K)))
    for _ in range(rng.randrange(3)):  # a few empty segments anywhere
        segs.append((rng.randrange(n_total + 1), 0, rng.randrange(K)))
    rng.shuffle(segs)
    return segs


def check_plan(B, segs, K, n_total):
    tile = B.cocodc_tile_elements(n_total)
    rc, so, ss, fs, cap = B.cocodc_debug_tile_plan(segs, K, n_total)
    assert rc == 0
    S = len(segs)
    T = ss[S]
    # walked order: grouped by fragment, listed order inside a fragment
    walked = [sg for p in range(K) for sg in segs if sg[2] == p]
    assert so[:S] == [o for o, _, _ in walked]
    slot = 0
    for j, (o, l, p) in enumerate(walked):
        assert ss[j] == slot
        if l:
            slot += (o + l - 1) // tile - o // tile + 1
    assert T == slot
    # every fragment owns the contiguous slot range of its segments
    assert fs[0] == 0 and fs[K] == T and all(a <= b for a, b in zip(fs, fs[1:]))
    for p in range(K):
        want = sum(((o + l - 1) // tile - o // tile + 1) for o, l, q in segs if q == p and l)
        assert fs[p + 1] - fs[p] == want
    # the workspace has room for every tile's partial sums
    assert T <= cap
    assert B.cocodc_workspace_bytes_segmented(S, K, n_total) >= 32 * T + 48 * (S + K + 2)


@settings(max_examples=150, deadline=None)
@given(st.integers(0, 2 ** 32), st.integers(1, 400_000), st.integers(1, 40), st.integers(1, 9), st.booleans())
def test_random_segment_tables(B, seed, n_used, S, K, large):
    rng = random.Random(seed)
    n_total = n_used + ((1 << 24) if large else 0)  # large: the 4096-element tile applies
    check_plan(B, random_table(rng, n_used, S, K), K, n_total)


def test_boundary_tables(B):
    assert B.cocodc_tile_elements(1 << 20) == 2048 and B.cocodc_tile_elements(1 << 24) == 4096
    for n_big in (0, 1 << 24):  # both tile sizes
        tile = B.cocodc_tile_elements(3 * 16384 + n_big)
        check_plan(B, [(0, tile, 0)], 1, 3 * 16384 + n_big)
        check_plan(B, [(tile - 1, 2, 0), (tile + 1, tile - 1, 1), (2 * tile, 1, 0)], 2, 3 * 16384 + n_big)
    tile = 2048
    check_plan(B, [(0, tile, 0)], 1, tile)
    check_plan(B, [(tile - 1, 2, 0), (tile + 1, tile - 1, 1), (2 * tile, 1, 0)], 2, 3 * tile)
    check_plan(B, [(0, 0, 0)], 3, 10)
    check_plan(B, [(i * 3, 2, i % 5) for i in range(4096)], 5, 4096 * 3)  # the maximum number of segments
    n = 6_607_343_616
    per = n // 32
    check_plan(B, [(p * per, per, p) for p in range(32)], 32, n)
    rc = B.cocodc_debug_tile_plan([(0, 1, 0)] * 4097, 1, 10)[0]
    assert rc == B.COCODC_ERR_RANGE
