"""Host-side check of the work decomposition of stage 3 (Eq. 3-4 over ragged heads): the plan the
library's kernels evaluate (httm_attention_split_plan runs the same functions on the host) must cut
the tiles in excess into segments that cover every (query tile, key tile) pair exactly once, in
slots nobody else writes, within the scratch size the library asks for.  No GPU needed."""
import numpy as np
import pytest

import paper_2511_21317_amd as httm

SLOT_BYTES = 256 * 66 * 4


def _offsets(lengths):
    return [int(x) for x in np.concatenate([[0], np.cumsum(lengths)])]


def _check_plan(mq, mk, cus):
    qo, ko = _offsets(mq), _offsets(mk)
    p = httm.attention_split_plan(qo, ko, cus)
    H = len(mq)
    full = [m // 256 for m in mq]
    ragged = [h for h in range(H) if mq[h] % 256]
    T = sum(full) + len(ragged)
    if p["n_tiles"] == 0:
        assert p["kept_full"] == sum(full) and p["split_ragged"] == 0 and p["slots"] == 0
        return p
    R = T % cus
    assert p["n_tiles"] == R and 0 < R
    assert p["slots"] * SLOT_BYTES <= httm.attention_scratch_bytes(H)
    assert 1 <= p["shares"] <= 512 and p["span"] >= 1
    # which tiles are split: the first split_ragged partial tiles (head order) and the last full tiles
    n_split_full = R - p["split_ragged"]
    assert p["kept_full"] == sum(full) - n_split_full and 0 <= p["split_ragged"] <= len(ragged)
    want_tiles = [(h, full[h] * 256) for h in ragged[:p["split_ragged"]]]
    flat_full = [(h, t * 256) for h in range(H) for t in range(full[h])]
    want_tiles += flat_full[p["kept_full"]:]
    tiles = p["tiles"]
    assert [(int(t[0]), int(t[1])) for t in tiles] == want_tiles
    # the segments: one per slot; a slot may be unused (a share and a tile end at the same unit)
    seg = p["segments"]
    assert seg.shape[0] == p["slots"] == p["shares"] + R - 1
    cover = {tile: [] for tile in want_tiles}
    units_of_share = np.zeros(p["shares"], dtype=np.int64)
    tiles_of_share = [[] for _ in range(p["shares"])]
    u = p["share_units"]
    used = 0
    for slot in range(p["slots"]):
        head, q0, t0, t1, sl = (int(x) for x in seg[slot])
        assert sl == slot
        if t0 >= t1:
            continue
        used += 1
        e = want_tiles.index((head, q0))
        s_ = slot - e
        assert 0 <= s_ < p["shares"]
        kt = -(-mk[head] // 64)
        assert 0 <= t0 < t1 <= kt
        cover[(head, q0)].append((s_, t0, t1))
        units_of_share[s_] += t1 - t0
        tiles_of_share[s_].append(e)
    for s_ in range(p["shares"]):
        want_units = u if s_ < p["shares"] - 1 else p["units"] - u * (p["shares"] - 1)
        assert units_of_share[s_] == want_units, f"share {s_} has {units_of_share[s_]} units"
        t = tiles_of_share[s_]
        assert t == list(range(t[0], t[0] + len(t))) and len(t) <= p["span"]      # consecutive tiles
    slots = set(range(used))
    for e, tile in enumerate(want_tiles):
        head = tile[0]
        kt = -(-mk[head] // 64)
        pieces = sorted(cover[tile])
        # the pieces of a tile partition its key tiles, in share order, shares consecutive
        assert pieces[0][1] == 0 and pieces[-1][2] == kt
        for a, b in zip(pieces, pieces[1:]):
            assert a[2] == b[1] and b[0] == a[0] + 1
        assert len(pieces) <= 34
        assert (int(tiles[e][2]), int(tiles[e][3])) == (pieces[0][0], pieces[-1][0])
    assert sum(len(v) for v in cover.values()) == used
    return p


def test_plans_of_the_five_workloads():
    want = {266: 0, 5516: 96, 6376: 144, 28650: 0, 28700: 16}
    for M, n in want.items():
        p = _check_plan([M] * 16, [M] * 16, 256)
        assert p["n_tiles"] == n, (M, p["n_tiles"])
        if n:
            assert 240 <= p["shares"] <= 512 and p["span"] == 2


@pytest.mark.parametrize("seed", range(200))
def test_random_launches_are_covered_exactly_once(seed):
    rng = np.random.default_rng(31000 + seed)
    H = int(rng.integers(1, 20))
    cus = int(rng.choice([256, 256, 256, 64, 304, 8]))
    kind = seed % 4
    if kind == 0:     # equal heads, like a plan's merged sequences
        mq = [int(rng.integers(1, 40000))] * H
        mk = [int(rng.integers(1, 40000))] * H
    elif kind == 1:   # ragged heads
        mq = [int(rng.integers(0, 30000)) for _ in range(H)]
        mk = [int(rng.integers(512, 20000)) for _ in range(H)]
    elif kind == 2:   # few long tiles against long keys
        mq = [int(rng.integers(1, 3000)) for _ in range(H)]
        mk = [int(rng.integers(5000, 200000)) for _ in range(H)]
    else:             # heads of very different key lengths: shares that span several tiles
        mq = [int(rng.integers(200, 70000)) for _ in range(H)]
        mk = [int(rng.choice([512, 700, 5000, 60000])) for _ in range(H)]
    _check_plan(mq, mk, cus)


def test_many_heads_with_partial_tiles():
    # 64 heads, every one with a partial tile: more runs of tiles than the plan can describe is refused
    # (no split), fewer is split
    _check_plan([20000 + 3 * h for h in range(64)], [9000] * 64, 256)
    _check_plan([256 * 7 + 5] * 40, [9000] * 40, 256)


def test_split_is_taken_where_it_pays_and_only_there():
    assert _check_plan([522] * 16, [522] * 16, 256)["n_tiles"] == 0            # too short to pay
    assert _check_plan([256 * 16] * 16, [4096] * 16, 256)["n_tiles"] == 0      # a multiple of the CU count
    assert _check_plan([256 * 16 + 1] * 16, [8192] * 16, 256)["n_tiles"] == 16
    assert _check_plan([256 * 31] * 16, [32768] * 16, 256)["n_tiles"] == 240   # 496 tiles: 240 in excess, long keys
    assert _check_plan([256 * 31] * 16, [8192] * 16, 256)["n_tiles"] == 0      # the same with shorter keys: no gain
    assert _check_plan([300] * 4, [100] * 4, 256)["n_tiles"] == 0              # fewer than 512 keys
