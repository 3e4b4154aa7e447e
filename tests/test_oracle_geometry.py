"""Pins for the oracle's geometry: temporal reordering (Sec. 3.3) and merged counts (Sec. 3.2)."""
import collections
import os

import numpy as np
import pytest

from oracle import httm_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden_rows():
    rows = []
    with open(os.path.join(HERE, "golden", "merged_counts.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            t = line.split()
            cfg, S, Hp, Wp, b, T = (int(x) for x in t[:6])
            rho, N, M = float(t[6]), int(t[7]), int(t[8])
            trip = [int(x) for x in t[9:]]
            hist = {(trip[i], trip[i + 1]): trip[i + 2] for i in range(0, len(trip), 3)}
            rows.append((cfg, orc.Geometry(S, Hp, Wp, b, T), rho, N, M, hist))
    return rows


GEOMS = [
    orc.Geometry(2, 16, 16, 4, 2),
    orc.Geometry(3, 3, 4, 2, 2),        # partial block in rows and in time
    orc.Geometry(5, 7, 5, 4, 3),        # partial everywhere
    orc.Geometry(1, 2, 2, 8, 4),        # block larger than the grid and the sequence
    orc.Geometry(4, 6, 6, 3, 1),        # purely spatial blocks
    orc.Geometry(4, 5, 3, 1, 4),        # purely temporal blocks
    orc.Geometry(3, 4, 4, 2, 2, n_special=0),
]


@pytest.mark.parametrize("g", GEOMS)
def test_pi_is_a_bijection_and_inverts(g):
    pi, blocks = orc.temporal_reorder(g)
    assert pi.shape == (g.N,)
    assert np.array_equal(np.sort(pi), np.arange(g.N))
    x = np.random.default_rng(0).standard_normal((3, g.N, 4)).astype(np.float32)
    xr = orc.reorder(x, pi)
    assert np.array_equal(orc.inverse_reorder(xr, pi), x)
    # reorder really is a row gather
    for j in (0, g.N // 2, g.N - 1):
        assert np.array_equal(xr[:, j], x[:, pi[j]])


@pytest.mark.parametrize("g", GEOMS)
def test_blocks_equal_bruteforce_sets(g):
    """Each block holds exactly the tokens {(f,y,x)} of one (frame group, window), in (f,y,x) order."""
    pi, blocks = orc.temporal_reorder(g)
    # brute force: classify every patch token by its block key
    by_key = collections.OrderedDict()
    for f in range(g.S):
        for y in range(g.Hp):
            for x in range(g.Wp):
                key = (f // g.T, y // g.b, x // g.b)
                by_key.setdefault(key, []).append((f, y, x))
    keys = sorted(by_key)
    assert len(keys) == len(blocks)
    pos = g.n_prefix
    for key, (start, n) in zip(keys, blocks):
        assert start == pos
        want = sorted(by_key[key])
        assert n == len(want)
        got = []
        for j in range(start, start + n):
            f, slot = divmod(int(pi[j]), g.tokens_per_frame)
            assert slot >= g.n_special
            y, x = divmod(slot - g.n_special, g.Wp)
            got.append((f, y, x))
        assert got == want
        pos += n
    assert pos == g.N
    # the prefix holds the specials in (frame, slot) order
    for j in range(g.n_prefix):
        f, s = divmod(j, g.n_special) if g.n_special else (0, 0)
        assert pi[j] == f * g.tokens_per_frame + s


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: f"cfg{r[0]}")
def test_merged_count_matches_closed_form(row):
    cfg, g, rho, N, M, hist = row
    assert g.N == N
    _, blocks = orc.temporal_reorder(g)
    ks, offs, m_total = orc.merged_layout(g, blocks, rho)
    assert m_total == M
    got = collections.Counter((n, k) for (_, n), k in zip(blocks, ks))
    assert dict(got) == hist
    # offsets are the running sum behind the special prefix
    assert offs[0] == g.n_prefix
    assert all(offs[i + 1] == offs[i] + ks[i] for i in range(len(ks) - 1))


def test_ratio_convention_of_the_experiments():
    """Sec. 4.1: 90 % merged leaves 10 %; 70 % merged leaves 30 % (block of 3840 tokens)."""
    assert orc.cluster_count(3840, 0.9) == 384
    assert orc.cluster_count(3840, 0.7) == 1152
    assert orc.cluster_count(7, 0.0) == 7
    assert orc.cluster_count(1, 0.99) == 1
    assert orc.cluster_count(4, 1.0) == 1


@pytest.mark.parametrize("n,k", [(32, 16), (64, 13), (256, 26), (160, 16), (100, 10), (5, 5), (7, 1), (9, 4)])
def test_dst_positions_are_strided_distinct_and_start_at_zero(n, k):
    d = orc.dst_positions(n, k)
    assert d[0] == 0 and len(set(d)) == k and d == sorted(d) and d[-1] < n
    gaps = np.diff(d + [n])
    assert gaps.max() - gaps.min() <= 1


@pytest.mark.parametrize("S,Hp,Wp,b,T", [(4, 5, 7, 2, 2), (3, 37, 37, 4, 4), (1, 4, 4, 4, 2), (8, 16, 16, 8, 3)])
def test_anchor_sizes_cover_frame_zero_exactly(S, Hp, Wp, b, T):
    """App. C.2: the anchored tokens are exactly the patch tokens of frame 0 (closed form: Hp*Wp of
    them, all in the first temporal group, at the front of their blocks)."""
    g = orc.Geometry(S, Hp, Wp, b, T, anchor=True)
    pi, blocks = orc.temporal_reorder(g)
    n0s = orc.anchor_sizes(g)
    assert len(n0s) == len(blocks)
    assert sum(n0s) == Hp * Wp
    tpf = g.tokens_per_frame
    for (start, n), n0 in zip(blocks, n0s):
        frames = pi[start:start + n] // tpf
        assert (frames[:n0] == 0).all() and (frames[n0:] != 0).all()
    assert orc.anchor_sizes(orc.Geometry(S, Hp, Wp, b, T)) == [0] * len(blocks)


@pytest.mark.parametrize("n,k,n0", [(64, 16, 16), (64, 20, 16), (64, 64, 16), (48, 12, 12), (7, 5, 3), (5, 5, 5)])
def test_anchored_dst_positions(n, k, n0):
    d = orc.dst_positions(n, k, n0)
    assert len(d) == k and len(set(d)) == k and d == sorted(d)
    assert d[:n0] == list(range(n0))
    if k > n0:
        assert d[n0] == n0                      # the first free token is a dst, as without anchoring
        rest = [p - n0 for p in d[n0:]]
        assert rest == orc.dst_positions(n - n0, k - n0)
    assert orc.cluster_count(n, 0.99, n0) == max(1, n0)
    assert orc.cluster_count(n, 0.0, n0) == n


def test_chunked_blocks_at_the_papers_setting():
    """Sec. 4.1: n_s = 128 consecutive tokens x n_t = 30 frames = blocks of 3840 tokens; a 37 x 37
    frame has 10 full runs and one of 89; 90 % / 70 % merging keeps 384 / 1152 per full block."""
    g = orc.Geometry(60, 37, 37, 128, 30, chunked=True)
    pi, blocks = orc.temporal_reorder(g)
    assert sorted(pi.tolist()) == list(range(g.N))
    assert len(blocks) == 2 * 11
    sizes = [n for _, n in blocks]
    assert sizes == ([3840] * 10 + [89 * 30]) * 2
    ks, offs, M = orc.merged_layout(g, blocks, 0.9)
    assert ks[:11] == [384] * 10 + [267] and M == g.n_prefix + 2 * (3840 + 267)
    assert orc.merged_layout(g, blocks, 0.7)[0][:11] == [1152] * 10 + [801]
    # a block = the same run of every frame of the group, frames stacked
    tpf = g.tokens_per_frame
    start, n = blocks[12]                      # second group, second run
    got = pi[start:start + n]
    assert (got // tpf).tolist() == [f for f in range(30, 60) for _ in range(128)]
    assert (got % tpf - g.n_special).tolist() == list(range(128, 256)) * 30
    # windows and runs agree when the window is a full row strip: b x b with b = Wp = Hp is one block per frame
    sq = orc.Geometry(4, 6, 6, 6, 2)
    ch = orc.Geometry(4, 6, 6, 36, 2, chunked=True)
    assert np.array_equal(orc.temporal_reorder(sq)[0], orc.temporal_reorder(ch)[0])
    assert orc.temporal_reorder(sq)[1] == orc.temporal_reorder(ch)[1]
