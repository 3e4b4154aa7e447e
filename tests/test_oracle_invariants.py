"""Invariants and special cases that pin the oracle to the paper's mathematics."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import httm_oracle as orc


def _rand_qkv(g, H=3, E=16, seed=0, dtype=np.float32):
    rng = np.random.default_rng(seed)
    return tuple(rng.standard_normal((H, g.N, E)).astype(dtype) for _ in range(3))


def _textbook_attention(q, k, v):
    """Eq. 3-4 with library softmax, float64, heads concatenated on channels."""
    H, N, E = q.shape
    q, k, v = (t.astype(np.float64) for t in (q, k, v))
    cols = [softmax(q[h] @ k[h].T / np.sqrt(E), axis=1) @ v[h] for h in range(H)]
    return np.concatenate(cols, axis=1)


@pytest.mark.parametrize("g", [orc.Geometry(3, 5, 6, 4, 2), orc.Geometry(2, 16, 16, 4, 2)])
def test_rho_zero_is_exact_softmax_attention(g):
    q, k, v = _rand_qkv(g)
    ref = _textbook_attention(q, k, v)
    for variant, rho in (("headwise", 0.0), ("none", 0.7)):
        res = orc.layer_forward(q, k, v, g, rho, rho, variant=variant)
        pi, blocks = res["pi"], res["blocks"]
        for h in range(q.shape[0]):
            assert np.array_equal(orc.rep_map(res["assign_q"][h], pi, g, blocks, 0.0), np.arange(g.N))
        assert np.abs(res["O"] - ref).max() < 2e-5
    res64 = orc.layer_forward(q, k, v, g, 0.0, 0.0, dtype=np.float64)
    assert np.abs(res64["O"] - ref).max() < 1e-12


def _duplicated_tokens(g, rho, H, E, rng):
    """Every block filled with k distinct vectors, vector m at dst position j_m and copied to
    the src positions up to j_{m+1}-1."""
    pi, blocks = orc.temporal_reorder(g)
    xr = np.empty((H, g.N, E), dtype=np.float32)
    xr[:, :g.n_prefix] = rng.standard_normal((H, g.n_prefix, E))
    for (start, n) in blocks:
        k = orc.cluster_count(n, rho)
        d = orc.dst_positions(n, k) + [n]
        for m in range(k):
            vec = rng.standard_normal((H, 1, E))
            xr[:, start + d[m]:start + d[m + 1]] = vec
    return orc.inverse_reorder(xr, pi)


def test_merging_duplicated_tokens_leaves_outputs_unchanged():
    """With equal multiplicity for every key, merged attention equals unmerged attention."""
    g = orc.Geometry(4, 8, 8, 4, 2, n_special=0)      # blocks of 32, rho=0.75 -> k=8, 4 copies each
    rho = 0.75
    rng = np.random.default_rng(3)
    H, E = 2, 16
    q = _duplicated_tokens(g, rho, H, E, rng)
    k = _duplicated_tokens(g, rho, H, E, rng)
    v = _duplicated_tokens(g, rho, H, E, rng)          # V's copies follow their own pattern = K's
    # make V constant on K's clusters: same structure as k (same dst stride), so it already is.
    merged = orc.layer_forward(q, k, v, g, rho, rho)
    plain = orc.layer_forward(q, k, v, g, 0.0, 0.0)
    assert np.abs(merged["O"] - plain["O"]).max() < 2e-5
    pi, blocks = merged["pi"], merged["blocks"]
    for h in range(H):
        # each src matched its own copy with similarity 1
        assert np.allclose(merged["score_q"][h], 1.0, atol=1e-6)
        # merged tokens equal the originals at the dst positions
        qr = orc.reorder(q[h], pi)
        for (start, n), kk, off in zip(blocks, *orc.merged_layout(g, blocks, rho)[:2]):
            for m, j in enumerate(orc.dst_positions(n, kk)):
                assert np.allclose(merged["q_m"][h][off + m], qr[start + j], atol=1e-6)


def test_query_only_duplication_works_for_any_geometry():
    g = orc.Geometry(3, 5, 7, 4, 2)                   # specials, partial blocks
    rho = 0.6
    rng = np.random.default_rng(4)
    H, E = 2, 8
    q = _duplicated_tokens(g, rho, H, E, rng)
    k, v = (rng.standard_normal((H, g.N, E)).astype(np.float32) for _ in range(2))
    merged = orc.layer_forward(q, k, v, g, rho, 0.0)
    plain = orc.layer_forward(q, k, v, g, 0.0, 0.0)
    assert np.abs(merged["O"] - plain["O"]).max() < 2e-5


def test_unequal_multiplicity_changes_the_output():
    """No size-weighted bias (Eq. 3): with specials (multiplicity 1) next to duplicated keys
    the merged layer legitimately differs from the unmerged one."""
    g = orc.Geometry(2, 4, 4, 4, 2, n_special=5)
    rho = 0.75
    rng = np.random.default_rng(5)
    q, k, v = (_duplicated_tokens(g, rho, 1, 8, rng) for _ in range(3))
    merged = orc.layer_forward(q, k, v, g, rho, rho)
    plain = orc.layer_forward(q, k, v, g, 0.0, 0.0)
    assert np.abs(merged["O"] - plain["O"]).max() > 1e-3


def test_block_similarities_are_entries_of_the_global_matrix():
    """App. B, Prop. 1: block-wise similarity values are the global cosine matrix at the same pairs."""
    g = orc.Geometry(3, 5, 6, 4, 2)
    rho = 0.5
    (q, _, _) = _rand_qkv(g, H=1, E=16, seed=11)
    pi, blocks = orc.temporal_reorder(g)
    xr = orc.reorder(q[0], pi)
    x64 = xr.astype(np.float64)
    unit = x64 / np.linalg.norm(x64, axis=1, keepdims=True)
    W = unit @ unit.T                                         # global all-to-all cosine matrix
    assign, score, gap = orc.blockwise_tome(xr, g, blocks, rho)
    ks, offs, M = orc.merged_layout(g, blocks, rho)
    for (start, n), k, off in zip(blocks, ks, offs):
        dpos = orc.dst_positions(n, k)
        for j in range(n):
            if j in dpos:
                assert assign[start + j] == off + dpos.index(j)
                continue
            row = W[start + j, [start + d for d in dpos]]
            m = int(np.argmax(row))
            if np.sort(row)[-1] - (np.sort(row)[-2] if k > 1 else -np.inf) > 1e-5:
                assert assign[start + j] == off + m
            assert abs(score[start + j] - row.max()) < 1e-5
            if k > 1:
                assert abs(gap[start + j] - (np.sort(row)[-1] - np.sort(row)[-2])) < 1e-5


def _mean_best_similarity(xr, g, blocks, dst_set):
    """Mean over src tokens of their best cosine similarity to the dst tokens of the same block."""
    x64 = xr.astype(np.float64)
    unit = x64 / np.linalg.norm(x64, axis=1, keepdims=True)
    tot, cnt = 0.0, 0
    for (start, n) in blocks:
        idx = np.arange(start, start + n)
        d = [j for j in idx if j in dst_set]
        s = [j for j in idx if j not in dst_set]
        if not d or not s:
            continue
        tot += (unit[s] @ unit[d].T).max(axis=1).sum()
        cnt += len(s)
    return tot / cnt


def test_larger_blocks_never_lower_matching_quality():
    """App. B, Prop. 3(i): with the same src/dst sets, nested larger blocks give a mean
    best-match similarity that is at least as high."""
    small = orc.Geometry(4, 8, 8, 2, 2, n_special=0)
    large_s = orc.Geometry(4, 8, 8, 4, 2, n_special=0)     # each 4x4 window = 4 nested 2x2 windows
    large_t = orc.Geometry(4, 8, 8, 2, 4, n_special=0)     # each T=4 group = 2 nested T=2 groups
    (q, _, _) = _rand_qkv(small, H=1, E=8, seed=21)
    pi_s, blocks_s = orc.temporal_reorder(small)
    # dst set (as input indices) defined on the small blocks
    dst_inputs = set()
    for (start, n) in blocks_s:
        for j in orc.dst_positions(n, orc.cluster_count(n, 0.5)):
            dst_inputs.add(int(pi_s[start + j]))
    base = _mean_best_similarity(orc.reorder(q[0], pi_s), small, blocks_s,
                                 {j for j in range(small.N) if int(pi_s[j]) in dst_inputs})
    for g2 in (large_s, large_t):
        pi2, blocks2 = orc.temporal_reorder(g2)
        dst2 = {j for j in range(g2.N) if int(pi2[j]) in dst_inputs}
        assert _mean_best_similarity(orc.reorder(q[0], pi2), g2, blocks2, dst2) >= base - 1e-12


def test_constituents_share_bit_identical_outputs():
    """Eq. 5: every token of a merged query reads the same output row."""
    g = orc.Geometry(3, 6, 5, 4, 2)
    q, k, v = _rand_qkv(g, H=2, E=16, seed=31)
    res = orc.layer_forward(q, k, v, g, 0.7, 0.5)
    pi, blocks = res["pi"], res["blocks"]
    E = 16
    for h in range(2):
        rep = orc.rep_map(res["assign_q"][h], pi, g, blocks, 0.7)
        Oh = res["O"][:, h * E:(h + 1) * E]
        assert np.array_equal(Oh, Oh[rep])
        # a dst / special token's output is its own merged row
        inv = np.empty(g.N, dtype=np.int64)
        inv[pi] = np.arange(g.N)
        for i in np.flatnonzero(rep == np.arange(g.N)):
            assert np.array_equal(Oh[i], res["o_m"][h][res["assign_q"][h][inv[i]]])


def test_attention_is_invariant_to_key_order():
    rng = np.random.default_rng(41)
    qm, km, vm = (rng.standard_normal((50, 16)).astype(np.float32) for _ in range(3))
    perm = rng.permutation(50)
    a = orc.attention(qm, km, vm)
    b = orc.attention(qm, km[perm], vm[perm])
    assert np.abs(a - b).max() < 1e-5
    # and rows are independent: a subset of rows is exact
    rows = np.array([3, 17, 49])
    assert np.array_equal(orc.attention(qm, km, vm, rows=rows), a[rows])
    assert np.allclose(orc.attention(qm, km, vm, chunk=7), a, atol=1e-6)


def test_uniform_variant_with_identical_heads_equals_headwise():
    g = orc.Geometry(2, 6, 6, 4, 2)
    rng = np.random.default_rng(51)
    one = [rng.standard_normal((1, g.N, 16)).astype(np.float32) for _ in range(3)]
    q, k, v = (np.repeat(t, 4, axis=0) for t in one)      # power-of-two head count: mean is exact
    a = orc.layer_forward(q, k, v, g, 0.5, 0.75, variant="headwise")
    b = orc.layer_forward(q, k, v, g, 0.5, 0.75, variant="uniform")
    for h in range(4):
        assert np.array_equal(a["assign_q"][h], b["assign_q"][h])
        assert np.array_equal(a["assign_k"][h], b["assign_k"][h])
    assert np.array_equal(a["O"], b["O"])


def test_uniform_variant_shares_one_topology_and_differs_from_headwise():
    g = orc.Geometry(2, 8, 8, 4, 2)
    q, k, v = _rand_qkv(g, H=4, E=16, seed=61)
    u = orc.layer_forward(q, k, v, g, 0.5, 0.5, variant="uniform")
    hw = orc.layer_forward(q, k, v, g, 0.5, 0.5, variant="headwise")
    for h in range(1, 4):
        assert np.array_equal(u["assign_q"][0], u["assign_q"][h])
    assert any(not np.array_equal(hw["assign_q"][0], hw["assign_q"][h]) for h in range(1, 4))
    # the shared topology is the matching of the head-averaged tokens
    pi, blocks = u["pi"], u["blocks"]
    mean_q = q.astype(np.float64).mean(axis=0).astype(np.float32)
    a, _, _ = orc.blockwise_tome(orc.reorder(mean_q, pi), g, blocks, 0.5)
    assert (a != u["assign_q"][0]).mean() < 0.01


def test_exact_ties_go_to_the_lowest_cluster_and_zero_vectors_are_safe():
    xb = np.zeros((6, 4), dtype=np.float32)
    xb[0] = [1, 0, 0, 0]
    xb[3] = [1, 0, 0, 0]          # k=2 -> dst at positions 0 and 3, identical
    xb[1] = [2, 0, 0, 0]
    xb[2] = [0, 0, 0, 0]          # zero vector: similarity 0 to everything
    xb[4] = [3, 1, 0, 0]
    xb[5] = [-1, 0, 0, 0]
    cluster, score, gap = orc.match_block(xb, 2)
    assert cluster.tolist() == [0, 0, 0, 1, 0, 0]
    assert np.isfinite(score).all()
    assert gap[1] == 0.0 and gap[2] == 0.0
    assert score[2] == 0.0 and abs(score[5] + 1.0) < 1e-6


def test_mean_uses_raw_tokens_and_v_follows_k():
    g = orc.Geometry(1, 2, 2, 2, 1, n_special=0)          # one block of 4 tokens
    blocks = [(0, 4)]
    kr = np.array([[1, 0], [10, 0.1], [0, 1], [0.1, 7]], dtype=np.float32)   # k=2: dst at 0 and 2
    vr = np.array([[1, 1], [2, 2], [30, 30], [40, 40]], dtype=np.float32)
    ak, _, _ = orc.blockwise_tome(kr, g, blocks, 0.5)
    assert ak.tolist() == [0, 0, 1, 1]
    km = orc.block_aggregate(kr, ak, g, blocks, 0.5)
    vm = orc.block_aggregate(vr, ak, g, blocks, 0.5)
    assert np.allclose(km, [[5.5, 0.05], [0.05, 4.0]])     # raw mean, not mean of unit vectors
    assert np.allclose(vm, [[1.5, 1.5], [35, 35]])
