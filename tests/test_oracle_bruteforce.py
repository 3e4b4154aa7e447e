"""Brute force on tiny inputs: a literal pure-Python float64 re-statement of the layer,
built from the paper's definitions with none of the oracle's code, must agree with the oracle.

The brute force works in INPUT coordinates throughout (it never reorders anything): blocks are
sets of tokens, a src token merges into the most similar dst token of its block (Eq. 1), merged
tokens are means (Sec. 3.2), attention is Eq. 3-4 over the set of merged tokens, and each input
token reads the output of the merged token that contains it (Eq. 5)."""
import math

import numpy as np
import pytest

from oracle import httm_oracle as orc


def _dot(a, b):
    return math.fsum(x * y for x, y in zip(a, b))


def _cos(a, b):
    return _dot(a, b) / (max(math.sqrt(_dot(a, a)), 1e-12) * max(math.sqrt(_dot(b, b)), 1e-12))


def _blocks_bruteforce(S, Hp, Wp, b, T, n_special, chunked=False):
    """Token sets per block, each listed in (frame, row, col) order, blocks in (group,by,bx) order.
    chunked: a spatial block is a run of b consecutive patch tokens of the frame (Sec. 4.1, n_s)
    instead of a b x b window."""
    tpf = n_special + Hp * Wp
    groups = {}
    for f in range(S):
        for y in range(Hp):
            for x in range(Wp):
                key = (f // T, (y * Wp + x) // b, 0) if chunked else (f // T, y // b, x // b)
                groups.setdefault(key, []).append(f * tpf + n_special + y * Wp + x)
    specials = [f * tpf + s for f in range(S) for s in range(n_special)]
    return specials, [groups[key] for key in sorted(groups)]


def _merge_head(x, specials, blocks, rho, anchor_below=0, dst_frac=0.0):
    """x: list of N vectors.  Returns (clusters, owner): clusters = list of member lists (input
    indices, dst first), in merged order; owner[i] = index into clusters for input token i.
    Tokens with input index < anchor_below (= the tokens of frame 0 under first-frame anchoring,
    App. C.2) are always dst; the other dst are strided over the rest of the block.
    dst_frac > 0: the general rule of Sec. 3.2 - that share of the block are dst, and only the r src
    tokens with the highest best-match similarity merge (ties: earlier token first)."""
    clusters = [[i] for i in specials]
    owner = {i: c for c, i in enumerate(specials)}
    for toks in blocks:
        n = len(toks)
        anchored = [p for p, i in enumerate(toks) if i < anchor_below]
        others = [p for p, i in enumerate(toks) if i >= anchor_below]
        r = int(math.floor(rho * n + 1e-9))
        if dst_frac > 0.0:
            kd = max(1, int(math.floor(dst_frac * n + 1e-9)), len(anchored))
            r = min(r, n - kd)
        else:
            kd = max(1, n - r, len(anchored))
            r = n - kd
        free = kd - len(anchored)
        dpos = anchored + [others[(m * len(others)) // free] for m in range(free)]
        base = len(clusters)
        for m, p in enumerate(dpos):
            clusters.append([toks[p]])
            owner[toks[p]] = base + m
        matches = []                                   # (score, position, best cluster) of every src token
        for p, i in enumerate(toks):
            if p in dpos:
                continue
            best_m, best_s = 0, -float("inf")
            for m, dp in enumerate(dpos):
                s = _cos(x[i], x[toks[dp]])
                if s > best_s:                       # strict: lowest m wins exact ties
                    best_m, best_s = m, s
            matches.append((best_s, p, best_m))
        chosen = {p for _, p, _ in sorted(matches, key=lambda t: (-t[0], t[1]))[:r]}
        for s_, p, m in matches:                       # in ascending position
            if p in chosen:
                clusters[base + m].append(toks[p])
                owner[toks[p]] = base + m
            else:
                owner[toks[p]] = len(clusters)
                clusters.append([toks[p]])
    return clusters, owner


def _mean(vectors):
    E = len(vectors[0])
    return [math.fsum(v[c] for v in vectors) / len(vectors) for c in range(E)]


def _layer_bruteforce(q, k, v, S, Hp, Wp, b, T, n_special, rho_q, rho_kv, anchor=False, chunked=False,
                      dst_frac=0.0):
    H, N, E = q.shape
    specials, blocks = _blocks_bruteforce(S, Hp, Wp, b, T, n_special, chunked)
    anchor_below = (n_special + Hp * Wp) if anchor else 0      # input indices of frame 0
    out = np.zeros((N, H * E))
    owners_q, owners_k = [], []
    for h in range(H):
        qh, kh, vh = q[h].tolist(), k[h].tolist(), v[h].tolist()
        cq, own_q = _merge_head(qh, specials, blocks, rho_q, anchor_below, dst_frac)
        ck, own_k = _merge_head(kh, specials, blocks, rho_kv, anchor_below, dst_frac)
        qm = [_mean([qh[i] for i in mem]) for mem in cq]
        km = [_mean([kh[i] for i in mem]) for mem in ck]
        vm = [_mean([vh[i] for i in mem]) for mem in ck]      # V follows K's matches
        om = []
        for qrow in qm:
            logit = [_dot(qrow, krow) / math.sqrt(E) for krow in km]
            mx = max(logit)
            w = [math.exp(l - mx) for l in logit]
            z = math.fsum(w)
            om.append([math.fsum(wj * vrow[c] for wj, vrow in zip(w, vm)) / z for c in range(E)])
        for i in range(N):
            out[i, h * E:(h + 1) * E] = om[own_q[i]]
        owners_q.append([cq[own_q[i]][0] for i in range(N)])   # representative = the dst token
        owners_k.append([ck[own_k[i]][0] for i in range(N)])
    return out, np.array(owners_q), np.array(owners_k)


CASES = [
    # S, Hp, Wp, b, T, n_special, rho_q, rho_kv
    (3, 3, 4, 2, 2, 5, 0.5, 0.5),
    (2, 4, 4, 2, 2, 5, 0.75, 0.5),
    (4, 3, 3, 2, 3, 1, 0.6, 0.8),
    (2, 5, 2, 4, 1, 0, 0.5, 0.0),
    (3, 2, 6, 3, 4, 2, 0.9, 0.34),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_oracle_equals_bruteforce(case, dtype):
    S, Hp, Wp, b, T, nsp, rho_q, rho_kv = case
    g = orc.Geometry(S, Hp, Wp, b, T, n_special=nsp)
    H, E = 2, 8
    rng = np.random.default_rng(1234 + S * 100 + Hp * 10 + Wp)
    q, k, v = (rng.standard_normal((H, g.N, E)) for _ in range(3))
    ref_out, ref_rep_q, ref_rep_k = _layer_bruteforce(q, k, v, S, Hp, Wp, b, T, nsp, rho_q, rho_kv)

    res = orc.layer_forward(q, k, v, g, rho_q, rho_kv, dtype=dtype)
    pi, blocks = res["pi"], res["blocks"]
    for h in range(H):
        assert np.array_equal(orc.rep_map(res["assign_q"][h], pi, g, blocks, rho_q), ref_rep_q[h])
        assert np.array_equal(orc.rep_map(res["assign_k"][h], pi, g, blocks, rho_kv), ref_rep_k[h])
    tol = 1e-5 if dtype == np.float32 else 1e-12
    assert np.abs(res["O"] - ref_out).max() < tol


CHUNKED = [
    # S, Hp, Wp, n_s, n_t, n_special, rho_q, rho_kv: spatial blocks are runs of n_s tokens (Sec. 4.1)
    (3, 3, 4, 5, 2, 5, 0.5, 0.5),        # 12 patch tokens in runs of 5, 5, 2
    (4, 3, 3, 4, 3, 1, 0.9, 0.7),
    (5, 2, 5, 10, 4, 0, 0.75, 0.3),      # one run = the whole frame
    (2, 4, 4, 7, 1, 2, 0.6, 0.6),        # n_t = 1: purely spatial blocks
]


@pytest.mark.parametrize("anchor", [False, True])
@pytest.mark.parametrize("case", CHUNKED)
def test_oracle_equals_bruteforce_with_chunked_blocks(case, anchor):
    S, Hp, Wp, b, T, nsp, rho_q, rho_kv = case
    g = orc.Geometry(S, Hp, Wp, b, T, n_special=nsp, anchor=anchor, chunked=True)
    H, E = 2, 8
    rng = np.random.default_rng(777 + S * 100 + Hp * 10 + Wp)
    q, k, v = (rng.standard_normal((H, g.N, E)) for _ in range(3))
    ref_out, ref_rep_q, ref_rep_k = _layer_bruteforce(q, k, v, S, Hp, Wp, b, T, nsp, rho_q, rho_kv,
                                                      anchor=anchor, chunked=True)
    res = orc.layer_forward(q, k, v, g, rho_q, rho_kv, dtype=np.float64)
    pi, blocks = res["pi"], res["blocks"]
    for h in range(H):
        assert np.array_equal(orc.rep_map(res["assign_q"][h], pi, g, blocks, rho_q), ref_rep_q[h])
        assert np.array_equal(orc.rep_map(res["assign_k"][h], pi, g, blocks, rho_kv), ref_rep_k[h])
    assert np.abs(res["O"] - ref_out).max() < 1e-12


TOP_R = [
    # S, Hp, Wp, b, T, n_special, rho_q, rho_kv, dst_frac, anchor, chunked
    (3, 3, 4, 2, 2, 5, 0.5, 0.5, 0.25, False, False),
    (4, 4, 4, 2, 3, 1, 0.6, 0.3, 0.25, False, False),
    (2, 4, 4, 4, 2, 0, 0.9, 0.9, 0.25, False, False),      # the ratio asks for more than there are src
    (3, 2, 6, 5, 3, 2, 0.4, 0.7, 0.5, False, True),
    (4, 3, 3, 2, 2, 2, 0.5, 0.5, 0.25, True, False),       # with first-frame anchoring
    (3, 3, 4, 2, 2, 5, 0.0, 0.5, 0.25, False, False),      # queries not merged at all
]


@pytest.mark.parametrize("case", TOP_R)
def test_oracle_equals_bruteforce_with_top_r_selection(case):
    """Sec. 3.2 as written: a fixed share of dst tokens, and only the r most similar src merge."""
    S, Hp, Wp, b, T, nsp, rho_q, rho_kv, dst_frac, anchor, chunked = case
    g = orc.Geometry(S, Hp, Wp, b, T, n_special=nsp, anchor=anchor, chunked=chunked, dst_frac=dst_frac)
    H, E = 2, 8
    rng = np.random.default_rng(31 + S * 100 + Hp * 10 + Wp)
    q, k, v = (rng.standard_normal((H, g.N, E)) for _ in range(3))
    ref_out, ref_rep_q, ref_rep_k = _layer_bruteforce(q, k, v, S, Hp, Wp, b, T, nsp, rho_q, rho_kv,
                                                      anchor=anchor, chunked=chunked, dst_frac=dst_frac)
    res = orc.layer_forward(q, k, v, g, rho_q, rho_kv, dtype=np.float64)
    pi, blocks = res["pi"], res["blocks"]
    for h in range(H):
        assert np.array_equal(orc.rep_map(res["assign_q"][h], pi, g, blocks, rho_q), ref_rep_q[h])
        assert np.array_equal(orc.rep_map(res["assign_k"][h], pi, g, blocks, rho_kv), ref_rep_k[h])
    assert np.abs(res["O"] - ref_out).max() < 1e-12
    # sizes: a block of n tokens keeps n - min(floor(rho n), n - kd)
    ks, _, M = orc.merged_layout(g, blocks, rho_q)
    kds = orc.dst_counts(g, blocks, rho_q)
    for (_, n), k_, kd in zip(blocks, ks, kds):
        assert k_ == n - min(int(math.floor(rho_q * n + 1e-9)), n - kd) and 1 <= kd <= k_
    assert res["q_m"][0].shape[0] == M


def test_top_r_rule_reduces_to_alg1_when_every_src_merges():
    """With dst_frac = 1 - rho (and no rounding trouble) the two rules describe the same partition."""
    g0 = orc.Geometry(2, 4, 4, 2, 2)
    g1 = orc.Geometry(2, 4, 4, 2, 2, dst_frac=0.25)
    rng = np.random.default_rng(3)
    q, k, v = (rng.standard_normal((2, g0.N, 8)) for _ in range(3))
    a = orc.layer_forward(q, k, v, g0, 0.75, 0.75, dtype=np.float64)
    b_ = orc.layer_forward(q, k, v, g1, 0.75, 0.75, dtype=np.float64)
    assert np.array_equal(a["O"], b_["O"]) and all(np.array_equal(x, y) for x, y in zip(a["assign_q"], b_["assign_q"]))


ANCHORED = [
    (3, 3, 4, 2, 2, 5, 0.5, 0.5),
    (4, 3, 3, 2, 3, 1, 0.6, 0.8),
    (2, 4, 4, 2, 2, 5, 0.9, 0.9),    # the ratio asks for fewer clusters than frame 0 has tokens
    (5, 2, 5, 3, 4, 0, 0.75, 0.3),
    (1, 3, 3, 2, 2, 2, 0.5, 0.5),    # a single frame: every token is anchored, nothing merges
]


@pytest.mark.parametrize("case", ANCHORED)
def test_oracle_equals_bruteforce_with_first_frame_anchoring(case):
    """App. C.2: all frame-0 tokens are dst.  The brute force decides "frame 0" from the input
    index; the oracle from the position inside the reordered block."""
    S, Hp, Wp, b, T, nsp, rho_q, rho_kv = case
    g = orc.Geometry(S, Hp, Wp, b, T, n_special=nsp, anchor=True)
    H, E = 2, 8
    rng = np.random.default_rng(4321 + S * 100 + Hp * 10 + Wp)
    q, k, v = (rng.standard_normal((H, g.N, E)) for _ in range(3))
    ref_out, ref_rep_q, ref_rep_k = _layer_bruteforce(q, k, v, S, Hp, Wp, b, T, nsp, rho_q, rho_kv,
                                                      anchor=True)
    res = orc.layer_forward(q, k, v, g, rho_q, rho_kv, dtype=np.float64)
    pi, blocks = res["pi"], res["blocks"]
    tpf = nsp + Hp * Wp
    for h in range(H):
        rq = orc.rep_map(res["assign_q"][h], pi, g, blocks, rho_q)
        assert np.array_equal(rq, ref_rep_q[h])
        assert np.array_equal(orc.rep_map(res["assign_k"][h], pi, g, blocks, rho_kv), ref_rep_k[h])
        assert np.array_equal(rq[:tpf], np.arange(tpf))       # frame 0 is never merged away
    assert np.abs(res["O"] - ref_out).max() < 1e-12
    # anchoring is not a no-op on these cases (except the single-frame one)
    plain = orc.layer_forward(q, k, v, orc.Geometry(S, Hp, Wp, b, T, n_special=nsp), rho_q, rho_kv,
                              dtype=np.float64)
    if S > 1:
        assert np.abs(plain["O"] - res["O"]).max() > 1e-6


def test_bruteforce_catches_a_transposed_or_dropped_term():
    """The pin is sensitive: planting typical mistakes in a copy of the oracle's steps changes O."""
    g = orc.Geometry(2, 4, 4, 2, 2)
    rng = np.random.default_rng(7)
    q, k, v = (rng.standard_normal((2, g.N, 8)) for _ in range(3))
    ref_out, _, _ = _layer_bruteforce(q, k, v, 2, 4, 4, 2, 2, 5, 0.5, 0.5)
    good = orc.layer_forward(q, k, v, g, 0.5, 0.5, dtype=np.float64)["O"]
    assert np.abs(good - ref_out).max() < 1e-12
    # V merged with its own matches instead of K's -> must differ
    pi, blocks = orc.temporal_reorder(g)
    h = 0
    qr, kr, vr = (orc.reorder(t[h], pi) for t in (q, k, v))
    aq, _, _ = orc.blockwise_tome(qr, g, blocks, 0.5)
    ak, _, _ = orc.blockwise_tome(kr, g, blocks, 0.5)
    av, _, _ = orc.blockwise_tome(vr, g, blocks, 0.5)
    qm = orc.block_aggregate(qr, aq, g, blocks, 0.5)
    km = orc.block_aggregate(kr, ak, g, blocks, 0.5)
    vm_wrong = orc.block_aggregate(vr, av, g, blocks, 0.5)
    o_wrong = orc.inverse_reorder(orc.unmerge_by_cluster(orc.attention(qm, km, vm_wrong), aq), pi)
    assert np.abs(o_wrong - ref_out[:, :8]).max() > 1e-3
    # unmerging with K's assignment instead of Q's -> must differ
    vm = orc.block_aggregate(vr, ak, g, blocks, 0.5)
    o_wrong2 = orc.inverse_reorder(orc.unmerge_by_cluster(orc.attention(qm, km, vm), ak), pi)
    assert np.abs(o_wrong2 - ref_out[:, :8]).max() > 1e-3
