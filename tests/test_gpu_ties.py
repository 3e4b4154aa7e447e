"""Exact similarity ties and zero vectors (Eq. 1 and the best-match rule: the lowest cluster wins) on
every matching kernel instance: 32-, 256- and 512-token blocks (1-, 4- and 8-wave workgroups) and
3840-token blocks (the tiled matcher with its keyed arg-max), in Q and in K (V follows K).

Tokens are iid Gaussian vectors (best-vs-second gaps of about 1e-2; a handful per head lie inside
fp32 summation noise, below 1e-5, and only those may differ), so every exact tie is a planted one or
follows from one, and all of them must be resolved as the oracle resolves them:
  * dst m2 is an exact copy of dst m1 < m2, and a src token is a third copy: it ties between the two
    at the maximum (similarity 1) and must join m1.  The pairs are chosen so that the two dst sit in
    one group of accumulator registers, in the two lane halves of an MFMA tile, in different
    32-dst steps and in different 64-dst tiles;
  * an all-zero src token has similarity 0 to every dst: an all-way tie that cluster 0 wins;
  * an all-zero dst token has similarity 0 to every src: src tokens whose other similarities are all
    negative join it - decided identically on both sides.
"""
import numpy as np
import pytest
import torch

import paper_2511_21317_amd as httm
from oracle import httm_oracle as orc
from synth.vggt_tokens import Workload

from gpu_util import check_output, f32, oracle_geom, plan_for, require_gpu, run_stages

pytestmark = pytest.mark.gpu

# (m1, m2): cluster indices of the duplicated dst tokens, used when the block keeps more than m2 clusters
PAIRS = [(0, 1), (2, 6), (3, 35), (5, 70), (9, 200), (10, 300), (12, 1100)]
ZERO_DST = 40      # cluster whose dst token is zeroed (when the block keeps that many)

CASES = [
    # name, index, S, Hp, Wp, b, T, rho_q, shift; rho_kv
    (Workload("ties_block32", 41, 4, 8, 8, 4, 2, 0.75, 1, H=2), 0.5),
    (Workload("ties_block256", 42, 4, 16, 16, 8, 4, 0.6, 1, H=2), 0.3),                        # k = 103 / 180
    (Workload("ties_block512", 43, 8, 16, 16, 8, 8, 0.75, 1, H=2), 0.4),                       # k = 128 / 308
    (Workload("ties_block3840", 44, 30, 16, 16, 128, 30, 0.9, 1, H=2, chunked=True), 0.7),     # k = 384 / 1152
]


def _plant(x, g, pi, blocks, rho):
    """x: [H, N, 64] float32 in input order, modified in place.  Returns the reordered positions of
    the planted tie tokens and zero tokens."""
    tied, zeros = [], []
    for (start, n), n0 in zip(blocks, orc.anchor_sizes(g)):
        k = orc.cluster_count(n, rho, n0)
        d = orc.dst_positions(n, k, n0)
        dset = set(d)
        free = [j for j in range(n) if j not in dset]          # src positions, ascending
        if len(free) < 4:
            continue
        used = 0
        for m1, m2 in PAIRS:
            if m2 >= k or used + 1 >= len(free) - 2:
                continue
            x[:, pi[start + d[m2]]] = x[:, pi[start + d[m1]]]
            # the src copy goes to a src position behind dst m2, so that it is not next to dst m1
            cand = [j for j in free if j > d[m2]] or free
            j = cand[used % len(cand)]
            while (start + j) in tied:
                j = free[(free.index(j) + 1) % len(free)]
            x[:, pi[start + j]] = x[:, pi[start + d[m1]]]
            tied.append(start + j)
            used += 1
        # an all-zero src token: the last free position that carries no copy
        for j in reversed(free):
            if (start + j) not in tied:
                x[:, pi[start + j]] = 0.0
                zeros.append(start + j)
                break
        if k > ZERO_DST + 1:
            x[:, pi[start + d[ZERO_DST]]] = 0.0
    return np.asarray(tied), np.asarray(zeros)


@pytest.mark.parametrize("w,rho_kv", CASES, ids=lambda c: c.name if isinstance(c, Workload) else str(c))
def test_exact_ties_and_zero_vectors_follow_the_lowest_cluster_rule(w, rho_kv):
    require_gpu()
    print(f"[case] {w.name} N={w.N} rho_q={w.rho} rho_kv={rho_kv}", flush=True)
    g = oracle_geom(w)
    pi, blocks = orc.temporal_reorder(g)
    gen = torch.Generator().manual_seed(9000 + w.index)
    q, k, v = (torch.randn((w.H, w.N, 64), generator=gen).to(torch.bfloat16).float().numpy() for _ in range(3))
    tied_q, zero_q = _plant(q, g, pi, blocks, w.rho)
    tied_k, zero_k = _plant(k, g, pi, blocks, rho_kv)
    assert tied_q.size and tied_k.size and zero_q.size and zero_k.size
    q, k, v = (torch.from_numpy(t).to(torch.bfloat16).cuda() for t in (q, k, v))
    plan = plan_for(w, rho_kv=rho_kv)
    got = run_stages(plan, q, k, v)
    ref = orc.layer_forward(f32(q), f32(k), f32(v), g, w.rho, rho_kv)
    n_exact = 0
    for h in range(w.H):
        for name, gap, tied, zeros in (("assign_q", "gap_q", tied_q, zero_q), ("assign_k", "gap_k", tied_k, zero_k)):
            a = got[name][h].cpu().numpy()
            # the planted tokens are exact ties in the oracle: this is what the case is about
            assert (ref[gap][h][tied] == 0).all() and (ref[gap][h][zeros] == 0).all(), name
            assert np.array_equal(a[tied], ref[name][h][tied]), f"{w.name} {name} head {h}: a planted tie went wrong"
            assert np.array_equal(a[zeros], ref[name][h][zeros]), f"{w.name} {name} head {h}: a zero row went wrong"
            # every exact tie (planted, or induced: a src that prefers a duplicated dst) and every clear
            # decision equal; only a gap inside fp32 summation noise (0 < gap < 1e-5, a handful of
            # tokens at most, a hundred times tighter than the acceptance bar) may go either way
            bad = np.flatnonzero(a != ref[name][h])
            gp = ref[gap][h][bad]
            assert ((gp > 0) & (gp < 1e-5)).all() and bad.size <= 4, (
                f"{w.name} {name} head {h}: {bad.size} indices differ, first at {bad[:5]}, gap {gp[:5]}")
            n_exact += int((ref[gap][h] == 0).sum())
        # merged rows: one bf16 rounding from the oracle's fp32 mean (clusters of equal membership)
        for name, asg in (("q_m", "assign_q"), ("k_m", "assign_k"), ("v_m", "assign_k")):
            if np.array_equal(got[asg][h].cpu().numpy(), ref[asg][h]):
                mean = ref[name][h] * (got["key_scale"] if name == "k_m" else np.float32(1.0))
                assert (np.abs(f32(got[name][h]) - mean) <= 2.0 ** -8 * np.abs(mean) + 1e-30).all(), (name, h)
    print(f"{w.name}: {n_exact} exact ties resolved as the oracle resolves them", flush=True)
    if all(np.array_equal(got[a][h].cpu().numpy(), ref[a][h]) for a in ("assign_q", "assign_k") for h in range(w.H)):
        check_output(f32(got["out"]), ref["O"], f"{w.name} layer output", relative_to_magnitude=True)
    out = torch.empty_like(got["out"])
    httm.layer_forward(plan, q, k, v, out, httm.alloc_workspace(plan))
    torch.cuda.synchronize()
    assert torch.equal(out, got["out"])
    plan.close()


TOPR_CASES = [
    Workload("topr_ties_block256", 45, 4, 16, 16, 8, 4, 0.5, 1, H=2, dst_frac=0.25),     # kd = 64, r = 128 of 192 src
    Workload("topr_ties_block512", 46, 8, 16, 16, 8, 8, 0.5, 1, H=2, dst_frac=0.25),     # kd = 128, r = 256 of 384 src
    Workload("topr_ties_block3840", 47, 30, 16, 16, 128, 30, 0.5, 1, H=2, chunked=True, dst_frac=0.25),   # kd = 960, r = 1920 of 2880
]


@pytest.mark.parametrize("w", TOPR_CASES, ids=lambda w: w.name)
def test_top_r_selection_breaks_ties_at_its_boundary_by_position(w):
    """General rule of Sec. 3.2: only the r src tokens with the highest best similarity merge.  Here
    more than r src tokens of every block are exact copies of one dst token (similarity 1, the
    highest there is), so the selection boundary falls inside a group of equal scores: the copies at
    the lowest positions merge, the others stay clusters of their own."""
    require_gpu()
    print(f"[case] {w.name} N={w.N}", flush=True)
    g = oracle_geom(w)
    pi, blocks = orc.temporal_reorder(g)
    gen = torch.Generator().manual_seed(9000 + w.index)
    q, k, v = (torch.randn((w.H, w.N, 64), generator=gen).to(torch.bfloat16).float().numpy() for _ in range(3))
    n_copies = {}
    for x in (q, k):
        for (start, n) in blocks:
            kd = orc.dst_count(n, w.rho, 0, w.dst_frac)
            r = n - orc.cluster_count(n, w.rho, 0, w.dst_frac)
            d = orc.dst_positions(n, kd, 0)
            dset = set(d)
            free = [j for j in range(n) if j not in dset]
            copies = free[3::1][: r + (len(free) - r) // 2]          # more than r of them, not all
            for j in copies:
                x[:, pi[start + j]] = x[:, pi[start + d[3]]]
            n_copies[start] = (len(copies), r)
    assert all(c > r > 0 for c, r in n_copies.values())
    q, k, v = (torch.from_numpy(t).to(torch.bfloat16).cuda() for t in (q, k, v))
    plan = plan_for(w)
    got = run_stages(plan, q, k, v)
    ref = orc.layer_forward(f32(q), f32(k), f32(v), g, w.rho, w.rho)
    for h in range(w.H):
        for name in ("assign_q", "assign_k"):
            a = got[name][h].cpu().numpy()
            bad = np.flatnonzero(a != ref[name][h])
            assert bad.size == 0, f"{w.name} {name} head {h}: {bad.size} indices differ, first at {bad[:5]}"
    check_output(f32(got["out"]), ref["O"], f"{w.name} layer output", relative_to_magnitude=True)
    plan.close()
