"""Pins of the oracle's adaptive outlier filtering (Sec. 3.4, Alg. 2; Alg. 1's second attention).

A pure-Python float64 brute force in INPUT coordinates that shares no code with the oracle
(member lists, math.fsum), small hand-worked thresholds, and the properties Sec. 3.4 states."""
import math

import numpy as np
import pytest

from oracle import httm_oracle as orc
from test_oracle_bruteforce import _blocks_bruteforce, _dot, _mean, _merge_head


def _attend(qrow, km, vm, E):
    logit = [_dot(qrow, krow) / math.sqrt(E) for krow in km]
    mx = max(logit)
    w = [math.exp(l - mx) for l in logit]
    z = math.fsum(w)
    return [math.fsum(wj * vrow[c] for wj, vrow in zip(w, vm)) / z for c in range(E)]


def _layer_bruteforce_filtered(q, k, v, S, Hp, Wp, b, T, n_special, rho_q, rho_kv, frac):
    H, N, E = q.shape
    specials, blocks = _blocks_bruteforce(S, Hp, Wp, b, T, n_special)
    heads = []
    devs = []                                     # (deviation, head, token) of every token
    for h in range(H):
        qh, kh, vh = q[h].tolist(), k[h].tolist(), v[h].tolist()
        cq, own_q = _merge_head(qh, specials, blocks, rho_q)
        ck, _ = _merge_head(kh, specials, blocks, rho_kv)
        km = [_mean([kh[i] for i in mem]) for mem in ck]
        vm = [_mean([vh[i] for i in mem]) for mem in ck]
        for mem in cq:
            mu = _mean([qh[i] for i in mem])
            for i in mem:
                d = math.sqrt(math.fsum((a - m) ** 2 for a, m in zip(qh[i], mu))) if len(mem) > 1 else 0.0
                devs.append((d, h, i))
        heads.append((qh, cq, own_q, km, vm))
    budget = int(math.floor(frac * H * N + 1e-9))
    ranked = sorted(devs, key=lambda t: -t[0])
    tau = ranked[budget][0] if budget < len(ranked) else -math.inf     # largest value outside the budget
    outliers = {(h, i) for d, h, i in devs if d > tau}
    out = np.zeros((N, H * E))
    for h, (qh, cq, own_q, km, vm) in enumerate(heads):
        om = []
        for mem in cq:
            rest = [i for i in mem if (h, i) not in outliers]
            om.append(_attend(_mean([qh[i] for i in rest]), km, vm, E) if rest else None)
        for i in range(N):
            row = _attend(qh[i], km, vm, E) if (h, i) in outliers else om[own_q[i]]
            out[i, h * E:(h + 1) * E] = row
    return out, outliers, tau


CASES = [
    # S, Hp, Wp, b, T, n_special, rho_q, rho_kv, outlier fraction
    (3, 3, 4, 2, 2, 5, 0.5, 0.5, 0.10),
    (2, 4, 4, 2, 2, 5, 0.75, 0.5, 0.05),
    (4, 3, 3, 2, 3, 1, 0.6, 0.8, 0.25),
    (3, 2, 6, 3, 4, 2, 0.9, 0.34, 0.15),
    (2, 4, 4, 4, 2, 0, 0.9, 0.5, 0.5),      # so many outliers that whole clusters dissolve
]


@pytest.mark.parametrize("case", CASES)
def test_filtered_layer_equals_bruteforce(case):
    S, Hp, Wp, b, T, nsp, rho_q, rho_kv, frac = case
    g = orc.Geometry(S, Hp, Wp, b, T, n_special=nsp)
    H, E = 3, 8
    rng = np.random.default_rng(99 + S * 100 + Hp * 10 + Wp)
    q, k, v = (rng.standard_normal((H, g.N, E)) for _ in range(3))
    ref_out, ref_outliers, ref_tau = _layer_bruteforce_filtered(q, k, v, S, Hp, Wp, b, T, nsp, rho_q,
                                                                rho_kv, frac)
    res = orc.layer_forward(q, k, v, g, rho_q, rho_kv, dtype=np.float64, outlier_frac=frac)
    pi = res["pi"]
    got = {(h, int(pi[j])) for h in range(H) for j in np.flatnonzero(res["outlier_mask"][h])}
    assert got == ref_outliers
    assert abs(res["tau"] - ref_tau) < 1e-12
    assert np.abs(res["O"] - ref_out).max() < 1e-12
    budget = int(math.floor(frac * H * g.N + 1e-9))
    mergeable = sum(int((e > 0).sum()) for e in res["eps"])
    assert len(got) == min(budget, mergeable)     # continuous random data: no ties, budget used in full


def test_threshold_is_an_order_statistic_and_ties_stay_inside_the_budget():
    eps = np.array([3.0, 9.0, 0.0, 7.0, 1.0, 8.0, 2.0, 6.0, 4.0, 5.0])
    assert orc.outlier_budget(10, 0.3) == 3
    tau = orc.outlier_threshold(eps, 0.3)
    assert tau == 6.0 and sorted(eps[eps > tau]) == [7.0, 8.0, 9.0]
    assert orc.outlier_threshold(eps, 0.0) == 9.0 and not (eps > 9.0).any()
    assert orc.outlier_threshold(eps, 0.09) == 9.0                    # budget rounds down to 0
    tied = np.array([1.0, 1.0, 1.0, 5.0, 5.0, 5.0])
    tau = orc.outlier_threshold(tied, 0.34)                            # budget 2, three values tie
    assert tau == 5.0 and int((tied > tau).sum()) == 0
    assert orc.outlier_threshold(tied, 0.5) == 1.0 and int((tied > 1.0).sum()) == 3


def test_filter_properties():
    g = orc.Geometry(4, 6, 5, 2, 2)
    H, E = 4, 16
    rng = np.random.default_rng(5)
    q, k, v = (rng.standard_normal((H, g.N, E)).astype(np.float32) for _ in range(3))
    q[2] *= 3.0                                   # one head with larger deviations takes more of the budget
    plain = orc.layer_forward(q, k, v, g, 0.5, 0.5)
    same = orc.layer_forward(q, k, v, g, 0.5, 0.5, outlier_frac=1e-9)   # budget 0
    assert np.array_equal(plain["O"], same["O"]) and not any(m.any() for m in same["outlier_mask"])
    res = orc.layer_forward(q, k, v, g, 0.5, 0.5, outlier_frac=0.1)
    counts = [int(m.sum()) for m in res["outlier_mask"]]
    assert sum(counts) == orc.outlier_budget(H * g.N, 0.1)
    assert counts[2] > max(counts[0], counts[1], counts[3])             # shared budget, Sec. 3.4 step 3
    pi, blocks = res["pi"], res["blocks"]
    for h in range(H):
        aq, mask, eps = res["assign_q"][h], res["outlier_mask"][h], res["eps"][h]
        size = np.bincount(aq, minlength=res["q_m"][h].shape[0])
        assert (eps[size[aq] == 1] == 0).all() and not mask[size[aq] == 1].any()   # unmerged: deviation 0
        assert not mask[:g.n_prefix].any()                                          # specials never merge
        # clusters without outliers keep their merged token bit for bit; the others are the mean of the rest
        touched = np.zeros(size.shape, dtype=bool)
        touched[aq[mask]] = True
        assert np.array_equal(res["q_m"][h][~touched], plain["q_m"][h][~touched])
        qr = orc.reorder(q[h], pi)
        for slot in np.flatnonzero(touched)[:20]:
            rest = np.flatnonzero((aq == slot) & ~mask)
            if rest.size:
                assert np.allclose(res["q_m"][h][slot], qr[rest].mean(axis=0), atol=1e-5)
        # an outlier's output row is plain attention of its own query over the merged keys/values
        o_r = orc.reorder(res["O"][:, h * E:(h + 1) * E], pi)
        rows = np.flatnonzero(mask)
        want = orc.attention(qr[rows], res["k_m"][h], res["v_m"][h])
        assert np.array_equal(o_r[rows], want)
        # everybody else still reads the row of its (recomputed) merged query
        keep = np.flatnonzero(~mask)
        assert np.array_equal(o_r[keep], res["o_m"][h][aq[keep]])


def test_deviation_is_taken_before_the_outliers_leave():
    """Planted mistake: measuring the deviation against the recomputed merged tokens (or keeping
    the deviation of unmerged tokens) selects a different set."""
    g = orc.Geometry(2, 4, 4, 2, 2)
    rng = np.random.default_rng(11)
    q = rng.standard_normal((2, g.N, 8))
    pi, blocks = orc.temporal_reorder(g)
    qr = [orc.reorder(q[h], pi) for h in range(2)]
    aq = [orc.blockwise_tome(x, g, blocks, 0.75)[0] for x in qr]
    qm, masks, eps, tau = orc.block_aggregate_quantile(qr, aq, g, blocks, 0.75, 0.2)
    eps_wrong = [orc.deviations(x, a, m) for x, a, m in zip(qr, aq, qm)]     # against the filtered means
    tau_wrong = orc.outlier_threshold(np.concatenate(eps_wrong), 0.2)
    assert any((e > tau_wrong).tolist() != m.tolist() for e, m in zip(eps_wrong, masks))
