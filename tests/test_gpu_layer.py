"""GPU parity of httm_layer_forward (the call the benchmark times) on the five workloads.

Workloads 1-3 are compared head by head in full.  Workloads 4-5 run on the GPU at full size, in the
benchmark's launch configuration; the oracle matches and aggregates every head, evaluates its
attention in full for four heads and for a seeded sample of merged query rows against all keys for
the others (rows are independent), so every compared number is still an exact oracle value."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2511_21317_amd as httm
import synth
import synth.vggt_tokens
from oracle import httm_oracle as orc

from gpu_util import (check_assign, check_output, f32, key_scale, oracle_geom, plan_for, require_gpu, round_bf16,
                      run_layer, run_stages)

pytestmark = pytest.mark.gpu


def _inputs(w):
    print(f"[case] {w.name} N={w.N}", flush=True)
    return synth.make_qkv(w, device="cuda")


@pytest.mark.parametrize("idx,anchor", [(1, False), (2, False), (3, False), (2, True), (3, True)],
                         ids=["cfg1", "cfg2", "cfg3", "cfg2_anchored", "cfg3_anchored"])
def test_layer_forward_matches_oracle_in_full(idx, anchor):
    require_gpu()
    w = synth.workload(idx)
    if anchor:   # first-frame anchoring (App. C.2) on the same tokens
        w = dataclasses.replace(w, name=w.name + "_anchored", anchor=True)
    q, k, v = _inputs(w)
    plan = plan_for(w)
    out, views = run_layer(plan, q, k, v)
    ref = orc.layer_forward(f32(q), f32(k), f32(v), oracle_geom(w), w.rho, w.rho)
    aq, ak = views["assign_q"].cpu().numpy(), views["assign_k"].cpu().numpy()
    bad = 0
    for h in range(w.H):
        bad += check_assign(aq[h], ref["assign_q"][h], ref["gap_q"][h], f"cfg{idx} assign_q head {h}")
        bad += check_assign(ak[h], ref["assign_k"][h], ref["gap_k"][h], f"cfg{idx} assign_k head {h}")
    err, rel = check_output(f32(out), ref["O"], f"cfg{idx} layer output")
    print(f"cfg{idx}: index mismatches {bad}, max_abs {err:.4g}, rel_l2 {rel:.4g}", flush=True)
    # the fused layer and the four separate stage calls give identical bits
    staged = run_stages(plan, q, k, v, with_scores=False)
    assert torch.equal(staged["out"], out)
    assert torch.equal(staged["assign_q"], views["assign_q"]) and torch.equal(staged["q_m"], views["q_m"])
    assert torch.equal(staged["v_m"], views["v_m"])
    # run-to-run identical
    out2, _ = run_layer(plan, q, k, v)
    assert torch.equal(out, out2)
    plan.close()


def _touched_clusters(a_gpu, a_ref, M):
    """Merged slots whose membership differs between the GPU and the oracle (an allowed tie moved a
    token from one to the other)."""
    touched = np.zeros(M, dtype=bool)
    bad = np.flatnonzero(a_gpu != a_ref)
    touched[a_gpu[bad]] = True
    touched[a_ref[bad]] = True
    return touched


def _full_size_check(w, q, k, v, out, views, full_heads, n_rows, tag, rho_q, rho_kv, kscale, heads=None):
    """Every head of a full-size run against the oracle: indices (with the tie statistic over all
    heads), merged q / k / v rows, then attention and layer output - every merged query row for the
    heads in `full_heads`, a seeded sample of rows plus the head's last query tile for the others."""
    g = oracle_geom(w)
    pi, blocks = orc.temporal_reorder(g)
    rng = np.random.default_rng(w.index)
    heads = list(range(w.H)) if heads is None else heads
    n_bad = n_tok = 0
    worst = 0.0
    for h in heads:
        qr, kr, vr = (orc.reorder(f32(t[h]), pi) for t in (q, k, v))
        aq, _, gq = orc.blockwise_tome(qr, g, blocks, rho_q)
        ak, _, gk = orc.blockwise_tome(kr, g, blocks, rho_kv)
        aq_gpu, ak_gpu = views["assign_q"][h].cpu().numpy(), views["assign_k"][h].cpu().numpy()
        n_bad += check_assign(aq_gpu, aq, gq, f"{tag} assign_q head {h}")
        n_bad += check_assign(ak_gpu, ak, gk, f"{tag} assign_k head {h}")
        n_tok += aq.size + ak.size
        qm = orc.block_aggregate(qr, aq, g, blocks, rho_q)
        km = orc.block_aggregate(kr, ak, g, blocks, rho_kv)
        vm = orc.block_aggregate(vr, ak, g, blocks, rho_kv)
        # merged rows: one bf16 rounding (half an ulp = 2^-9 relative) from the oracle's fp32 mean,
        # outside the clusters an allowed tie touched
        tq, tk = _touched_clusters(aq_gpu, aq, qm.shape[0]), _touched_clusters(ak_gpu, ak, km.shape[0])
        for name, mean, keep in (("q_m", qm, ~tq), ("k_m", km * kscale, ~tk), ("v_m", vm, ~tk)):
            got = f32(views[name][h])
            assert (np.abs(got - mean) <= 2.0 ** -8 * np.abs(mean) + 1e-30)[keep].all(), f"{tag} {name} head {h}"
        if h in full_heads:
            rows = np.arange(qm.shape[0])
        else:
            rows = rng.choice(qm.shape[0], size=min(n_rows, qm.shape[0]), replace=False)
            # always with the head's last query tile of 256 rows (partial, and run in pieces at cfg 5)
            rows = np.unique(np.concatenate([rows, np.arange((qm.shape[0] - 1) // 256 * 256, qm.shape[0])]))
        rows = rows[~tq[rows]]
        om_rows = orc.attention(qm, km, vm, rows=rows)
        err, _ = check_output(f32(views["o_m"][h][torch.from_numpy(rows).cuda()]), om_rows, f"{tag} o_m head {h}")
        # unmerge + inverse reorder: every input token whose merged query is among the rows
        row_of = -np.ones(qm.shape[0], dtype=np.int64)
        row_of[rows] = np.arange(rows.size)
        sel = np.flatnonzero((row_of[aq] >= 0) & (aq_gpu == aq))     # reordered positions covered
        want = om_rows[row_of[aq[sel]]]
        got = f32(out[torch.from_numpy(pi[sel]).cuda(), h * 64:(h + 1) * 64])
        err2, rel2 = check_output(got, want, f"{tag} output head {h}")
        worst = max(worst, err, err2)
        print(f"{tag} head {h}: {rows.size} merged rows, {sel.size} output rows checked "
              f"({'all' if h in full_heads else 'sampled'}), max_abs {err2:.4g}, rel_l2 {rel2:.4g}", flush=True)
    frac = n_bad / max(n_tok, 1)
    print(f"{tag}: {n_bad} of {n_tok} merge indices differ from the oracle ({frac:.2e} of all tokens of "
          f"{len(heads)} heads, Q and K), every one at a similarity gap below 1e-3; worst output error {worst:.4g}",
          flush=True)
    assert n_bad <= 1e-3 * n_tok


@pytest.mark.parametrize("idx,log2_keys", [(4, True), (5, True), (5, False)])
def test_layer_forward_full_size_all_heads(idx, log2_keys):
    """Workloads 4 and 5 through httm_layer_forward in the benchmark's launch configuration.  With
    log2 keys (what the benchmark times): all 16 heads - indices, merged rows, four heads with every
    attention row and every output token, twelve on samples.  With plain keys (indices and q_m / v_m do
    not depend on the key scale): three heads."""
    require_gpu()
    w = synth.workload(idx)
    q, k, v = _inputs(w)
    plan = plan_for(w, log2_keys=log2_keys)
    out, views = run_layer(plan, q, k, v)
    assert plan.M_q == {4: 28650, 5: 28700}[idx]
    _full_size_check(w, q, k, v, out, views, full_heads=[0, 5, 11, 15] if log2_keys else [7], n_rows=1024,
                     tag=f"cfg{idx}{'' if log2_keys else ' plain keys'}",
                     rho_q=w.rho, rho_kv=w.rho, kscale=key_scale(plan), heads=None if log2_keys else [2, 7, 13])
    # properties that hold at any size: constituents of one merged query share identical output rows
    pi = torch.from_numpy(orc.temporal_reorder(oracle_geom(w))[0]).cuda()
    for h in range(w.H):
        aq = views["assign_q"][h].long()
        o_h = out[:, h * 64:(h + 1) * 64]
        assert torch.equal(o_h[pi], views["o_m"][h][aq])
        assert int(aq.max()) == plan.M_q - 1 and int(aq.min()) == 0
    plan.close()


def test_unmerged_baseline_is_plain_attention():
    """variant 'none' (r = 0): M = N, the layer is exact softmax attention (Eq. 3-4)."""
    require_gpu()
    w = synth.workload(2)
    q, k, v = _inputs(w)
    plan = plan_for(w, variant="none")
    assert plan.M_q == w.N
    out, views = run_layer(plan, q, k, v)
    heads = [0, 7, 15]
    got = f32(out)
    for h in heads:
        want = orc.attention(f32(q[h]), f32(k[h]), f32(v[h]))
        check_output(got[:, h * 64:(h + 1) * 64], want, f"unmerged head {h}")
    plan.close()


def test_unmerged_baseline_full_size_sampled_rows():
    """r = 0 on the largest workload: the oracle evaluates sampled query rows against all keys."""
    require_gpu()
    w = synth.workload(5)
    q, k, v = _inputs(w)
    h = 3
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(w.N, size=512, replace=False))
    om = torch.empty((w.N, 64), dtype=torch.bfloat16, device="cuda")
    print("[step] httm_attention M=N=274800, one head", flush=True)
    httm.attention(q[h], k[h], v[h], om, [0, w.N], [0, w.N], 0.125)
    torch.cuda.synchronize()
    want = orc.attention(f32(q[h]), f32(k[h]), f32(v[h]), rows=rows, chunk=128)
    check_output(f32(om[torch.from_numpy(rows).cuda()]), want, "cfg5 r=0 sampled rows")


@pytest.mark.parametrize("idx", [2, 3])
def test_head_uniform_variant(idx):
    require_gpu()
    w = synth.workload(idx)
    q, k, v = _inputs(w)
    plan = plan_for(w, variant="uniform")
    out, views = run_layer(plan, q, k, v)
    ref = orc.layer_forward(f32(q), f32(k), f32(v), oracle_geom(w), w.rho, w.rho, variant="uniform")
    aq, ak = views["assign_q"].cpu().numpy(), views["assign_k"].cpu().numpy()
    for h in range(w.H):
        assert np.array_equal(aq[h], aq[0]) and np.array_equal(ak[h], ak[0])
    check_assign(aq[0], ref["assign_q"][0], ref["gap_q"][0], "uniform assign_q")
    check_assign(ak[0], ref["assign_k"][0], ref["gap_k"][0], "uniform assign_k")
    check_output(f32(out), ref["O"], f"cfg{idx} uniform output")
    staged = run_stages(plan, q, k, v, with_scores=False)
    assert torch.equal(staged["out"], out)
    plan.close()


@pytest.mark.parametrize("w,rho_kv", [
    (synth.vggt_tokens.Workload("uniform_big_b16T8", 71, 8, 16, 20, 16, 8, 0.75, 1, H=3), 0.5),                    # 2048 + 512
    (synth.vggt_tokens.Workload("uniform_paper_blocks", 72, 30, 16, 16, 128, 30, 0.9, 1, H=3, chunked=True), 0.7),  # 3840
], ids=lambda c: getattr(c, "name", str(c)))
def test_head_uniform_variant_on_blocks_of_more_than_512_tokens(w, rho_kv):
    """One topology for all heads (Sec. 3.2's counter-example) on the two-kernel path: the shared
    matching runs on the head-averaged fp32 tokens with the dst tokens tiled through LDS."""
    require_gpu()
    q, k, v = _inputs(w)
    plan = plan_for(w, variant="uniform", rho_kv=rho_kv)
    out, views = run_layer(plan, q, k, v)
    ref = orc.layer_forward(f32(q), f32(k), f32(v), oracle_geom(w), w.rho, rho_kv, variant="uniform")
    aq, ak = views["assign_q"].cpu().numpy(), views["assign_k"].cpu().numpy()
    for h in range(w.H):
        assert np.array_equal(aq[h], aq[0]) and np.array_equal(ak[h], ak[0])
    nq = check_assign(aq[0], ref["assign_q"][0], ref["gap_q"][0], f"{w.name} assign_q")
    nk = check_assign(ak[0], ref["assign_k"][0], ref["gap_k"][0], f"{w.name} assign_k")
    from gpu_util import oracle_continued_from, output_bar
    want = oracle_continued_from(ref, f32(q), f32(k), f32(v), oracle_geom(w), w.rho, rho_kv, aq, ak)
    bar_abs, bar_rel, _, _ = output_bar(ref, key_scale(plan))
    got = f32(out)
    err = float(np.abs(got - want).max())
    rel = float(np.linalg.norm(got - want) / np.linalg.norm(want))
    print(f"{w.name}: {nq} + {nk} shared indices differ, max_abs {err:.4g} (bar {bar_abs:.4g}), rel_l2 {rel:.4g}", flush=True)
    assert err < bar_abs and rel < bar_rel
    staged = run_stages(plan, q, k, v, with_scores=True)
    assert torch.equal(staged["out"], out)
    plan.close()


def test_head_uniform_variant_full_size():
    """Workload 5, one topology for all heads (from the head-averaged tokens): the shared indices of Q
    and K against the oracle for every head, then merged rows, attention rows and layer outputs of
    two heads (sampled rows plus the last query tile)."""
    require_gpu()
    w = synth.workload(5)
    q, k, v = _inputs(w)
    plan = plan_for(w, variant="uniform")
    out, views = run_layer(plan, q, k, v)
    g = oracle_geom(w)
    pi, blocks = orc.temporal_reorder(g)
    # the shared topology from the oracle's head-averaged tokens (all heads needed for the mean)
    aq, _, gq = orc.blockwise_tome(orc.reorder(orc.head_mean(f32(q)), pi), g, blocks, w.rho)
    ak, _, gk = orc.blockwise_tome(orc.reorder(orc.head_mean(f32(k)), pi), g, blocks, w.rho)
    aq_gpu, ak_gpu = views["assign_q"].cpu().numpy(), views["assign_k"].cpu().numpy()
    for h in range(w.H):
        assert np.array_equal(aq_gpu[h], aq_gpu[0]) and np.array_equal(ak_gpu[h], ak_gpu[0])
    nq = check_assign(aq_gpu[0], aq, gq, "cfg5 uniform assign_q")
    nk = check_assign(ak_gpu[0], ak, gk, "cfg5 uniform assign_k")
    print(f"cfg5 uniform: {nq} + {nk} of {aq.size} shared indices differ (gap < 1e-3)", flush=True)
    tq, tk = _touched_clusters(aq_gpu[0], aq, plan.M_q), _touched_clusters(ak_gpu[0], ak, plan.M_k)
    rng = np.random.default_rng(59)
    ks = key_scale(plan)
    for h in (2, 9):
        qr, kr, vr = (orc.reorder(f32(t[h]), pi) for t in (q, k, v))
        qm = orc.block_aggregate(qr, aq, g, blocks, w.rho)
        km = orc.block_aggregate(kr, ak, g, blocks, w.rho)
        vm = orc.block_aggregate(vr, ak, g, blocks, w.rho)
        for name, mean, keep in (("q_m", qm, ~tq), ("k_m", km * ks, ~tk), ("v_m", vm, ~tk)):
            assert (np.abs(f32(views[name][h]) - mean) <= 2.0 ** -8 * np.abs(mean) + 1e-30)[keep].all(), (name, h)
        rows = np.unique(np.concatenate([rng.choice(plan.M_q, size=1024, replace=False),
                                         np.arange((plan.M_q - 1) // 256 * 256, plan.M_q)]))
        rows = rows[~tq[rows]]
        om_rows = orc.attention(qm, km, vm, rows=rows)
        check_output(f32(views["o_m"][h][torch.from_numpy(rows).cuda()]), om_rows, f"cfg5 uniform o_m head {h}")
        row_of = -np.ones(plan.M_q, dtype=np.int64)
        row_of[rows] = np.arange(rows.size)
        sel = np.flatnonzero((row_of[aq] >= 0) & (aq_gpu[0] == aq))
        got = f32(out[torch.from_numpy(pi[sel]).cuda(), h * 64:(h + 1) * 64])
        err, rel = check_output(got, om_rows[row_of[aq[sel]]], f"cfg5 uniform output head {h}")
        print(f"cfg5 uniform head {h}: {sel.size} output rows checked, max_abs {err:.4g}, rel_l2 {rel:.4g}", flush=True)
    plan.close()
