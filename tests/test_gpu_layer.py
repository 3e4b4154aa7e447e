"""GPU parity of httm_layer_forward (the call the benchmark times) on the five workloads.

Workloads 1-3 are compared head by head in full.  Workloads 4-5 run on the GPU at full size, in the
benchmark's launch configuration; the oracle is evaluated for a few heads only (heads are independent
in the head-wise method), and its attention for a seeded sample of merged query rows against all
keys (rows are independent), so every compared number is still an exact oracle value."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2511_21317_amd as httm
import synth
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


def _sampled_head_check(w, q, k, v, out, views, heads, n_rows, tag, rho_q, rho_kv, kscale):
    g = oracle_geom(w)
    pi, blocks = orc.temporal_reorder(g)
    rng = np.random.default_rng(w.index)
    for h in heads:
        qr, kr, vr = (orc.reorder(f32(t[h]), pi) for t in (q, k, v))
        aq, _, gq = orc.blockwise_tome(qr, g, blocks, rho_q)
        ak, _, gk = orc.blockwise_tome(kr, g, blocks, rho_kv)
        check_assign(views["assign_q"][h].cpu().numpy(), aq, gq, f"{tag} assign_q head {h}")
        check_assign(views["assign_k"][h].cpu().numpy(), ak, gk, f"{tag} assign_k head {h}")
        qm = orc.block_aggregate(qr, aq, g, blocks, rho_q)
        km = orc.block_aggregate(kr, ak, g, blocks, rho_kv)
        vm = orc.block_aggregate(vr, ak, g, blocks, rho_kv)
        ok_k = (views["assign_k"][h].cpu().numpy() == ak).all()
        if ok_k:     # no tie mismatch in this head: merged rows are one bf16 rounding from the fp32 mean
            assert (np.abs(f32(views["k_m"][h]) - km * kscale) <= 2.0 ** -8 * np.abs(km * kscale) + 1e-30).all()
            assert (np.abs(f32(views["v_m"][h]) - vm) <= 2.0 ** -8 * np.abs(vm) + 1e-30).all()
        rows = rng.choice(qm.shape[0], size=min(n_rows, qm.shape[0]), replace=False)
        # always with the head's last query tile of 256 rows (partial, and run in pieces at cfg 5)
        rows = np.unique(np.concatenate([rows, np.arange((qm.shape[0] - 1) // 256 * 256, qm.shape[0])]))
        om_rows = orc.attention(qm, km, vm, rows=rows)
        check_output(f32(views["o_m"][h][torch.from_numpy(rows).cuda()]), om_rows, f"{tag} o_m head {h}")
        # unmerge + inverse reorder of the sampled rows: every input token whose merged query was sampled
        row_of = -np.ones(qm.shape[0], dtype=np.int64)
        row_of[rows] = np.arange(rows.size)
        sel = np.flatnonzero(row_of[aq] >= 0)                  # reordered positions covered by the sample
        want = om_rows[row_of[aq[sel]]]
        got = f32(out[torch.from_numpy(pi[sel]).cuda(), h * 64:(h + 1) * 64])
        err, rel = check_output(got, want, f"{tag} output head {h}")
        print(f"{tag} head {h}: {sel.size} output rows checked, max_abs {err:.4g}, rel_l2 {rel:.4g}", flush=True)


@pytest.mark.parametrize("idx,log2_keys", [(4, True), (5, True), (5, False)])
def test_layer_forward_full_size_sampled(idx, log2_keys):
    require_gpu()
    w = synth.workload(idx)
    q, k, v = _inputs(w)
    plan = plan_for(w, log2_keys=log2_keys)
    out, views = run_layer(plan, q, k, v)
    assert plan.M_q == {4: 28650, 5: 28700}[idx]
    _sampled_head_check(w, q, k, v, out, views, heads=[0, 11] if log2_keys else [7], n_rows=1024,
                        tag=f"cfg{idx}{'' if log2_keys else ' plain keys'}",
                        rho_q=w.rho, rho_kv=w.rho, kscale=key_scale(plan))
    # properties that hold at any size: constituents of one merged query share identical output rows
    h = 5
    aq = views["assign_q"][h].long()
    pi = torch.from_numpy(orc.temporal_reorder(oracle_geom(w))[0]).cuda()
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


def test_head_uniform_variant_full_size():
    require_gpu()
    w = synth.workload(5)
    q, k, v = _inputs(w)
    plan = plan_for(w, variant="uniform")
    out, views = run_layer(plan, q, k, v)
    g = oracle_geom(w)
    pi, blocks = orc.temporal_reorder(g)
    # the shared topology from the oracle's head-averaged tokens (all heads needed for the mean)
    mean_q = orc.head_mean(f32(q))
    aq, _, gq = orc.blockwise_tome(orc.reorder(mean_q, pi), g, blocks, w.rho)
    del mean_q
    for h in (0, 9):
        check_assign(views["assign_q"][h].cpu().numpy(), aq, gq, f"cfg5 uniform assign_q head {h}")
    h = 9
    qm = orc.block_aggregate(orc.reorder(f32(q[h]), pi), aq, g, blocks, w.rho)
    if (views["assign_q"][h].cpu().numpy() == aq).all():
        assert (np.abs(f32(views["q_m"][h]) - qm) <= 2.0 ** -8 * np.abs(qm) + 1e-30).all()
    plan.close()
