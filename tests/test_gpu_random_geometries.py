"""GPU parity of the layer on seeded random geometries: odd grids, block shapes that do not divide
them, both block kinds, anchoring, separate ratios, both key conventions, the head-uniform variant.
Every case is small enough for the oracle to evaluate in full."""
import numpy as np
import pytest
import torch

import paper_2511_21317_amd as httm
import synth
from oracle import httm_oracle as orc
from synth.vggt_tokens import Workload

from gpu_util import (TIE_FRACTION, TIE_GAP, check_output, f32, oracle_continued_from, oracle_geom, output_bar,
                      plain_keys, plan_for, require_gpu, run_layer, run_stages)

pytestmark = pytest.mark.gpu

RHOS = [0.0, 0.3, 0.5, 0.75, 0.9, 1.0]


def _draw(seed):
    """A geometry and its options from one seed (plain Python / NumPy integers, no method arithmetic)."""
    rng = np.random.default_rng(7000 + seed)
    chunked = bool(rng.integers(0, 2))
    S = int(rng.integers(1, 10))
    Hp, Wp = int(rng.integers(3, 21)), int(rng.integers(3, 21))
    T = int(rng.integers(1, 6))
    b = int(rng.integers(5, 260)) if chunked else int(rng.integers(2, 9))
    n_special = int(rng.choice([0, 1, 5]))
    H = int(rng.integers(1, 4))
    w = Workload(f"rand{seed}_S{S}_{Hp}x{Wp}_b{b}T{T}{'_chunked' if chunked else ''}", 100 + seed, S, Hp, Wp, b, T,
                 float(rng.choice(RHOS)), 1, H=H, n_special=n_special, anchor=bool(rng.integers(0, 2)),
                 chunked=chunked)
    rho_kv = float(rng.choice(RHOS))
    variant = "uniform" if rng.integers(0, 4) == 0 else "headwise"
    log2_keys = bool(rng.integers(0, 2))
    return w, rho_kv, variant, log2_keys


def _draw_big(seed):
    """The same with blocks of 513 .. 4096 tokens (runs of b patch tokens over T frames): the two-kernel
    path of stage 2."""
    rng = np.random.default_rng(424200 + seed)
    Hp, Wp = int(rng.integers(8, 21)), int(rng.integers(8, 21))
    P = Hp * Wp
    T = int(rng.integers(2, 13))
    S = int(rng.integers(T, max(T, min(3 * T, 6000 // (P + 5))) + 1))
    b_lo, b_hi = max(8, -(-520 // T)), max(8, min(P, 4096 // T))
    b = int(rng.integers(min(b_lo, b_hi), b_hi + 1))
    w = Workload(f"big{seed}_S{S}_{Hp}x{Wp}_b{b}T{T}_chunked", 900 + seed, S, Hp, Wp, b, T,
                 float(rng.choice(RHOS)), 1, H=int(rng.integers(1, 3)), n_special=int(rng.choice([0, 1, 5])),
                 anchor=bool(rng.integers(0, 2)), chunked=True)
    rho_kv = float(rng.choice(RHOS))
    variant = "uniform" if rng.integers(0, 4) == 0 else "headwise"
    return w, rho_kv, variant, bool(rng.integers(0, 2))


@pytest.mark.parametrize("seed", range(40))
def test_layer_on_a_random_geometry(seed):
    _check_layer(*_draw(seed))


@pytest.mark.parametrize("seed", range(24))
def test_layer_on_a_random_geometry_with_big_blocks(seed):
    _check_layer(*_draw_big(seed))


def _check_layer(w, rho_kv, variant, log2_keys):
    require_gpu()
    g = oracle_geom(w)
    _, blocks = orc.temporal_reorder(g)
    max_block = max((n for _, n in blocks), default=0)
    print(f"[case] {w.name} N={w.N} H={w.H} rho_q={w.rho} rho_kv={rho_kv} {variant} anchor={w.anchor} "
          f"log2_keys={log2_keys} largest block {max_block}", flush=True)
    if w.N > 6000:
        pytest.skip("larger than the oracle should evaluate in full here")
    q, k, v = synth.make_qkv(w, device="cuda")
    plan = plan_for(w, variant=variant, rho_kv=rho_kv, log2_keys=log2_keys)
    got = run_stages(plan, q, k, v, with_scores=False)
    ref = orc.layer_forward(f32(q), f32(k), f32(v), g, w.rho, rho_kv, variant=variant)
    assert plan.M_q == ref["q_m"][0].shape[0] and plan.M_k == ref["k_m"][0].shape[0]
    aq, ak = got["assign_q"].cpu().numpy(), got["assign_k"].cpu().numpy()
    pi = ref["pi"]
    for h in range(w.H):
        # indices: equal except at near-ties (the oracle's best-vs-second gap below 1e-3).  The 0.1 %
        # allowance of the workloads is not applied: these inputs have a few dozen to a few thousand
        # tokens of a smooth field, and on the smallest grids near-ties are the rule, not the exception
        # - there the count is bounded by the number of near-tie tokens the oracle itself reports.
        for a_gpu, name, gap in ((aq[h], "assign_q", "gap_q"), (ak[h], "assign_k", "gap_k")):
            bad = np.flatnonzero(a_gpu != ref[name][h])
            assert (ref[gap][h][bad] < TIE_GAP).all(), f"{w.name} {name} head {h}: differs at gap {ref[gap][h][bad].max()}"
            near = int((ref[gap][h] < TIE_GAP).sum())
            assert bad.size <= max(TIE_FRACTION * a_gpu.size, near), f"{w.name} {name} head {h}: {bad.size} indices differ"
        # merged tokens: one bf16 rounding from the oracle's fp32 mean, outside clusters touched by a tie
        for name, asg, a_gpu in (("q_m", "assign_q", aq), ("k_m", "assign_k", ak), ("v_m", "assign_k", ak)):
            bad = np.flatnonzero(a_gpu[h] != ref[asg][h])
            keep = np.ones(ref[name][h].shape[0], dtype=bool)
            keep[a_gpu[h][bad]] = False
            keep[ref[asg][h][bad]] = False
            mean = ref[name][h] * (got["key_scale"] if name == "k_m" else np.float32(1.0))
            assert (np.abs(f32(got[name][h]) - mean) <= 2.0 ** -8 * np.abs(mean) + 1e-30)[keep].all(), (w.name, name, h)
        # stage 3 on the GPU's own merged tokens against the oracle's attention on the same tokens
        want = orc.attention(f32(got["q_m"][h]), plain_keys(plan, f32(got["k_m"][h])), f32(got["v_m"][h]))
        check_output(f32(got["o_m"][h]), want, f"{w.name} attention head {h}", relative_to_magnitude=True)
        # stage 4: bit-exact copies of the merged outputs
        want_r = orc.unmerge_by_cluster(got["o_m"][h].cpu().view(torch.int16).numpy(), aq[h].astype(np.int64))
        assert np.array_equal(got["out"].cpu().view(torch.int16).numpy()[:, h * 64:(h + 1) * 64],
                              orc.inverse_reorder(want_r, pi))
    # end to end against the all-fp32 oracle, downstream of the GPU's own (checked) cluster decisions
    # where an allowed tie went the other way.  The bar is the spec bar, or twice what bf16 storage
    # of the intermediates costs on this very case (gpu_util.output_bar: with a few hundred keys per row
    # and un-normalised values that alone passes 2e-2; tests/test_tolerance_model.py pins the model).
    out_f = f32(got["out"])
    assert np.isfinite(out_f).all()
    want = oracle_continued_from(ref, f32(q), f32(k), f32(v), g, w.rho, rho_kv, aq, ak)
    bar_abs, bar_rel, e_abs, e_rel = output_bar(ref, got["key_scale"])
    err = float(np.abs(out_f - want).max())
    rel = float(np.linalg.norm(out_f - want) / max(np.linalg.norm(want), 1e-30))
    print(f"{w.name}: max_abs {err:.4g} (bf16 storage alone {e_abs:.4g}, bar {bar_abs:.4g}), "
          f"rel_l2 {rel:.4g} (storage {e_rel:.4g}, bar {bar_rel:.4g})", flush=True)
    assert err < bar_abs and rel < bar_rel, f"{w.name} layer output: max_abs={err:.4g} rel_l2={rel:.4g}"
    out, _ = run_layer(plan, q, k, v)
    assert torch.equal(out, got["out"])                  # the layer call = the four stages, bit for bit
    plan.close()
