"""GPU parity, stage by stage, through the C ABI: HIP kernels vs the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import paper_2511_21317_amd as httm
import synth
from oracle import httm_oracle as orc
from synth.vggt_tokens import Workload

from gpu_util import (check_assign, check_output, excuse_tie_tokens, f32, oracle_geom, plain_keys, plan_for, require_gpu,
                      round_bf16, run_layer, run_stages)

pytestmark = pytest.mark.gpu

# Small shapes that span several tiles and have ragged tails; name, S, Hp, Wp, b, T, rho, shift
ODD = [
    Workload("odd_partial_everywhere", 11, 5, 7, 9, 4, 3, 0.6, 1, H=3),
    Workload("odd_single_token_blocks", 12, 3, 13, 9, 4, 2, 0.5, 1, H=2),    # 1x1xT corner blocks
    Workload("odd_block512_b8T8", 13, 9, 10, 12, 8, 8, 0.9, 1, H=2),          # 512-token blocks + partials
    Workload("odd_block512_b16T2", 14, 3, 17, 16, 16, 2, 0.75, 1, H=2),
    Workload("odd_keep_one", 15, 4, 8, 8, 4, 2, 1.0, 1, H=2),                 # rho = 1: one cluster per block
    Workload("odd_no_special", 16, 4, 12, 15, 3, 2, 0.5, 1, H=2, n_special=0),
    Workload("odd_k_gt_32", 17, 4, 16, 16, 8, 4, 0.25, 1, H=2),               # 256-token blocks, k = 192
    # first-frame anchoring (App. C.2): frame-0 tokens are dst whatever the ratio
    Workload("anchored_ratio_below_frame0", 18, 6, 13, 9, 4, 4, 0.9, 1, H=2, anchor=True),   # k = n0
    Workload("anchored_mixed_dst", 19, 5, 12, 15, 4, 3, 0.5, 1, H=3, anchor=True),            # k > n0
    Workload("anchored_block512", 20, 9, 10, 12, 8, 8, 0.75, 1, H=2, anchor=True),
    # chunked spatial blocks (Sec. 4.1): runs of b consecutive tokens of a frame x T frames
    Workload("chunked_ns50_nt5", 22, 7, 11, 13, 50, 5, 0.8, 1, H=2, chunked=True),          # 250-token blocks
    Workload("chunked_ns128_nt4_anchored", 23, 6, 16, 20, 128, 4, 0.9, 1, H=2, chunked=True, anchor=True),
    # blocks of more than 512 tokens: the two-kernel path
    Workload("big_b16T8", 24, 8, 16, 20, 16, 8, 0.75, 1, H=2),                              # 2048 + 512
    Workload("big_chunked_ns128_nt30", 25, 33, 12, 16, 128, 30, 0.9, 1, H=2, chunked=True),  # 3840, 1920, 384, 192
    Workload("big_chunked_anchored_k_gt_n0", 26, 12, 10, 13, 100, 12, 0.5, 1, H=2, chunked=True, anchor=True),
]


def _inputs(w):
    print(f"[case] {w.name} N={w.N} H={w.H}", flush=True)
    return synth.make_qkv(w, device="cuda")


def _oracle_stages(w, q, k, v, rho_q=None, rho_kv=None):
    rq = w.rho if rho_q is None else rho_q
    rk = rq if rho_kv is None else rho_kv
    return orc.layer_forward(f32(q), f32(k), f32(v), oracle_geom(w), rq, rk)


@pytest.mark.parametrize("w", [synth.workload(1), synth.workload(2), synth.workload(3)] + ODD,
                         ids=lambda w: w.name)
def test_reorder_is_a_bit_exact_gather_and_inverts(w):
    require_gpu()
    q, _, _ = _inputs(w)
    plan = plan_for(w)
    qr = torch.empty_like(q)
    back = torch.empty_like(q)
    httm.reorder(plan, q, qr, 0)
    httm.reorder(plan, qr, back, 1)
    torch.cuda.synchronize()
    pi, _ = orc.temporal_reorder(oracle_geom(w))
    want = orc.reorder(q.cpu().view(torch.int16).numpy(), pi)        # raw bf16 bit patterns
    assert np.array_equal(qr.cpu().view(torch.int16).numpy(), want)
    assert torch.equal(back, q)
    plan.close()


@pytest.mark.parametrize("w", [synth.workload(1), synth.workload(2), synth.workload(3)] + ODD,
                         ids=lambda w: w.name)
def test_every_stage_matches_the_oracle(w):
    require_gpu()
    q, k, v = _inputs(w)
    plan = plan_for(w)
    got = run_stages(plan, q, k, v)
    ref = _oracle_stages(w, q, k, v)
    H = w.H
    n_bad = 0
    for name, gap in (("assign_q", "gap_q"), ("assign_k", "gap_k")):
        g_all = got[name].cpu().numpy()
        for h in range(H):
            n_bad += check_assign(g_all[h], ref[name][h], ref[gap][h], f"{w.name} {name} head {h}")
    # scores
    for name in ("score_q", "score_k"):
        g_all = got[name].cpu().numpy()
        for h in range(H):
            same = got["assign" + name[5:]].cpu().numpy()[h] == ref["assign" + name[5:]][h]
            assert np.abs(g_all[h] - ref[name][h])[same].max() < 1e-5
    # merged tokens: fp32 sums in the oracle's order, rounded once to bf16.  Clusters touched by
    # an (allowed) tie mismatch legitimately differ and are left out.
    for name, asg in (("q_m", "assign_q"), ("k_m", "assign_k"), ("v_m", "assign_k")):
        g_all = f32(got[name])
        a_all = got[asg].cpu().numpy()
        for h in range(H):
            bad = np.flatnonzero(a_all[h] != ref[asg][h])
            keep = np.ones(g_all[h].shape[0], dtype=bool)
            keep[a_all[h][bad]] = False
            keep[ref[asg][h][bad]] = False
            # (merged keys: times the plan's factor, in fp32, before the one rounding)
            mean = ref[name][h] * (got["key_scale"] if name == "k_m" else np.float32(1.0))
            want = round_bf16(mean)
            exact = (g_all[h] == want).all(axis=1)[keep]
            assert exact.mean() > 0.999, f"{name} head {h}: {1 - exact.mean():.3g} rows differ"
            # never further than one bf16 rounding (half an ulp = 2^-9 relative) from the fp32 mean
            assert (np.abs(g_all[h] - mean) <= 2.0 ** -8 * np.abs(mean) + 1e-30)[keep].all()
    # attention on the GPU's own merged tokens vs the oracle's attention on the same tokens
    for h in range(H):
        want = orc.attention(f32(got["q_m"][h]), plain_keys(plan, f32(got["k_m"][h])), f32(got["v_m"][h]))
        check_output(f32(got["o_m"][h]), want, f"{w.name} attention head {h}", relative_to_magnitude=w.index > 5)
    # unmerge: bit-exact copies of the GPU's o_m rows
    om_bits = got["o_m"].cpu().view(torch.int16).numpy()
    aq = got["assign_q"].cpu().numpy().astype(np.int64)
    pi = ref["pi"]
    o_r_bits = got["o_r"].cpu().view(torch.int16).numpy()
    o_hn_bits = got["o_hn"].cpu().view(torch.int16).numpy()
    out_bits = got["out"].cpu().view(torch.int16).numpy()
    for h in range(H):
        want_r = orc.unmerge_by_cluster(om_bits[h], aq[h])
        assert np.array_equal(o_r_bits[h], want_r)
        want_in = orc.inverse_reorder(want_r, pi)
        assert np.array_equal(o_hn_bits[h], want_in)
        assert np.array_equal(out_bits[:, h * 64:(h + 1) * 64], want_in)
    # and the end-to-end output against the all-fp32 oracle.  A query token whose cluster differs by
    # an allowed tie reads another merged row, and the two merged queries involved have other
    # constituents: those tokens are left out (there are at most TIE_FRACTION of them).
    got_o = f32(got["out"])
    want_o = excuse_tie_tokens(got_o, ref["O"], aq, ref)
    check_output(got_o, want_o, f"{w.name} layer output (stage by stage)",
                 relative_to_magnitude=w.index > 5)
    plan.close()


def test_separate_query_and_key_ratios():
    require_gpu()
    w = synth.workload(2)
    q, k, v = _inputs(w)
    plan = plan_for(w, rho_q=0.75, rho_kv=0.25)
    got = run_stages(plan, q, k, v, with_scores=False)
    ref = _oracle_stages(w, q, k, v, 0.75, 0.25)
    assert plan.M_q == ref["q_m"][0].shape[0] and plan.M_k == ref["k_m"][0].shape[0] and plan.M_q != plan.M_k
    for h in range(w.H):
        check_assign(got["assign_q"][h].cpu().numpy(), ref["assign_q"][h], ref["gap_q"][h], f"q head {h}")
        check_assign(got["assign_k"][h].cpu().numpy(), ref["assign_k"][h], ref["gap_k"][h], f"k head {h}")
    check_output(f32(got["out"]), ref["O"], "rho_q=0.75 rho_kv=0.25")
    plan.close()


def test_paper_scale_blocks_with_separate_ratios():
    """Sec. 4.1: n_s = 128, n_t = 30 (blocks of 3840 tokens), 90 % of the queries and 70 % of the
    keys / values merged: 384 and 1152 clusters per full block."""
    require_gpu()
    w = Workload("paper_ns128_nt30", 27, 30, 16, 16, 128, 30, 0.9, 1, H=2, chunked=True)
    q, k, v = _inputs(w)
    plan = plan_for(w, rho_q=0.9, rho_kv=0.7)
    assert plan.M_q == 30 * 5 + 2 * 384 and plan.M_k == 30 * 5 + 2 * 1152
    got = run_stages(plan, q, k, v)
    ref = _oracle_stages(w, q, k, v, 0.9, 0.7)
    for h in range(w.H):
        check_assign(got["assign_q"].cpu().numpy()[h], ref["assign_q"][h], ref["gap_q"][h], "paper-scale assign_q")
        check_assign(got["assign_k"].cpu().numpy()[h], ref["assign_k"][h], ref["gap_k"][h], "paper-scale assign_k")
        for name, asg in (("q_m", "assign_q"), ("k_m", "assign_k"), ("v_m", "assign_k")):
            if np.array_equal(got[asg].cpu().numpy()[h], ref[asg][h]):
                want = ref[name][h] * (got["key_scale"] if name == "k_m" else np.float32(1.0))
                assert (np.abs(f32(got[name][h]) - want) <= 2.0 ** -8 * np.abs(want) + 1e-30).all(), name
    got_o = f32(got["out"])
    want_o = excuse_tie_tokens(got_o, ref["O"], got["assign_q"].cpu().numpy().astype(np.int64), ref)
    check_output(got_o, want_o, "paper-scale blocks, layer output", relative_to_magnitude=True)
    plan.close()


RAGGED = [
    ([1, 63, 64, 65, 129, 300], [7, 64, 1, 200, 513, 65]),
    ([128, 0, 5, 257], [64, 33, 0, 1000]),            # a head without queries, a head without keys
    ([2000], [3001]),
    ([90 + 3 * h for h in range(64)], [70 + 5 * h for h in range(64)]),   # the largest head count the ABI takes
]


@pytest.mark.parametrize("mq,mk", RAGGED)
def test_attention_on_ragged_heads(mq, mk):
    require_gpu()
    print(f"[case] ragged attention mq={mq} mk={mk}", flush=True)
    gen = torch.Generator().manual_seed(1000 + sum(mq))
    qo = np.concatenate([[0], np.cumsum(mq)])
    ko = np.concatenate([[0], np.cumsum(mk)])
    qm = torch.randn((int(qo[-1]), 64), generator=gen).to(torch.bfloat16).cuda()
    km = torch.randn((int(ko[-1]), 64), generator=gen).to(torch.bfloat16).cuda()
    vm = torch.randn((int(ko[-1]), 64), generator=gen).to(torch.bfloat16).cuda()
    om = torch.full_like(qm, float("nan"))
    httm.attention(qm, km, vm, om, qo, ko, 0.125)
    torch.cuda.synchronize()
    for h in range(len(mq)):
        got = f32(om[qo[h]:qo[h + 1]])
        if mq[h] == 0:
            continue
        if mk[h] == 0:
            assert (got == 0).all()
            continue
        want = orc.attention(f32(qm[qo[h]:qo[h + 1]]), f32(km[ko[h]:ko[h + 1]]), f32(vm[ko[h]:ko[h + 1]]))
        check_output(got, want, f"ragged head {h} ({mq[h]}x{mk[h]})")


@pytest.mark.parametrize("seed", range(12))
def test_attention_on_random_ragged_heads(seed):
    """Both stage-3 entry points on seeded random head lengths: empty heads, lengths around the tile
    sizes (32, 64, 128, 256), problems on either side of the choice between 128- and 256-row tiles."""
    require_gpu()
    rng = np.random.default_rng(8000 + seed)
    H = int(rng.integers(1, 7))
    pick = lambda: int(rng.choice([0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, int(rng.integers(1, 3000))]))
    mq, mk = [pick() for _ in range(H)], [pick() for _ in range(H)]
    if seed % 4 == 3:                     # many tiles: the 256-row configuration
        mq = [int(rng.integers(20000, 30000)) for _ in range(H)]
        mk = [int(rng.integers(1, 400)) for _ in range(H)]
    print(f"[case] random ragged attention seed {seed} mq={mq} mk={mk}", flush=True)
    gen = torch.Generator().manual_seed(8000 + seed)
    qo = [int(x) for x in np.concatenate([[0], np.cumsum(mq)])]
    ko = [int(x) for x in np.concatenate([[0], np.cumsum(mk)])]
    qm = torch.randn((max(qo[-1], 1), 64), generator=gen).to(torch.bfloat16).cuda()
    kf = torch.randn((max(ko[-1], 1), 64), generator=gen)
    vm = torch.randn((max(ko[-1], 1), 64), generator=gen).to(torch.bfloat16).cuda()
    for log2 in (False, True):
        km = (_log2_keys(kf) if log2 else kf.to(torch.bfloat16)).cuda()
        om = torch.full_like(qm, float("nan"))
        if log2:
            httm.attention_log2(qm, km, vm, om, qo, ko)
        else:
            httm.attention(qm, km, vm, om, qo, ko, 0.125)
        torch.cuda.synchronize()
        for h in range(H):
            got = f32(om[qo[h]:qo[h + 1]])
            if mq[h] == 0:
                continue
            if mk[h] == 0:
                assert (got == 0).all()
                continue
            kk = f32(km[ko[h]:ko[h + 1]])
            if log2:
                kk = kk / np.float32(httm.LOG2_KEY_SCALE)
            rows = np.arange(mq[h]) if mq[h] <= 4000 else np.sort(rng.choice(mq[h], size=2000, replace=False))
            want = orc.attention(f32(qm[qo[h]:qo[h + 1]])[rows], kk, f32(vm[ko[h]:ko[h + 1]]))
            check_output(got[rows], want, f"random ragged head {h} ({mq[h]}x{mk[h]}, log2={log2})")
        assert torch.isnan(om[qo[-1]:].float()).all()       # nothing written past the last head


def test_attention_partial_tiles_in_a_large_grid():
    """In a grid of many workgroups a short partial tile is computed by the workgroup of the head's
    last full tile (second pass); longer partial tiles and heads that are a whole number of tiles
    sit beside it.  Checks the rows around every head's end and start."""
    require_gpu()
    mq = [65536 + 20, 65536 + 100, 65536 + 200, 65536, 40]
    mk = [70, 130, 64, 200, 90]
    print(f"[case] large-grid ragged attention mq={mq} mk={mk}", flush=True)
    gen = torch.Generator().manual_seed(4242)
    qo = np.concatenate([[0], np.cumsum(mq)])
    ko = np.concatenate([[0], np.cumsum(mk)])
    qm = torch.randn((int(qo[-1]), 64), generator=gen).to(torch.bfloat16).cuda()
    km = torch.randn((int(ko[-1]), 64), generator=gen).to(torch.bfloat16).cuda()
    vm = torch.randn((int(ko[-1]), 64), generator=gen).to(torch.bfloat16).cuda()
    om = torch.full_like(qm, float("nan"))
    httm.attention(qm, km, vm, om, qo, ko, 0.125)
    torch.cuda.synchronize()
    assert not torch.isnan(om.float()).any()
    for h in range(len(mq)):
        rows = np.unique(np.concatenate([np.arange(min(300, mq[h])),
                                         np.arange(max(0, mq[h] - 800), mq[h])]))
        got = f32(om[qo[h]:qo[h + 1]])[rows]
        want = orc.attention(f32(qm[qo[h]:qo[h + 1]])[rows], f32(km[ko[h]:ko[h + 1]]),
                             f32(vm[ko[h]:ko[h + 1]]))
        check_output(got, want, f"large-grid ragged head {h} ({mq[h]}x{mk[h]})")


def test_attention_with_large_logits_stays_finite():
    """Online softmax: rows whose maximum moves a lot between key tiles."""
    require_gpu()
    gen = torch.Generator().manual_seed(77)
    qm = (torch.randn((200, 64), generator=gen) * 6).to(torch.bfloat16).cuda()
    km = (torch.randn((700, 64), generator=gen) * 6).to(torch.bfloat16).cuda()
    vm = torch.randn((700, 64), generator=gen).to(torch.bfloat16).cuda()
    om = torch.empty_like(qm)
    httm.attention(qm, km, vm, om, [0, 200], [0, 700], 0.125)
    torch.cuda.synchronize()
    want = orc.attention(f32(qm), f32(km), f32(vm))
    got = f32(om)
    assert np.isfinite(got).all()
    check_output(got, want, "large logits", relative_to_magnitude=True)


@pytest.mark.parametrize("where", ["second_step", "late", "everywhere_growing"])
def test_attention_shift_is_raised_when_later_keys_dominate(where):
    """The softmax shift is fixed from the first 32 keys; keys whose logits exceed it by more than
    2^60 must take the overflow path (raise the shift, rescale the accumulators) and still match."""
    require_gpu()
    gen = torch.Generator().manual_seed(99)
    mq, mk = 150, 1000
    qm = torch.randn((mq, 64), generator=gen) * 3
    km = torch.randn((mk, 64), generator=gen) * 0.01          # first keys: logits ~ 0
    vm = torch.randn((mk, 64), generator=gen)
    if where == "second_step":
        km[32:64] = torch.randn((32, 64), generator=gen) * 40     # jump right after the first step
    elif where == "late":
        km[700:] = torch.randn((300, 64), generator=gen) * 40
    else:
        km = torch.randn((mk, 64), generator=gen) * torch.linspace(0.01, 60, mk)[:, None]
    qm, km, vm = (t.to(torch.bfloat16).cuda() for t in (qm, km, vm))
    om = torch.empty_like(qm)
    httm.attention(qm, km, vm, om, [0, mq], [0, mk], 0.125)
    torch.cuda.synchronize()
    want = orc.attention(f32(qm), f32(km), f32(vm))
    logits = f32(qm) @ f32(km).T * 0.125
    jump = (logits.max(axis=1) - logits[:, :32].max(axis=1)) * 1.4427
    assert (jump > 60).mean() > 0.5, "the case must actually exercise the overflow path"
    got = f32(om)
    assert np.isfinite(got).all()
    check_output(got, want, f"shift raise ({where})", relative_to_magnitude=True)


def _log2_keys(km: torch.Tensor) -> torch.Tensor:
    """bf16 keys times log2(e)/8, rounded to bf16: what stage 2 hands to httm_attention_log2."""
    return (km.float() * float(np.float32(httm.LOG2_KEY_SCALE))).to(torch.bfloat16)


def _check_log2_attention(qm, k2, vm, qo, ko, what, relative=False, value_scale=1.0):
    """httm_attention_log2 against the oracle's attention on the keys the kernel was given,
    their factor divided out again."""
    om = torch.full_like(qm, float("nan"))
    httm.attention_log2(qm, k2, vm, om, qo, ko)
    torch.cuda.synchronize()
    got = f32(om)
    assert np.isfinite(got).all(), what
    for h in range(len(qo) - 1):
        if qo[h + 1] == qo[h] or ko[h + 1] == ko[h]:
            continue
        kk = f32(k2[ko[h]:ko[h + 1]]) / np.float32(httm.LOG2_KEY_SCALE)
        want = orc.attention(f32(qm[qo[h]:qo[h + 1]]), kk, f32(vm[ko[h]:ko[h + 1]]))
        # (values of another magnitude: the bar is read in units of that magnitude)
        check_output(got[qo[h]:qo[h + 1]] / value_scale, want / value_scale, f"{what} head {h}",
                     relative_to_magnitude=relative)
    return got


@pytest.mark.parametrize("mq,mk", RAGGED + [([700, 1030, 256, 1, 300], [70, 130, 64, 200, 90])])
def test_log2_key_attention_on_ragged_heads(mq, mk):
    require_gpu()
    print(f"[case] ragged log2-key attention mq={mq} mk={mk}", flush=True)
    gen = torch.Generator().manual_seed(2000 + sum(mq))
    qo = [int(x) for x in np.concatenate([[0], np.cumsum(mq)])]
    ko = [int(x) for x in np.concatenate([[0], np.cumsum(mk)])]
    qm = torch.randn((qo[-1], 64), generator=gen).to(torch.bfloat16).cuda()
    k2 = _log2_keys(torch.randn((ko[-1], 64), generator=gen)).cuda()
    vm = torch.randn((ko[-1], 64), generator=gen).to(torch.bfloat16).cuda()
    om = torch.full_like(qm, float("nan"))
    httm.attention_log2(qm, k2, vm, om, qo, ko)
    torch.cuda.synchronize()
    for h in range(len(mq)):
        got = f32(om[qo[h]:qo[h + 1]])
        if mq[h] == 0:
            continue
        if mk[h] == 0:
            assert (got == 0).all()
            continue
        kk = f32(k2[ko[h]:ko[h + 1]]) / np.float32(httm.LOG2_KEY_SCALE)
        want = orc.attention(f32(qm[qo[h]:qo[h + 1]]), kk, f32(vm[ko[h]:ko[h + 1]]))
        check_output(got, want, f"ragged log2-key head {h} ({mq[h]}x{mk[h]})")


@pytest.mark.parametrize("case", ["huge_positive", "huge_negative", "growing", "one_head_of_three", "nan_free_zero_keys",
                                  "large_values"])
def test_log2_key_attention_leaves_the_unshifted_range(case):
    """Rows whose sum of 2^(q.k') is not inside [2^-64, 2^64] cannot use unshifted weights: their
    tiles are marked by the fast kernel and redone with per-row shifts.  The result must match the
    oracle whichever kernel computed a tile."""
    require_gpu()
    gen = torch.Generator().manual_seed(4100)
    mq, mk = 600, 900
    q = torch.randn((mq, 64), generator=gen)
    k = torch.randn((mk, 64), generator=gen)
    v = torch.randn((mk, 64), generator=gen)
    qo, ko = [0, mq], [0, mk]
    if case == "huge_positive":          # logits of several hundred log2 units
        q, k = q * 6, k * 6
    elif case == "huge_negative":        # every logit far below zero: the row sums underflow unshifted
        k = -q[:1].repeat(mk, 1) * 3 + 0.05 * k
        q = q[:1].repeat(mq, 1) * 4 + 0.05 * q
    elif case == "growing":
        k = k * torch.linspace(0.01, 60, mk)[:, None]
        q = q * 3
    elif case == "one_head_of_three":    # ordinary heads around a head that leaves the range
        q = torch.cat([q, q * 8, q])
        k = torch.cat([k, k * 8, k])
        v = torch.cat([v, v, v])
        qo, ko = [0, mq, 2 * mq, 3 * mq], [0, mk, 2 * mk, 3 * mk]
    elif case == "large_values":         # row sums near the top of the accepted range, values of 1e12
        q, k = q * 2.2, k * 2.2
        v = v * 1e12
    else:                                # zero keys: every weight is exactly 1
        k = torch.zeros_like(k)
    qm = q.to(torch.bfloat16).cuda()
    k2 = _log2_keys(k).cuda()
    vm = v.to(torch.bfloat16).cuda()
    logits2 = f32(qm[:mq]) @ f32(k2[:mk]).T
    sums = np.log2(np.exp2(logits2 - logits2.max(axis=1, keepdims=True)).sum(axis=1)) + logits2.max(axis=1)
    outside = (sums < -64) | (sums > 64)
    if case in ("huge_positive", "huge_negative", "growing"):
        assert outside.mean() > 0.5, "the case must actually leave the unshifted range"
    elif case == "nan_free_zero_keys":
        assert not outside.any()
    elif case == "large_values":
        assert (~outside).mean() > 0.5 and sums.max() > 30, "most rows must stay on the fast path, some near its top"
    _check_log2_attention(qm, k2, vm, qo, ko, f"log2 keys ({case})", relative=True,
                          value_scale=1e12 if case == "large_values" else 1.0)


def test_log2_key_attention_rewrites_a_buffer_that_holds_old_marks():
    """The output buffer of an earlier call, marks included, must not influence the next call."""
    require_gpu()
    gen = torch.Generator().manual_seed(4200)
    mq, mk = 512, 300
    qm = torch.randn((mq, 64), generator=gen).to(torch.bfloat16).cuda()
    k2 = _log2_keys(torch.randn((mk, 64), generator=gen)).cuda()
    vm = torch.randn((mk, 64), generator=gen).to(torch.bfloat16).cuda()
    om = torch.empty_like(qm)
    om.view(torch.int16).fill_(0x7FA5)               # every element looks like the redo mark
    httm.attention_log2(qm, k2, vm, om, [0, mq], [0, mk])
    torch.cuda.synchronize()
    kk = f32(k2) / np.float32(httm.LOG2_KEY_SCALE)
    check_output(f32(om), orc.attention(f32(qm), kk, f32(vm)), "old marks")


@pytest.mark.parametrize("w", [synth.workload(1), synth.workload(2)] + ODD[:2], ids=lambda w: w.name)
def test_plain_key_plans_take_the_general_kernel(w):
    """Without HTTM_FLAG_LOG2_KEYS the merged keys are the plain means and stage 3 scales in fp32."""
    require_gpu()
    q, k, v = _inputs(w)
    plan = plan_for(w, log2_keys=False)
    assert not plan.log2_keys
    got = run_stages(plan, q, k, v)
    ref = _oracle_stages(w, q, k, v)
    for h in range(w.H):
        check_assign(got["assign_k"][h].cpu().numpy(), ref["assign_k"][h], ref["gap_k"][h], f"{w.name} assign_k")
        if np.array_equal(got["assign_k"][h].cpu().numpy(), ref["assign_k"][h]):
            assert (f32(got["k_m"][h]) == round_bf16(ref["k_m"][h])).all(axis=1).mean() > 0.999
        want = orc.attention(f32(got["q_m"][h]), f32(got["k_m"][h]), f32(got["v_m"][h]))
        check_output(f32(got["o_m"][h]), want, f"{w.name} attention head {h}", relative_to_magnitude=w.index > 5)
    aq = got["assign_q"].cpu().numpy().astype(np.int64)
    got_o = f32(got["out"])
    check_output(got_o, excuse_tie_tokens(got_o, ref["O"], aq, ref), f"{w.name} plain keys, stage by stage",
                 relative_to_magnitude=w.index > 5)
    out, _ = run_layer(plan, q, k, v)
    assert torch.equal(out, got["out"])                   # the layer call = the four stages
    plan.close()


def test_bad_arguments_launch_nothing():
    require_gpu()
    w = synth.workload(1)
    q, k, v = _inputs(w)
    plan = plan_for(w)
    with pytest.raises(httm.HttmError):
        httm.reorder(plan, q, q, 0)                                   # in-place
    with pytest.raises(httm.HttmError):
        httm.reorder(plan, q[:, :100].contiguous(), torch.empty_like(q), 0)   # wrong shape
    out = torch.empty((w.N, w.H * 64), dtype=torch.bfloat16, device="cuda")
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(httm.HttmError, match="workspace"):
        httm.layer_forward(plan, q, k, v, out, small)
    with pytest.raises(httm.HttmError):
        httm.attention(q[0], k[0], v[0], torch.empty_like(q[0]), [0, w.N], [0, w.N], scale=-1.0)
    plan.close()
