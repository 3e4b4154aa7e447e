"""Stage 3 (Eq. 3-4) with scratch memory: the query tiles in excess of a multiple of the CU count run
in segments over the keys that are added up afterwards, so that any tile count fills the chip.
Checked against the oracle's attention on the rows of the tiles that ran in segments, and against
the same call without scratch on all rows."""
import numpy as np
import pytest
import torch

import paper_2511_21317_amd as httm
from oracle import httm_oracle as orc
from gpu_util import require_gpu, f32, check_output

pytestmark = pytest.mark.gpu


def _log2_keys(k):
    return (k.float() * float(np.float32(httm.LOG2_KEY_SCALE))).to(torch.bfloat16)


def _case(mq, mk, seed, key_gain=None):
    gen = torch.Generator().manual_seed(seed)
    qo = [int(x) for x in np.concatenate([[0], np.cumsum(mq)])]
    ko = [int(x) for x in np.concatenate([[0], np.cumsum(mk)])]
    qm = torch.randn((qo[-1], 64), generator=gen).to(torch.bfloat16)
    k = torch.randn((ko[-1], 64), generator=gen)
    if key_gain is not None:
        k = key_gain(k, ko)
    vm = torch.randn((ko[-1], 64), generator=gen).to(torch.bfloat16)
    return qm.cuda(), _log2_keys(k).cuda(), vm.cuda(), qo, ko


def _run_both(qm, k2, vm, qo, ko):
    H = len(qo) - 1
    plain = torch.full_like(qm, float("nan"))
    httm.attention_log2(qm, k2, vm, plain, qo, ko)
    scratch = torch.full((httm.attention_scratch_bytes(H),), 0xFF, dtype=torch.uint8, device="cuda")   # NaN bit patterns
    split = torch.full_like(qm, float("nan"))
    httm.attention_log2(qm, k2, vm, split, qo, ko, scratch=scratch)
    torch.cuda.synchronize()
    _run_both.scratch_written = bool((scratch[:4096] != 0xFF).any())   # the pieces of the first partial tile
    return f32(plain), f32(split)


def _partial_rows(qo, h):
    mq = qo[h + 1] - qo[h]
    return qo[h] + (mq // 256) * 256, qo[h + 1]


# The tiles in excess of a multiple of the 256 CUs - the partial tiles first, then full tiles from the
# end - run in segments.  Here 512 or 520 full tiles plus the partial ones; ragged lengths, one head
# without a partial tile; the last case splits 8 full tiles as well.
CASES = [
    ([16384 + 37] * 8, [8229] * 8),
    ([16384 + 1, 16384 + 255, 16384 + 128, 16384, 16384 + 64, 16384 + 65, 16384 + 200, 16384 + 31],
     [5000, 4100, 9000, 4096, 7777, 4500, 6001, 8192]),
    ([32768 + 100] * 4, [12001] * 4),
    ([16640 + 37] * 8, [8229] * 8),
]


@pytest.mark.parametrize("mq,mk", CASES)
def test_tiles_in_pieces_match_the_oracle_and_the_whole_tiles(mq, mk):
    require_gpu()
    print(f"[case] split attention mq={mq} mk={mk}", flush=True)
    qm, k2, vm, qo, ko = _case(mq, mk, 4000 + sum(mq) % 997)
    plain, split = _run_both(qm, k2, vm, qo, ko)
    assert np.isfinite(split).all()
    assert _run_both.scratch_written, "the launch did not take the split"
    # split and whole tiles differ by the fp32 rounding of the partial sums only: one bf16 step, or -
    # where the weighted values cancel to almost nothing - the fp32 noise of sums of terms of size one
    d = np.abs(split - plain)
    assert (d <= 2.0 ** -7 * np.abs(plain) + 1e-5).all(), f"{d.max()}"
    n_full = sum(m // 256 for m in mq)
    excess = (n_full + sum(1 for m in mq if m % 256)) % 256
    n_split_full = max(0, excess - sum(1 for m in mq if m % 256))
    for h in range(len(mq)):
        r0, r1 = _partial_rows(qo, h)
        if h == len(mq) - 1:
            r0 -= 256 * n_split_full            # the full tiles that are split are the last ones of the last head
        # rows of the tiles that stay whole: the same workgroups ran them
        assert np.array_equal(split[qo[h]:r0], plain[qo[h]:r0]), f"head {h}: whole tiles differ"
        if r1 == r0:
            continue
        kk = f32(k2[ko[h]:ko[h + 1]]) / np.float32(httm.LOG2_KEY_SCALE)
        want = orc.attention(f32(qm[r0:r1]), kk, f32(vm[ko[h]:ko[h + 1]]))
        check_output(split[r0:r1], want, f"split, head {h}")
        check_output(plain[r0:r1], want, f"whole, head {h}")


def test_a_partial_tile_that_leaves_the_unshifted_range_is_redone_with_shifts():
    """Keys of one piece of one head give weights far above 2^64: the sum of the pieces fails the
    window test, the tile gets the mark and the kernel with per-row shifts redoes it (whole)."""
    require_gpu()
    mq, mk = [16384 + 37] * 8, [8229] * 8

    def gain(k, ko):
        k = k.clone()
        k[ko[3] + 6000:ko[3] + 6100] *= 60.0     # head 3, inside one piece
        k[ko[5]:ko[5 + 1]] *= 0.0                # head 5: all weights 1 (row sum = number of keys)
        return k

    qm, k2, vm, qo, ko = _case(mq, mk, 4242, gain)
    plain, split = _run_both(qm, k2, vm, qo, ko)
    assert np.isfinite(split).all()
    for h in (3, 5, 0):
        r0, r1 = _partial_rows(qo, h)
        kk = f32(k2[ko[h]:ko[h + 1]]) / np.float32(httm.LOG2_KEY_SCALE)
        want = orc.attention(f32(qm[r0:r1]), kk, f32(vm[ko[h]:ko[h + 1]]))
        check_output(split[r0:r1], want, f"split, head {h}")
    r0, r1 = _partial_rows(qo, 3)
    assert np.array_equal(split[r0:r1], plain[r0:r1])     # both came from the kernel with shifts


def _split_rows(mq, mk):
    """Per head: the query rows of the tiles the library runs in segments (from its own host-side plan)."""
    qo = [int(x) for x in np.concatenate([[0], np.cumsum(mq)])]
    ko = [int(x) for x in np.concatenate([[0], np.cumsum(mk)])]
    plan = httm.attention_split_plan(qo, ko, torch.cuda.get_device_properties(0).multi_processor_count)
    rows = {h: [] for h in range(len(mq))}
    for head, q0, _, _ in plan["tiles"]:
        rows[int(head)].append(np.arange(int(q0), min(int(q0) + 256, mq[int(head)])))
    return {h: (np.concatenate(r) if r else np.zeros(0, dtype=np.int64)) for h, r in rows.items()}, plan


# 300 to 700 tiles on 256 CUs, heads of 5 to 9 thousand keys: every count leaves some CUs a tile short
# without the split.  (tiles, heads): the rows per head are tiles / heads * 256 plus a ragged bit.
TILE_COUNTS = [(300, 4), (352, 16), (400, 16), (400, 8), (530, 8), (640, 5), (700, 7)]


@pytest.mark.parametrize("tiles,H", TILE_COUNTS)
@pytest.mark.parametrize("log2", [True, False], ids=["log2_keys", "plain_keys"])
def test_any_tile_count_runs_its_excess_in_segments(tiles, H, log2):
    require_gpu()
    rng = np.random.default_rng(5000 + tiles)
    per = tiles // H
    # heads with a partial last tile (one row to 255) and, for the remainder, one more full tile
    mq = [256 * (per - 1) + int(rng.integers(1, 256)) for _ in range(H)]
    for h in range(tiles - per * H):
        mq[h] += 256
    mk = [int(rng.integers(5000, 9000)) for _ in range(H)]
    assert sum(-(-m // 256) for m in mq) == tiles
    print(f"[case] {tiles} tiles in {H} heads, log2={log2}: mq={mq} mk={mk}", flush=True)
    rows, plan = _split_rows(mq, mk)
    assert plan["n_tiles"] == tiles % 256 and plan["slots"] > 0
    if log2:
        qm, km, vm, qo, ko = _case(mq, mk, 5100 + tiles)
        plain, split = _run_both(qm, km, vm, qo, ko)
        written = _run_both.scratch_written
        kscale = np.float32(httm.LOG2_KEY_SCALE)
    else:
        qm, km, vm, qo, ko = _plain_case(mq, mk, 5100 + tiles)
        plain, split, written = _run_both_plain(qm, km, vm, qo, ko)
        kscale = np.float32(1.0)
    assert written and np.isfinite(split).all()
    # the run without scratch uses 128-row tiles when the launch fits one round of those: then only
    # the oracle is the reference; else the tiles that stay whole ran in the same workgroups
    same_kernel = sum(-(-m // 128) for m in mq) > 768
    for h in range(H):
        kk = f32(km[ko[h]:ko[h + 1]]) / kscale
        vv = f32(vm[ko[h]:ko[h + 1]])
        r = rows[h]
        if r.size:
            want = orc.attention(f32(qm[qo[h]:qo[h + 1]]), kk, vv, rows=r)
            check_output(split[qo[h]:qo[h + 1]][r], want, f"{tiles} tiles, segments, head {h}")
        whole = np.setdiff1d(np.arange(mq[h]), r)
        if same_kernel:
            assert np.array_equal(split[qo[h]:qo[h + 1]][whole], plain[qo[h]:qo[h + 1]][whole]), f"head {h}: whole tiles differ"
        if whole.size == 0:          # every tile of this head ran in segments
            continue
        sample = whole[:: max(1, whole.size // 300)]
        want = orc.attention(f32(qm[qo[h]:qo[h + 1]]), kk, vv, rows=sample)
        check_output(split[qo[h]:qo[h + 1]][sample], want, f"{tiles} tiles, whole tiles, head {h}")
    # the two runs (other tile shapes, other key ranges per piece, other shifts for the bf16 weights)
    # agree to a few bf16 steps of the result and the rounding noise of the weights
    d = np.abs(split - plain)
    assert (d <= 2.0 ** -5 * np.abs(plain) + 1e-3).all(), f"{d.max()}"


def test_launches_where_the_split_cannot_pay_and_missing_room_run_every_tile_whole():
    require_gpu()
    # a head with fewer than 512 keys: no split
    qm, k2, vm, qo, ko = _case([16384 + 37] * 8, [8229] * 7 + [300], 4345)
    plain, split = _run_both(qm, k2, vm, qo, ko)
    assert np.array_equal(plain, split) and not _run_both.scratch_written
    # a multiple of the CU count: nothing in excess
    qm, k2, vm, qo, ko = _case([16384] * 8, [4100] * 8, 4346)
    plain, split = _run_both(qm, k2, vm, qo, ko)
    assert np.array_equal(plain, split) and not _run_both.scratch_written
    qm, k2, vm, qo, ko = _case([300, 700, 129], [500, 640, 90], 4343)
    plain, split = _run_both(qm, k2, vm, qo, ko)
    assert np.array_equal(plain, split) and not _run_both.scratch_written
    L = httm.lib()
    import ctypes as C
    qo_c = (C.c_int64 * 4)(*qo)
    ko_c = (C.c_int64 * 4)(*ko)
    small = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    rc = L.httm_attention_log2_scratch(C.c_void_p(qm.data_ptr()), C.c_void_p(k2.data_ptr()), C.c_void_p(vm.data_ptr()),
                                       C.c_void_p(qm.data_ptr()), qo_c, ko_c, 3, 64, C.c_void_p(small.data_ptr()),
                                       1024, None)
    assert rc == -1      # scratch given but smaller than httm_attention_scratch_bytes(H)


# ---- the same split in httm_attention (keys without the logit scale; every row has its shift) ----

def _plain_case(mq, mk, seed, key_gain=None):
    gen = torch.Generator().manual_seed(seed)
    qo = [int(x) for x in np.concatenate([[0], np.cumsum(mq)])]
    ko = [int(x) for x in np.concatenate([[0], np.cumsum(mk)])]
    qm = torch.randn((qo[-1], 64), generator=gen).to(torch.bfloat16)
    k = torch.randn((ko[-1], 64), generator=gen)
    if key_gain is not None:
        k = key_gain(k, ko)
    vm = torch.randn((ko[-1], 64), generator=gen).to(torch.bfloat16)
    return qm.cuda(), k.to(torch.bfloat16).cuda(), vm.cuda(), qo, ko


def _run_both_plain(qm, km, vm, qo, ko):
    H = len(qo) - 1
    plain = torch.full_like(qm, float("nan"))
    httm.attention(qm, km, vm, plain, qo, ko, 0.125)
    scratch = torch.full((httm.attention_scratch_bytes(H),), 0xFF, dtype=torch.uint8, device="cuda")
    split = torch.full_like(qm, float("nan"))
    httm.attention(qm, km, vm, split, qo, ko, 0.125, scratch=scratch)
    torch.cuda.synchronize()
    return f32(plain), f32(split), bool((scratch[:4096] != 0xFF).any())


def _gain_one_piece(k, ko):
    k = k.clone()
    k[ko[3] + 6000:ko[3] + 6100] *= 30.0     # head 3: one piece's shift far above the others'
    k[ko[5]:ko[5 + 1]] *= 0.0                # head 5: all weights equal
    return k


@pytest.mark.parametrize("mq,mk,gain", [(CASES[1][0], CASES[1][1], None), (CASES[3][0], CASES[3][1], None),
                                        (CASES[0][0], CASES[0][1], _gain_one_piece)])
def test_pieces_with_per_row_shifts_match_the_oracle_and_the_whole_tiles(mq, mk, gain):
    require_gpu()
    print(f"[case] split attention, plain keys mq={mq} mk={mk} gain={gain is not None}", flush=True)
    qm, km, vm, qo, ko = _plain_case(mq, mk, 4600 + sum(mq) % 997, gain)
    plain, split, written = _run_both_plain(qm, km, vm, qo, ko)
    assert np.isfinite(split).all()
    assert written, "the launch did not take the split"
    # the pieces round their weights to bf16 relative to their own shifts: a few 2^-9 steps of terms
    # that average out, and one bf16 step of the result
    # (with the amplified keys a row is dominated by a few keys with values of size one: the 2^-9
    # rounding of their weights, relative to other shifts in the two runs, shows in full where the
    # weighted values cancel)
    d = np.abs(split - plain)
    assert (d <= 2.0 ** -6 * np.abs(plain) + (5e-3 if gain is not None else 2e-4)).all(), f"{d.max()}"
    n_full = sum(m // 256 for m in mq)
    n_part = sum(1 for m in mq if m % 256)
    n_split_full = max(0, (n_full + n_part) % 256 - n_part)
    for h in range(len(mq)):
        r0, r1 = _partial_rows(qo, h)
        if h == len(mq) - 1:
            r0 -= 256 * n_split_full
        assert np.array_equal(split[qo[h]:r0], plain[qo[h]:r0]), f"head {h}: whole tiles differ"
        if r1 == r0:
            continue
        want = orc.attention(f32(qm[r0:r1]), f32(km[ko[h]:ko[h + 1]]), f32(vm[ko[h]:ko[h + 1]]))
        check_output(split[r0:r1], want, f"split, head {h}")
        check_output(plain[r0:r1], want, f"whole, head {h}")


def test_plain_keys_short_launch_takes_no_split():
    require_gpu()
    qm, km, vm, qo, ko = _plain_case([300, 700, 129], [500, 640, 90], 4343)
    plain, split, written = _run_both_plain(qm, km, vm, qo, ko)
    assert np.array_equal(plain, split) and not written
