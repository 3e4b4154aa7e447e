"""httm_attention_log2_static: stage 3 (Eq. 3-4) with the library's own static scratch, for callers
that cannot allocate.  Checked through the C ABI against httm_attention_log2_scratch (the entry
point it is a variant of) bit for bit, and against the oracle on the rows that ran in pieces; two
calls in a row, the second one smaller, then a launch too large for the static array."""
import numpy as np
import pytest
import torch

import paper_2511_21317_amd as httm
from oracle import httm_oracle as orc
from gpu_util import require_gpu, f32, check_output

pytestmark = pytest.mark.gpu


def _case(mq, mk, seed):
    gen = torch.Generator().manual_seed(seed)
    qo = [int(x) for x in np.concatenate([[0], np.cumsum(mq)])]
    ko = [int(x) for x in np.concatenate([[0], np.cumsum(mk)])]
    qm = torch.randn((qo[-1], 64), generator=gen).to(torch.bfloat16)
    k2 = (torch.randn((ko[-1], 64), generator=gen) * float(np.float32(httm.LOG2_KEY_SCALE))).to(torch.bfloat16)
    vm = torch.randn((ko[-1], 64), generator=gen).to(torch.bfloat16)
    return qm.cuda(), k2.cuda(), vm.cuda(), qo, ko


def _check_against_oracle(qm, k2, vm, qo, ko, got, h, r0, r1, what):
    kk = f32(k2[ko[h]:ko[h + 1]]) / np.float32(httm.LOG2_KEY_SCALE)
    want = orc.attention(f32(qm[qo[h] + r0:qo[h] + r1]), kk, f32(vm[ko[h]:ko[h + 1]]))
    check_output(f32(got[qo[h] + r0:qo[h] + r1]), want, what)


def test_static_scratch_entry_point_matches_the_one_with_caller_scratch():
    require_gpu()
    # 8 x (64 full tiles + a partial one) = 520 tiles on 256 CUs: the 8 partial tiles run in segments;
    # then 3 x (171 full + a partial one) = 516: fewer segments, which leaves stale rows of the first
    # call in the static array; then a short launch that uses no scratch at all
    cases = [([16384 + 37, 16384 + 200, 16384 + 1, 16384 + 255, 16384 + 128, 16384 + 64, 16384 + 65, 16384 + 31],
              [4200, 4100, 5000, 4096, 7777, 4500, 6001, 8192], 7001),
             ([43776 + 100, 43776 + 31, 43776 + 255], [4100, 6000, 4097], 7002),
             ([300, 1000, 77], [500, 64, 129], 7003)]
    for i, (mq, mk, seed) in enumerate(cases):
        print(f"[case] static scratch, call {i}: mq={mq} mk={mk}", flush=True)
        qm, k2, vm, qo, ko = _case(mq, mk, seed)
        H = len(mq)
        caller = torch.full((httm.attention_scratch_bytes(H),), 0xFF, dtype=torch.uint8, device="cuda")
        want = torch.full_like(qm, float("nan"))
        httm.attention_log2(qm, k2, vm, want, qo, ko, scratch=caller)
        got = torch.full_like(qm, float("nan"))
        httm.attention_log2_static(qm, k2, vm, got, qo, ko)
        torch.cuda.synchronize()
        used = bool((caller[:4096] != 0xFF).any())
        assert used == (i < 2), "the first two launches run tiles in pieces, the third does not"
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), f"call {i}: static != caller scratch"
        for h in range(H):          # the rows of every head's last tile, against the oracle
            r0 = (mq[h] - 1) // 256 * 256
            _check_against_oracle(qm, k2, vm, qo, ko, got, h, r0, mq[h], f"call {i} head {h}")
        del caller


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    require_gpu()
    # 456 full tiles on 256 CUs against 20 000 keys: the 200 tiles in excess would run as 512 shares,
    # 711 slots = 48 MB of partial results, more than the 32 MiB array holds
    mq, mk = [456 * 256], [20000]
    plan = httm.attention_split_plan([0, mq[0]], [0, mk[0]])
    assert plan["slots"] * 256 * 66 * 4 > 32 << 20
    qm, k2, vm, qo, ko = _case(mq, mk, 7004)
    out = torch.full_like(qm, float("nan"))
    with pytest.raises(httm.HttmError, match="workspace"):
        httm.attention_log2_static(qm, k2, vm, out, qo, ko)
    torch.cuda.synchronize()
    assert torch.isnan(out.float()).all(), "a refused call launches nothing"
