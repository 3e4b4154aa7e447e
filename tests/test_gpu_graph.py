"""httm_layer_forward under HIP graph capture: the call allocates nothing, never synchronises and
launches only kernels, so a captured layer must replay to the bits of the eager call - on every
replay, with new inputs in the captured buffers and eager work in between."""
import pytest
import torch

import paper_2511_21317_amd as httm
import synth
from gpu_util import require_gpu, plan_for

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("idx,frac", [(2, 0.0), (3, 0.0), (2, 0.1)], ids=["cfg2", "cfg3", "cfg2_filtered"])
def test_captured_layer_replays_to_the_bits_of_the_eager_call(idx, frac):
    require_gpu()
    w = synth.workload(idx)
    print(f"[case] graph capture of the layer, {w.name} outlier_frac={frac}", flush=True)
    plan = plan_for(w, outlier_frac=frac) if frac else plan_for(w)
    q, k, v = synth.make_qkv(w, device="cuda")
    ws = httm.alloc_workspace(plan)
    out = torch.empty((plan.N, plan.H * 64), dtype=torch.bfloat16, device="cuda")

    def eager(qq, kk, vv):
        o = torch.empty_like(out)
        httm.layer_forward(plan, qq, kk, vv, o, httm.alloc_workspace(plan))
        torch.cuda.synchronize()
        return o

    want = [eager(q, k, v)]                     # (also the warm-up: one-time attribute calls happen here)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        httm.layer_forward(plan, q, k, v, out, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        httm.layer_forward(plan, q, k, v, out, ws)
    gen = torch.Generator(device="cuda").manual_seed(77 + idx)
    for rep in range(3):
        if rep:
            # new tokens in the captured input buffers: a permutation of the frames' tokens plus noise
            for t in (q, k, v):
                noise = torch.randn(t.shape, generator=gen, device="cuda", dtype=torch.float32) * 0.05
                t.copy_((t.float().roll(rep * 37, dims=1) + noise).to(torch.bfloat16))
            want.append(eager(q, k, v))
        out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want[rep]), f"replay {rep} differs from the eager call"
        # eager work of the library between the replays
        httm.layer_forward(plan, q, k, v, torch.empty_like(out), httm.alloc_workspace(plan))
        torch.cuda.synchronize()
    plan.close()
