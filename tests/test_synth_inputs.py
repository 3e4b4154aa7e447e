"""The seeded synthetic workloads have the stated shapes and the structure the paper reports
(Sec. 3.1: spatial locality and temporal correspondence of the tokens)."""
import numpy as np
import torch

import synth
from synth.vggt_tokens import bf16_to_f32_numpy


def test_shapes_and_determinism():
    w = synth.workload(1)
    q, k, v = synth.make_qkv(w)
    assert w.N == 522 and q.shape == (16, 522, 64) and q.dtype == torch.bfloat16
    q2, k2, v2 = synth.make_qkv(w)
    assert torch.equal(q, q2) and torch.equal(k, k2) and torch.equal(v, v2)
    assert [synth.workload(i).N for i in range(1, 6)] == [522, 10992, 25024, 137400, 274800]
    x = bf16_to_f32_numpy(q)
    assert 0.7 < x.std() < 1.4          # ~unit variance so that logits/8 have ~unit std


def test_neighbours_and_next_frame_are_similar():
    w = synth.workload(1)
    q, _, _ = synth.make_qkv(w)
    x = bf16_to_f32_numpy(q)[3]
    x = x / np.linalg.norm(x, axis=1, keepdims=True)
    tpf = w.tokens_per_frame
    grid0 = x[5:tpf].reshape(w.Hp, w.Wp, -1)
    grid1 = x[tpf + 5:2 * tpf].reshape(w.Hp, w.Wp, -1)
    near = (grid0[:, :-1] * grid0[:, 1:]).sum(-1).mean()
    far = (grid0[:, :8] * grid0[:, 8:]).sum(-1).mean()
    # best temporal correspondence over the allowed shifts {-1,0,1}^2
    temporal = max((grid0 * np.roll(grid1, (dy, dx), axis=(0, 1))).sum(-1).mean()
                   for dy in (-2, -1, 0, 1, 2) for dx in (-2, -1, 0, 1, 2))
    assert near > 0.6 and near > far + 0.3
    assert temporal > 0.8
