"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side index tables agree with the oracle's (written independently, in Python)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2511_21317_amd as httm
from oracle import httm_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "httm.h")).read()
    return sorted(set(re.findall(r"HTTM_API\s+[\w\s\*]+?\b(httm_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 14 and "httm_layer_forward" in names and "httm_attention" in names
    L = httm.lib()
    for n in names:
        assert hasattr(L, n), f"libhttm.so does not export {n}"
    assert L.httm_version() == 100
    assert b"workspace" in L.httm_strerror(-3)


def test_the_benchmark_probe_library_loads_and_rejects_bad_arguments():
    """libhttm_probe.so is bench.py's measurement helper (a register-only MFMA loop), built next to the
    library; without a GPU only its argument check can run (no launch happens before it)."""
    path = os.path.join(ROOT, "paper_2511_21317_amd", "libhttm_probe.so")
    assert os.path.exists(path), "build() did not produce the probe library"
    L = C.CDLL(path)
    L.httm_probe_mfma_bf16.restype = C.c_double
    L.httm_probe_mfma_bf16.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    assert L.httm_probe_mfma_bf16(None, 10, 1, None) == 0.0
    assert L.httm_probe_mfma_bf16(C.c_void_p(256), 0, 1, None) == 0.0
    assert L.httm_probe_mfma_bf16(C.c_void_p(256), 10, 9, None) == 0.0


GEOMS = [
    (2, 16, 16, 4, 2, 0.5, 0.5),
    (8, 37, 37, 4, 2, 0.5, 0.5),
    (32, 21, 37, 4, 4, 0.75, 0.75),
    (100, 37, 37, 4, 4, 0.8, 0.8),
    (200, 37, 37, 8, 4, 0.9, 0.9),
    (3, 5, 7, 4, 2, 0.6, 0.3),
    (5, 3, 3, 8, 7, 0.9, 0.0),
]


CHUNKED_GEOMS = [
    (8, 37, 37, 128, 4, 0.9, 0.7),      # runs of 128 tokens (Sec. 4.1), 10 full + one of 89 per frame
    (5, 6, 7, 10, 2, 0.5, 0.5),
    (3, 4, 4, 64, 3, 0.75, 0.25),       # a run longer than the frame
]


@pytest.mark.parametrize("anchor", [False, True], ids=["plain", "anchored"])
@pytest.mark.parametrize("case", GEOMS + CHUNKED_GEOMS)
def test_host_tables_match_oracle(case, anchor):
    S, Hp, Wp, b, T, rq, rk = case
    chunked = case in CHUNKED_GEOMS
    g = httm.make_geom(S, Hp, Wp, b, T, rq, rk, anchor_first_frame=anchor, chunked_blocks=chunked)
    og = orc.Geometry(S, Hp, Wp, b, T, anchor=anchor, chunked=chunked)
    t = httm.geom_tables(g)
    s = httm.geom_sizes(g)
    pi, blocks = orc.temporal_reorder(og)
    assert s.N == og.N and s.n_prefix == og.n_prefix and s.n_blocks == len(blocks)
    assert np.array_equal(t["pi"], pi)
    assert t["block_start"].tolist() == [b_[0] for b_ in blocks]
    assert t["block_n"].tolist() == [b_[1] for b_ in blocks]
    kq, oq, Mq = orc.merged_layout(og, blocks, rq)
    kk, ok, Mk = orc.merged_layout(og, blocks, rk)
    assert t["block_kq"].tolist() == kq and t["block_offq"].tolist() == oq and s.M_q == Mq
    assert t["block_kk"].tolist() == kk and t["block_offk"].tolist() == ok and s.M_k == Mk
    assert s.max_block == max(n for _, n in blocks)
    w = httm.workspace_layout(g)
    assert w.total == s.workspace_bytes
    assert w.k_m - w.q_m >= 16 * Mq * 128 and w.assign_k - w.assign_q >= 16 * og.N * 4
    assert all(getattr(w, f) % 256 == 0 for f in ("q_m", "k_m", "v_m", "o_m", "assign_q", "assign_k"))


@pytest.mark.parametrize("anchor", [False, True], ids=["plain", "anchored"])
@pytest.mark.parametrize("case", GEOMS + CHUNKED_GEOMS + [(200, 37, 37, 8, 4, 0.9, 0.9), (7, 9, 5, 4, 3, 0.5, 0.5)])
def test_closed_form_of_the_reorder_inside_a_block(case, anchor):
    """Sec. 3.3: a block is frames x grid rows x columns, frame-major.  The kernels that read tokens in
    the caller's order use that closed form instead of pi; here it is evaluated with integer
    arithmetic for every token of every block and compared with the oracle's permutation, and every
    block must have one (else the kernels would fall back to index loads)."""
    S, Hp, Wp, b, T, rq, rk = case
    chunked = case in CHUNKED_GEOMS
    g = httm.make_geom(S, Hp, Wp, b, T, rq, rk, anchor_first_frame=anchor, chunked_blocks=chunked)
    og = orc.Geometry(S, Hp, Wp, b, T, anchor=anchor, chunked=chunked)
    pi, blocks = orc.temporal_reorder(og)
    f = httm.geom_block_forms(g)
    assert len(blocks) == len(f["block_dims"]) and (f["block_dims"] != 0).all()
    tpf = og.n_special + Hp * Wp
    row_len = Hp * Wp if chunked else Wp
    for (start, n), src0, dims in zip(blocks, f["block_src0"].tolist(), f["block_dims"].tolist()):
        nx, plane = dims & 0xFFFF, dims >> 16
        r = np.arange(n)
        want = src0 + (r // plane) * tpf + ((r % plane) // nx) * row_len + r % nx
        assert np.array_equal(want, pi[start:start + n])
    L = httm.lib()
    assert L.httm_geom_block_forms(C.byref(g), None, None) == -1


def test_closed_form_of_the_reorder_on_random_geometries():
    """60 seeded draws of frames, grid, block shape / kind, special-token count and anchoring: the
    closed form reproduces the library's own pi, which test_host_tables_match_oracle pins to the oracle."""
    rng = np.random.default_rng(20251121)
    for _ in range(60):
        chunked = bool(rng.integers(0, 2))
        S, Hp, Wp = int(rng.integers(1, 12)), int(rng.integers(1, 40)), int(rng.integers(1, 40))
        b = int(rng.integers(1, 300)) if chunked else int(rng.integers(1, 12))
        T = int(rng.integers(1, 7))
        ns = int(rng.choice([0, 1, 5]))
        g = httm.make_geom(S, Hp, Wp, b, T, 0.5, n_special=ns, chunked_blocks=chunked,
                           anchor_first_frame=bool(rng.integers(0, 2)))
        sz = httm.Sizes()
        if httm.lib().httm_geom_sizes(C.byref(g), C.byref(sz)) != 0:
            continue                                   # (a block larger than the library takes)
        t, f = httm.geom_tables(g), httm.geom_block_forms(g)
        tpf, row_len = ns + Hp * Wp, (Hp * Wp if chunked else Wp)
        assert (f["block_dims"] != 0).all(), (S, Hp, Wp, b, T, ns, chunked)
        for start, n, src0, dims in zip(t["block_start"].tolist(), t["block_n"].tolist(),
                                        f["block_src0"].tolist(), f["block_dims"].tolist()):
            nx, plane = dims & 0xFFFF, dims >> 16
            r = np.arange(n)
            want = src0 + (r // plane) * tpf + ((r % plane) // nx) * row_len + r % nx
            assert np.array_equal(want, t["pi"][start:start + n]), (S, Hp, Wp, b, T, ns, chunked)


def test_merged_lengths_of_the_five_workloads():
    want = {1: 266, 2: 5516, 3: 6376, 4: 28650, 5: 28700}   # tests/golden/merged_counts.txt
    import synth
    for i, M in want.items():
        w = synth.workload(i)
        s = httm.geom_sizes(httm.make_geom(w.S, w.Hp, w.Wp, w.b, w.T, w.rho))
        assert (s.M_q, s.M_k, s.N) == (M, M, w.N)
    none = httm.geom_sizes(httm.make_geom(8, 37, 37, 4, 2, 0.5, variant="none"))
    assert none.M_q == none.N == 10992


@pytest.mark.parametrize("case", [(8, 37, 37, 4, 2, 0.5, 0.5, 0.25), (3, 5, 7, 4, 2, 0.9, 0.3, 0.25),
                                  (5, 6, 7, 10, 2, 0.6, 0.0, 0.5)])
def test_host_tables_with_a_fixed_dst_share(case):
    """Sec. 3.2's general rule: a block keeps n - min(floor(rho n), number of src) clusters."""
    S, Hp, Wp, b, T, rq, rk, df = case
    g = httm.make_geom(S, Hp, Wp, b, T, rq, rk, dst_frac=df)
    og = orc.Geometry(S, Hp, Wp, b, T, dst_frac=df)
    t, s = httm.geom_tables(g), httm.geom_sizes(g)
    _, blocks = orc.temporal_reorder(og)
    kq, oq, Mq = orc.merged_layout(og, blocks, rq)
    kk, ok, Mk = orc.merged_layout(og, blocks, rk)
    assert t["block_kq"].tolist() == kq and t["block_offq"].tolist() == oq and s.M_q == Mq
    assert t["block_kk"].tolist() == kk and t["block_offk"].tolist() == ok and s.M_k == Mk
    L, sz = httm.lib(), httm.Sizes()
    big = httm.make_geom(8, 32, 32, 16, 4, 0.5, dst_frac=0.25)           # 1024-token blocks, and head-uniform
    assert L.httm_geom_sizes(C.byref(big), C.byref(sz)) == 0
    big = httm.make_geom(8, 32, 32, 16, 4, 0.5, dst_frac=0.25, variant="uniform")
    assert L.httm_geom_sizes(C.byref(big), C.byref(sz)) == 0
    bad = httm.make_geom(8, 16, 16, 4, 2, 0.5, dst_frac=1.5)
    assert L.httm_geom_sizes(C.byref(bad), C.byref(sz)) == -1
    assert L.httm_global_match(None, 10, 1, 64, 0.25, None, None, None) == -1


def test_outlier_budget_and_workspace_regions():
    """Sec. 3.4 step 3: the budget is floor(d * H * N); its three workspace regions exist only then."""
    g0 = httm.make_geom(8, 37, 37, 4, 2, 0.5)
    g1 = httm.make_geom(8, 37, 37, 4, 2, 0.5, outlier_frac=0.02)
    s0, s1 = httm.geom_sizes(g0), httm.geom_sizes(g1)
    assert s0.outlier_cap == 0 and s1.outlier_cap == orc.outlier_budget(16 * 10992, 0.02) == 3517
    w0, w1 = httm.workspace_layout(g0), httm.workspace_layout(g1)
    assert w0.eps_q == w0.q_out == w0.o_out == w0.attn_split
    assert w1.q_out - w1.eps_q >= 16 * 10992 * 4 and w1.o_out - w1.q_out >= 3517 * 128
    assert w1.attn_split - w1.o_out >= 3517 * 128 and w1.total == s1.workspace_bytes
    # stage 3's scratch region: a slot of 256 rows x (64 + 2) fp32 for each of the at most 512 shares +
    # 255 tiles in excess - 1 segments of a launch
    assert httm.attention_scratch_bytes(16) == (512 + 255) * 256 * 66 * 4
    for w in (w0, w1):
        assert w.total - w.attn_split >= httm.attention_scratch_bytes(16) and w.attn_split % 256 == 0
    assert httm.geom_sizes(httm.make_geom(8, 37, 37, 4, 2, 0.5, variant="none", outlier_frac=0.1)).outlier_cap == 0
    L, s = httm.lib(), httm.Sizes()
    for bad_frac in (-0.1, 0.6, float("nan")):
        bad = httm.make_geom(8, 37, 37, 4, 2, 0.5, outlier_frac=bad_frac)
        assert L.httm_geom_sizes(C.byref(bad), C.byref(s)) == -1
    # the filtered entry points refuse a missing plan before touching the GPU
    assert L.httm_reorder_match_merge_filtered(None, None, None, None, None, None, None, None, None,
                                               None, None, None) == -1
    assert L.httm_attention_outliers(None, None, None, None, None, None) == -1
    assert L.httm_unmerge_filtered(None, None, None, None, None, None) == -1


def test_argument_errors_are_reported_not_crashed():
    L = httm.lib()
    s = httm.Sizes()
    bad = httm.make_geom(2, 16, 16, 4, 2, 0.5, d_head=128)
    assert L.httm_geom_sizes(C.byref(bad), C.byref(s)) == -2
    bad = httm.make_geom(2, 16, 16, 16, 4, 0.5)            # 16*16*2 = 512 ok; 4 frames clipped to S=2
    assert L.httm_geom_sizes(C.byref(bad), C.byref(s)) == 0
    big = httm.make_geom(8, 32, 32, 16, 4, 0.5)            # 1024-token block: the two-kernel path
    assert L.httm_geom_sizes(C.byref(big), C.byref(s)) == 0
    bad = httm.make_geom(32, 32, 32, 16, 32, 0.5)          # 8192-token block
    assert L.httm_geom_sizes(C.byref(bad), C.byref(s)) == -2
    ok = httm.make_geom(8, 32, 32, 16, 4, 0.5, variant="uniform")    # head-uniform matching of big blocks: fine
    assert L.httm_geom_sizes(C.byref(ok), C.byref(s)) == 0
    ok = httm.make_geom(8, 32, 32, 16, 4, 0.5, outlier_frac=0.1)     # outlier filtering of big blocks: fine
    assert L.httm_geom_sizes(C.byref(ok), C.byref(s)) == 0
    bad = httm.make_geom(2, 16, 16, 4, 2, 1.5)
    assert L.httm_geom_sizes(C.byref(bad), C.byref(s)) == -1
    bad = httm.make_geom(0, 16, 16, 4, 2, 0.5)
    assert L.httm_geom_sizes(C.byref(bad), C.byref(s)) == -1
    bad = httm.make_geom(2, 16, 16, 4, 2, 0.5)
    bad.flags = 64                                           # a flag bit this library does not know
    assert L.httm_geom_sizes(C.byref(bad), C.byref(s)) == -1
    assert L.httm_geom_sizes(None, C.byref(s)) == -1
    # compute entry points reject null pointers before touching the GPU
    assert L.httm_reorder(None, None, None, 0, None) == -1
    assert L.httm_layer_forward(None, None, None, None, None, None, 0, None) == -1
    off = (C.c_int64 * 2)(0, 4)
    assert L.httm_attention(None, None, None, None, off, off, 1, 32, 0.125, None) == -2
    assert L.httm_attention(None, None, None, None, off, off, 1, 64, 0.125, None) == -1
    with pytest.raises(httm.HttmError):
        httm.geom_sizes(httm.make_geom(2, 16, 16, 4, 2, -0.1))
