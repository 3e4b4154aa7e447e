"""ctypes binding of libhttm.so.  Argument marshalling only: every step of the path runs in
the HIP kernels behind the C ABI declared in include/httm.h.  torch is used for device memory
and the current stream, nothing else.  There is no CPU fallback: if the library is missing or
a call fails, an exception is raised."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libhttm.so")   # the library built in-tree; nothing else is ever loaded

VARIANT_HEADWISE, VARIANT_UNIFORM, VARIANT_NONE = 0, 1, 2
VARIANTS = {"headwise": VARIANT_HEADWISE, "uniform": VARIANT_UNIFORM, "none": VARIANT_NONE}
MAX_BLOCK = 4096
MAX_HEADS = 64


class HttmError(RuntimeError):
    pass


class Geom(C.Structure):
    _fields_ = [("S", C.c_int32), ("Hp", C.c_int32), ("Wp", C.c_int32), ("n_special", C.c_int32),
                ("H", C.c_int32), ("d_head", C.c_int32), ("b", C.c_int32), ("T", C.c_int32),
                ("rho_q", C.c_double), ("rho_kv", C.c_double), ("variant", C.c_int32),
                ("flags", C.c_int32), ("outlier_frac", C.c_double), ("dst_frac", C.c_double)]


class Sizes(C.Structure):
    _fields_ = [(n, C.c_int64) for n in
                ("N", "n_prefix", "n_blocks", "max_block", "M_q", "M_k", "workspace_bytes", "outlier_cap")]


class WorkspaceLayout(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("q_m", "k_m", "v_m", "o_m", "assign_q", "assign_k", "eps_q",
                                         "q_out", "o_out", "attn_split", "total")]


_lib = None


def lib() -> C.CDLL:
    """Load libhttm.so (built in-tree by paper_2511_21317_amd.build) or raise."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise HttmError(f"{LIB_PATH} is missing: run `python -m paper_2511_21317_amd.build` "
                        "(or __graft_entry__.build()) first; there is no fallback path")
    L = C.CDLL(LIB_PATH)
    vp, i32p, i64p, f32p = C.c_void_p, C.c_void_p, C.POINTER(C.c_int64), C.c_void_p
    L.httm_version.restype = C.c_int
    L.httm_strerror.restype = C.c_char_p
    L.httm_strerror.argtypes = [C.c_int]
    L.httm_last_hip_error.restype = C.c_int
    L.httm_geom_sizes.argtypes = [C.POINTER(Geom), C.POINTER(Sizes)]
    L.httm_workspace_layout.argtypes = [C.POINTER(Geom), C.POINTER(WorkspaceLayout)]
    L.httm_geom_tables.argtypes = [C.POINTER(Geom)] + [vp] * 7
    L.httm_geom_block_forms.argtypes = [C.POINTER(Geom), vp, vp]
    L.httm_plan_create.argtypes = [C.POINTER(Geom), C.POINTER(vp)]
    L.httm_plan_clone.argtypes = [vp, C.POINTER(vp)]
    L.httm_plan_destroy.argtypes = [vp]
    L.httm_plan_query.argtypes = [vp, C.POINTER(Sizes)]
    L.httm_reorder.argtypes = [vp, vp, vp, C.c_int, vp]
    L.httm_match_merge.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32p, i32p, f32p, f32p, vp]
    L.httm_reorder_match_merge.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32p, i32p, f32p, f32p, vp]
    L.httm_attention.argtypes = [vp, vp, vp, vp, i64p, i64p, C.c_int, C.c_int, C.c_float, vp]
    L.httm_attention_scratch.argtypes = [vp, vp, vp, vp, i64p, i64p, C.c_int, C.c_int, C.c_float, vp, C.c_int64, vp]
    L.httm_attention_log2.argtypes = [vp, vp, vp, vp, i64p, i64p, C.c_int, C.c_int, vp]
    L.httm_attention_log2_scratch.argtypes = [vp, vp, vp, vp, i64p, i64p, C.c_int, C.c_int, vp, C.c_int64, vp]
    L.httm_attention_log2_static.argtypes = [vp, vp, vp, vp, i64p, i64p, C.c_int, C.c_int, vp]
    L.httm_attention_split_plan.argtypes = [i64p, i64p, C.c_int, C.c_int, vp, vp, C.c_int64, vp, C.c_int64]
    L.httm_attention_scratch_bytes.argtypes = [C.c_int]
    L.httm_attention_scratch_bytes.restype = C.c_int64
    L.httm_unmerge.argtypes = [vp, vp, i32p, vp, C.c_int, vp]
    L.httm_layer_forward.argtypes = [vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    L.httm_reorder_match_merge_filtered.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32p, i32p, f32p, vp, vp]
    L.httm_attention_outliers.argtypes = [vp, vp, vp, vp, vp, vp]
    L.httm_unmerge_filtered.argtypes = [vp, vp, vp, i32p, vp, vp]
    L.httm_outlier_stats.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_int32), vp]
    L.httm_global_match.argtypes = [vp, C.c_int64, C.c_int, C.c_int, C.c_double, i32p, f32p, vp]
    for name in ("httm_geom_sizes", "httm_workspace_layout", "httm_geom_tables", "httm_geom_block_forms", "httm_plan_create", "httm_plan_clone",
                 "httm_plan_destroy", "httm_plan_query", "httm_reorder", "httm_match_merge",
                 "httm_reorder_match_merge",
                 "httm_attention", "httm_attention_scratch", "httm_attention_log2", "httm_attention_log2_scratch", "httm_attention_log2_static", "httm_attention_split_plan", "httm_unmerge", "httm_layer_forward",
                 "httm_reorder_match_merge_filtered", "httm_attention_outliers", "httm_unmerge_filtered",
                 "httm_outlier_stats", "httm_global_match"):
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _check(rc: int, what: str):
    if rc != 0:
        L = lib()
        msg = L.httm_strerror(rc).decode()
        extra = f" (hipError_t {L.httm_last_hip_error()})" if rc == -4 else ""
        raise HttmError(f"{what} failed: {msg}{extra} [code {rc}]")


FLAG_ANCHOR_FIRST_FRAME = 1
FLAG_CHUNKED_BLOCKS = 2
FLAG_LOG2_KEYS = 4
LOG2_KEY_SCALE = 0.125 * 1.4426950408889634   # log2(e) / sqrt(64): the factor the scaled keys carry


def make_geom(S, Hp, Wp, b, T, rho_q, rho_kv=None, *, H=16, d_head=64, n_special=5,
              variant="headwise", anchor_first_frame=False, outlier_frac=0.0, chunked_blocks=False,
              dst_frac=0.0, log2_keys=False) -> Geom:
    if rho_kv is None:
        rho_kv = rho_q
    v = VARIANTS[variant] if isinstance(variant, str) else int(variant)
    flags = ((FLAG_ANCHOR_FIRST_FRAME if anchor_first_frame else 0) | (FLAG_CHUNKED_BLOCKS if chunked_blocks else 0)
             | (FLAG_LOG2_KEYS if log2_keys else 0))
    return Geom(S, Hp, Wp, n_special, H, d_head, b, T, float(rho_q), float(rho_kv), v, flags,
                float(outlier_frac), float(dst_frac))


def geom_sizes(g: Geom) -> Sizes:
    s = Sizes()
    _check(lib().httm_geom_sizes(C.byref(g), C.byref(s)), "httm_geom_sizes")
    return s


def workspace_layout(g: Geom) -> WorkspaceLayout:
    w = WorkspaceLayout()
    _check(lib().httm_workspace_layout(C.byref(g), C.byref(w)), "httm_workspace_layout")
    return w


def geom_tables(g: Geom) -> dict:
    """Host index tables of a geometry as int32 NumPy arrays (no GPU needed)."""
    s = geom_sizes(g)
    out = {"pi": np.empty(s.N, np.int32)}
    for name in ("block_start", "block_n", "block_kq", "block_kk", "block_offq", "block_offk"):
        out[name] = np.empty(s.n_blocks, np.int32)
    ptr = lambda a: a.ctypes.data_as(C.c_void_p)  # noqa: E731
    _check(lib().httm_geom_tables(C.byref(g), ptr(out["pi"]), ptr(out["block_start"]),
                                  ptr(out["block_n"]), ptr(out["block_kq"]), ptr(out["block_kk"]),
                                  ptr(out["block_offq"]), ptr(out["block_offk"])), "httm_geom_tables")
    return out


def geom_block_forms(g: Geom) -> dict:
    """The reorder inside every merging block in closed form (int32 NumPy arrays, no GPU needed)."""
    s = geom_sizes(g)
    out = {"block_src0": np.empty(s.n_blocks, np.int32), "block_dims": np.empty(s.n_blocks, np.int32)}
    ptr = lambda a: a.ctypes.data_as(C.c_void_p)  # noqa: E731
    _check(lib().httm_geom_block_forms(C.byref(g), ptr(out["block_src0"]), ptr(out["block_dims"])),
           "httm_geom_block_forms")
    return out


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype, shape=None) -> C.c_void_p:
    if not t.is_cuda:
        raise HttmError("tensor must live on the GPU")
    if t.dtype != dtype:
        raise HttmError(f"expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise HttmError("tensor must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise HttmError(f"expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return C.c_void_p(t.data_ptr())


class Plan:
    """Owns an httm_plan_t (device index tables of one geometry)."""

    def __init__(self, g: Geom, _clone_of=None):
        self.geom = g
        self._h = C.c_void_p()
        if _clone_of is None:
            _check(lib().httm_plan_create(C.byref(g), C.byref(self._h)), "httm_plan_create")
        else:
            _check(lib().httm_plan_clone(_clone_of._h, C.byref(self._h)), "httm_plan_clone")
        self.sizes = Sizes()
        _check(lib().httm_plan_query(self._h, C.byref(self.sizes)), "httm_plan_query")
        self.layout = workspace_layout(g)

    def clone(self) -> "Plan":
        """A second plan of the same geometry with buffers of its own (for a second stream)."""
        return Plan(self.geom, _clone_of=self)

    def close(self):
        if self._h:
            lib().httm_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # convenience
    @property
    def N(self): return int(self.sizes.N)
    @property
    def M_q(self): return int(self.sizes.M_q)
    @property
    def M_k(self): return int(self.sizes.M_k)
    @property
    def H(self): return int(self.geom.H)
    @property
    def outlier_cap(self): return int(self.sizes.outlier_cap)
    @property
    def log2_keys(self): return bool(self.geom.flags & FLAG_LOG2_KEYS)


def reorder(plan: Plan, src: torch.Tensor, dst: torch.Tensor, direction: int = 0):
    shape = (plan.H, plan.N, 64)
    _check(lib().httm_reorder(plan._h, _dev(src, torch.bfloat16, shape), _dev(dst, torch.bfloat16, shape),
                              int(direction), _stream()), "httm_reorder")
    return dst


def match_merge(plan: Plan, q_r, k_r, v_r, q_m, k_m, v_m, assign_q, assign_k, score_q=None, score_k=None):
    H, N = plan.H, plan.N
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    _check(lib().httm_match_merge(
        plan._h, _dev(q_r, bf, (H, N, 64)), _dev(k_r, bf, (H, N, 64)), _dev(v_r, bf, (H, N, 64)),
        _dev(q_m, bf, (H, plan.M_q, 64)), _dev(k_m, bf, (H, plan.M_k, 64)), _dev(v_m, bf, (H, plan.M_k, 64)),
        _dev(assign_q, i32, (H, N)), _dev(assign_k, i32, (H, N)),
        _dev(score_q, f32, (H, N)) if score_q is not None else None,
        _dev(score_k, f32, (H, N)) if score_k is not None else None, _stream()), "httm_match_merge")


def reorder_match_merge(plan: Plan, q, k, v, q_m, k_m, v_m, assign_q, assign_k, score_q=None, score_k=None):
    H, N = plan.H, plan.N
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    _check(lib().httm_reorder_match_merge(
        plan._h, _dev(q, bf, (H, N, 64)), _dev(k, bf, (H, N, 64)), _dev(v, bf, (H, N, 64)),
        _dev(q_m, bf, (H, plan.M_q, 64)), _dev(k_m, bf, (H, plan.M_k, 64)), _dev(v_m, bf, (H, plan.M_k, 64)),
        _dev(assign_q, i32, (H, N)), _dev(assign_k, i32, (H, N)),
        _dev(score_q, f32, (H, N)) if score_q is not None else None,
        _dev(score_k, f32, (H, N)) if score_k is not None else None, _stream()), "httm_reorder_match_merge")


def attention(q_m, k_m, v_m, o_m, q_offsets, k_offsets, scale: float = 0.125, scratch=None):
    """q_m/o_m: [sum M_q, 64] (or [H, M, 64]) bf16; offsets: sequences of H+1 row indices (host).
    scratch: a uint8 device tensor of at least attention_scratch_bytes(H) bytes, or None."""
    H = len(q_offsets) - 1
    qo = (C.c_int64 * (H + 1))(*[int(x) for x in q_offsets])
    ko = (C.c_int64 * (H + 1))(*[int(x) for x in k_offsets])
    bf = torch.bfloat16
    if scratch is None:
        _check(lib().httm_attention(_dev(q_m, bf), _dev(k_m, bf), _dev(v_m, bf), _dev(o_m, bf), qo, ko,
                                    H, 64, float(scale), _stream()), "httm_attention")
    else:
        _check(lib().httm_attention_scratch(_dev(q_m, bf), _dev(k_m, bf), _dev(v_m, bf), _dev(o_m, bf), qo, ko,
                                            H, 64, float(scale), _dev(scratch, torch.uint8), scratch.numel(),
                                            _stream()), "httm_attention_scratch")
    return o_m


def attention_split_plan(q_offsets, k_offsets, compute_units: int = 256) -> dict:
    """How stage 3 with scratch cuts a launch with these head lengths (host only, no GPU needed)."""
    H = len(q_offsets) - 1
    qo = (C.c_int64 * (H + 1))(*[int(x) for x in q_offsets])
    ko = (C.c_int64 * (H + 1))(*[int(x) for x in k_offsets])
    summary = np.zeros(8, np.int32)
    ptr = lambda a: a.ctypes.data_as(C.c_void_p)  # noqa: E731
    _check(lib().httm_attention_split_plan(qo, ko, H, int(compute_units), ptr(summary), None, 0, None, 0),
           "httm_attention_split_plan")
    names = ("n_tiles", "shares", "share_units", "span", "slots", "units", "kept_full", "split_ragged")
    out = {n: int(v) for n, v in zip(names, summary)}
    seg = np.zeros((out["slots"], 5), np.int32)
    tiles = np.zeros((out["n_tiles"], 4), np.int32)
    _check(lib().httm_attention_split_plan(qo, ko, H, int(compute_units), ptr(summary), ptr(seg), seg.shape[0],
                                           ptr(tiles), tiles.shape[0]), "httm_attention_split_plan")
    out["segments"], out["tiles"] = seg, tiles
    return out


def attention_scratch_bytes(H: int) -> int:
    return int(lib().httm_attention_scratch_bytes(int(H)))


def attention_log2(q_m, k_log2, v_m, o_m, q_offsets, k_offsets, scratch=None):
    """As attention(), for keys that carry the factor LOG2_KEY_SCALE (a plan with log2_keys).
    scratch: a uint8 device tensor of at least attention_scratch_bytes(H) bytes, or None."""
    H = len(q_offsets) - 1
    qo = (C.c_int64 * (H + 1))(*[int(x) for x in q_offsets])
    ko = (C.c_int64 * (H + 1))(*[int(x) for x in k_offsets])
    bf = torch.bfloat16
    if scratch is None:
        _check(lib().httm_attention_log2(_dev(q_m, bf), _dev(k_log2, bf), _dev(v_m, bf), _dev(o_m, bf), qo, ko,
                                         H, 64, _stream()), "httm_attention_log2")
    else:
        _check(lib().httm_attention_log2_scratch(_dev(q_m, bf), _dev(k_log2, bf), _dev(v_m, bf), _dev(o_m, bf),
                                                 qo, ko, H, 64, _dev(scratch, torch.uint8),
                                                 scratch.numel(), _stream()), "httm_attention_log2_scratch")
    return o_m


def attention_log2_static(q_m, k_log2, v_m, o_m, q_offsets, k_offsets):
    """attention_log2() with the library's own static scratch (httm_attention_log2_static): no
    allocation anywhere in the call."""
    H = len(q_offsets) - 1
    qo = (C.c_int64 * (H + 1))(*[int(x) for x in q_offsets])
    ko = (C.c_int64 * (H + 1))(*[int(x) for x in k_offsets])
    bf = torch.bfloat16
    _check(lib().httm_attention_log2_static(_dev(q_m, bf), _dev(k_log2, bf), _dev(v_m, bf), _dev(o_m, bf), qo, ko,
                                            H, 64, _stream()), "httm_attention_log2_static")
    return o_m


def unmerge(plan: Plan, o_m, assign_q, out, fuse_inverse_reorder: bool = True):
    H, N = plan.H, plan.N
    shape = (N, H * 64) if fuse_inverse_reorder else (H, N, 64)
    _check(lib().httm_unmerge(plan._h, _dev(o_m, torch.bfloat16, (H, plan.M_q, 64)),
                              _dev(assign_q, torch.int32, (H, N)), _dev(out, torch.bfloat16, shape),
                              1 if fuse_inverse_reorder else 0, _stream()), "httm_unmerge")
    return out


def layer_forward(plan: Plan, q, k, v, out, workspace):
    H, N = plan.H, plan.N
    bf = torch.bfloat16
    if workspace.dtype != torch.uint8:
        raise HttmError("workspace must be a uint8 tensor")
    _check(lib().httm_layer_forward(plan._h, _dev(q, bf, (H, N, 64)), _dev(k, bf, (H, N, 64)),
                                    _dev(v, bf, (H, N, 64)), _dev(out, bf, (N, H * 64)),
                                    _dev(workspace, torch.uint8), workspace.numel(), _stream()),
           "httm_layer_forward")
    return out


def workspace_views(plan: Plan, workspace: torch.Tensor) -> dict:
    """Typed views of the regions of the workspace of httm_layer_forward."""
    L, H, N = plan.layout, plan.H, plan.N
    def bf(off, rows):
        return workspace[off:off + H * rows * 128].view(torch.bfloat16).view(H, rows, 64)
    def i32(off):
        return workspace[off:off + H * N * 4].view(torch.int32).view(H, N)
    views = {"q_m": bf(L.q_m, plan.M_q), "k_m": bf(L.k_m, plan.M_k), "v_m": bf(L.v_m, plan.M_k),
             "o_m": bf(L.o_m, plan.M_q), "assign_q": i32(L.assign_q), "assign_k": i32(L.assign_k)}
    cap = plan.outlier_cap
    if cap:
        views["eps_q"] = workspace[L.eps_q:L.eps_q + H * N * 4].view(torch.float32).view(H, N)
        views["q_out"] = workspace[L.q_out:L.q_out + cap * 128].view(torch.bfloat16).view(cap, 64)
        views["o_out"] = workspace[L.o_out:L.o_out + cap * 128].view(torch.bfloat16).view(cap, 64)
    views["attn_split"] = workspace[L.attn_split:L.attn_split + attention_scratch_bytes(H)]   # stage 3's scratch
    return views


def reorder_match_merge_filtered(plan: Plan, q, k, v, q_m, k_m, v_m, assign_q, assign_k, eps_q, q_out):
    """Stage 2 with the adaptive outlier filter (plans with outlier_frac > 0)."""
    H, N = plan.H, plan.N
    bf, i32, f32 = torch.bfloat16, torch.int32, torch.float32
    _check(lib().httm_reorder_match_merge_filtered(
        plan._h, _dev(q, bf, (H, N, 64)), _dev(k, bf, (H, N, 64)), _dev(v, bf, (H, N, 64)),
        _dev(q_m, bf, (H, plan.M_q, 64)), _dev(k_m, bf, (H, plan.M_k, 64)), _dev(v_m, bf, (H, plan.M_k, 64)),
        _dev(assign_q, i32, (H, N)), _dev(assign_k, i32, (H, N)), _dev(eps_q, f32, (H, N)),
        _dev(q_out, bf, (plan.outlier_cap, 64)), _stream()), "httm_reorder_match_merge_filtered")


def attention_outliers(plan: Plan, q_out, k_m, v_m, o_out):
    bf = torch.bfloat16
    cap = plan.outlier_cap
    _check(lib().httm_attention_outliers(plan._h, _dev(q_out, bf, (cap, 64)),
                                         _dev(k_m, bf, (plan.H, plan.M_k, 64)),
                                         _dev(v_m, bf, (plan.H, plan.M_k, 64)),
                                         _dev(o_out, bf, (cap, 64)), _stream()), "httm_attention_outliers")
    return o_out


def unmerge_filtered(plan: Plan, o_m, o_out, assign_q, out):
    H, N = plan.H, plan.N
    bf = torch.bfloat16
    _check(lib().httm_unmerge_filtered(plan._h, _dev(o_m, bf, (H, plan.M_q, 64)),
                                       _dev(o_out, bf, (plan.outlier_cap, 64)),
                                       _dev(assign_q, torch.int32, (H, N)), _dev(out, bf, (N, H * 64)),
                                       _stream()), "httm_unmerge_filtered")
    return out


def outlier_stats(plan: Plan):
    """(tau, outliers per head) of the last filtered stage 2 on this plan; waits for the stream."""
    tau = C.c_float()
    counts = (C.c_int32 * plan.H)()
    _check(lib().httm_outlier_stats(plan._h, C.byref(tau), counts, _stream()), "httm_outlier_stats")
    return float(tau.value), [int(c) for c in counts]


def global_match(x, dst_frac: float, best_dst, sim=None):
    """Un-blocked matching of x [H, N, 64] (Sec. 3.3's comparison point): best_dst / sim [H, N]."""
    H, N = int(x.shape[0]), int(x.shape[1])
    _check(lib().httm_global_match(_dev(x, torch.bfloat16, (H, N, 64)), N, H, 64, float(dst_frac),
                                   _dev(best_dst, torch.int32, (H, N)),
                                   _dev(sim, torch.float32, (H, N)) if sim is not None else None, _stream()),
           "httm_global_match")
    return best_dst


def alloc_workspace(plan: Plan) -> torch.Tensor:
    return torch.empty(int(plan.sizes.workspace_bytes), dtype=torch.uint8, device="cuda")
