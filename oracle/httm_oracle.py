"""CPU oracle for the HTTM global-attention layer (arXiv 2511.21317).

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, step-by-step NumPy
implementation of what the paper's Algorithm 1 computes, including the
adaptive outlier filter of the queries (Algorithm 2).  It exists so that the HIP kernels can be checked against something
written independently from the paper.  Only the test-suite, the smoke check and
the benchmark's CPU-baseline leg may import it; the product path never does,
and this module imports nothing from the product.

Every function takes the steps of the paper in the paper's order:

    Alg. 1 step "TemporalReorder"   -> temporal_reorder
    Alg. 1 step "Reorder"           -> reorder
    Sec. 3.2 Eq. 1 + best match,
    Alg. 1 step "BlockwiseToMe"     -> blockwise_tome  (match_block per block)
    Sec. 3.2 mean of constituents,
    Alg. 1 step "BlockAggregate"    -> block_aggregate
    Sec. 3.2 Eq. 3-4                -> attention
    Sec. 3.4 steps 2-4, Alg. 2      -> deviations, outlier_threshold,
                                       remove_outliers, block_aggregate_quantile
    Sec. 3.2 Eq. 5                  -> unmerge_by_cluster
    Alg. 1 step "InverseReorder"    -> inverse_reorder
    Sec. 3.2 Eq. 6-7 (head concat)  -> layer_forward

Arithmetic runs in `dtype` (float32 by default, the precision the acceptance
bar is stated in; float64 is accepted for cross-checks).

Readings taken where the paper is silent (all listed in the design notes):
  * a spatial block is a b x b window of patches, stacked over T consecutive
    frames (Sec. 3.3 only fixes sizes n_s and n_t); partial windows at the
    right/bottom edge and a partial last frame group are blocks of their own;
  * the 5 special tokens of each frame are never merged and sit, in (frame,
    slot) order, in front of all blocks in the reordered sequence;
  * inside a block tokens are ordered (frame, row, column);
  * a block of n tokens keeps k = max(1, n - floor(rho*n + 1e-9)) clusters
    (Alg. 1 is parameterised by a cluster number per block; in Sec. 4.1 a merge
    ratio rho means that the share 1 - rho of the tokens remains);
  * the dst tokens of a block are those at positions floor(m*n/k), m = 0..k-1;
    every other token is src and merges into its most similar dst (lowest m on
    exact ties);
  * means are taken over the raw (un-normalised) tokens; V uses K's matches;
  * no size-weighted attention bias (Eq. 3 has none);
  * general rule (dst_frac > 0): floor(dst_frac * n) strided dst per block; the r = min(floor(rho * n),
    number of src) src with the highest best-match similarity merge (ties: lower position), the others
    stay clusters of their own behind the dst clusters, in ascending position;
  * outlier filtering: the deviation is taken to the fp32 mean; "top d %" is a
    budget of floor(d * H * N) tokens and the threshold is the largest deviation
    outside that budget (strictly greater = outlier); Alg. 2's "append retained
    outliers" and Alg. 1's second attention are the same computation and the
    second form is the one written out; key outlier quantile: unused (Sec. 3.4
    filters queries only).

Parity status: every function below is pinned by tests/test_oracle_*.py
(brute force, closed forms, invariants).  The conventions above are readings,
not statements of the paper, and are therefore "parity unpinned" against the
paper's own (unpublished) code.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

EPS_NORM = 1e-12


@dataclass(frozen=True)
class Geometry:
    """Token layout of one global-attention layer and the merging block shape."""
    S: int              # frames
    Hp: int             # patch rows per frame
    Wp: int             # patch columns per frame
    b: int              # spatial block edge (patches)
    T: int              # temporal block length (frames)
    n_special: int = 5  # special tokens at the front of each frame
    anchor: bool = False  # first-frame anchoring (App. C.2): every frame-0 token is a dst
    dst_frac: float = 0.0  # > 0: the general rule of Sec. 3.2 - this share of a block's tokens are dst and
                           # only the top-r src (by best similarity) merge; 0: Alg. 1's "k clusters per
                           # block", where every src merges
    chunked: bool = False  # spatial blocks are runs of b consecutive patch tokens of a frame (row-major)
                           # instead of b x b windows: the paper's own setting n_s = 128 (Sec. 4.1)

    @property
    def tokens_per_frame(self) -> int:
        return self.n_special + self.Hp * self.Wp

    @property
    def N(self) -> int:
        return self.S * self.tokens_per_frame

    @property
    def n_prefix(self) -> int:
        return self.S * self.n_special


# --------------------------------------------------------------------------
# Alg. 1, "TemporalReorder" / "Reorder" / "InverseReorder"   (Sec. 3.3)
# --------------------------------------------------------------------------

def token_index(g: Geometry, frame: int, slot: int) -> int:
    """Position of (frame, slot) in the layer's input sequence."""
    return frame * g.tokens_per_frame + slot


def spatial_windows(g: Geometry) -> list:
    """Patch slots (row-major index y * Wp + x) of every spatial block of a frame, in block order.

    Windowed form: b x b windows of the patch grid, row-major over windows, partial at the right /
    bottom edge.  Chunked form (Sec. 4.1 "spatial block size n_s"): runs of b consecutive patch
    tokens in the frame's own token order, the last run partial.
    """
    P = g.Hp * g.Wp
    if g.chunked:
        return [list(range(c, min(P, c + g.b))) for c in range(0, P, g.b)]
    out = []
    for by in range(-(-g.Hp // g.b)):
        rows = range(by * g.b, min(g.Hp, (by + 1) * g.b))
        for bx in range(-(-g.Wp // g.b)):
            cols = range(bx * g.b, min(g.Wp, (bx + 1) * g.b))
            out.append([y * g.Wp + x for y in rows for x in cols])
    return out


def temporal_reorder(g: Geometry):
    """Permutation pi and block list of the temporal reordering (Sec. 3.3).

    pi[j] is the input position of the token that sits at reordered position
    j.  `blocks` lists (start, n) in reordered coordinates: the same spatial
    block (see spatial_windows) of every frame of a temporal group, stacked.
    """
    pi = []
    for f in range(g.S):
        for s in range(g.n_special):
            pi.append(token_index(g, f, s))
    blocks = []
    n_groups = -(-g.S // g.T)
    for grp in range(n_groups):
        frames = range(grp * g.T, min(g.S, (grp + 1) * g.T))
        for window in spatial_windows(g):
            start = len(pi)
            for f in frames:
                for slot in window:
                    pi.append(token_index(g, f, g.n_special + slot))
            blocks.append((start, len(pi) - start))
    return np.asarray(pi, dtype=np.int64), blocks


def anchor_sizes(g: Geometry) -> list:
    """Per block (same order as `temporal_reorder`): number of leading tokens forced to be dst.

    First-frame anchoring (App. C.2, "Error Mitigation"): all tokens of frame 0 are dst tokens, so
    that similar tokens of later frames merge into them.  Blocks are frame-major, hence in the
    blocks of the first temporal group the frame-0 tokens are the first (rows x cols) positions;
    every other block has none.
    """
    n_groups = -(-g.S // g.T)
    out = []
    for grp in range(n_groups):
        for window in spatial_windows(g):
            out.append(len(window) if (g.anchor and grp == 0) else 0)
    return out


def reorder(x: np.ndarray, pi: np.ndarray) -> np.ndarray:
    """x[..., L, E] -> rows gathered into block order: out[j] = x[pi[j]]."""
    return np.take(x, pi, axis=-2)


def inverse_reorder(xr: np.ndarray, pi: np.ndarray) -> np.ndarray:
    """Undo `reorder`: out[pi[j]] = xr[j]."""
    out = np.empty_like(xr)
    out[..., pi, :] = xr
    return out


# --------------------------------------------------------------------------
# Sec. 3.2 "Merging" restricted to blocks (Sec. 3.3); Alg. 1 "BlockwiseToMe"
# --------------------------------------------------------------------------

def dst_count(n: int, rho: float, n0: int = 0, dst_frac: float = 0.0) -> int:
    """Number of dst tokens of a block.  Alg. 1's rule (dst_frac = 0): as many as the block keeps.
    General rule (the src / dst partition of Sec. 3.2; the 25 % / 75 % example of Sec. 3.3):
    floor(dst_frac * n), at least one, at least the n0 anchored tokens."""
    if dst_frac <= 0.0:
        return cluster_count(n, rho, n0)
    return max(1, int(math.floor(dst_frac * n + 1e-9)), n0)


def cluster_count(n: int, rho: float, n0: int = 0, dst_frac: float = 0.0) -> int:
    """Tokens a block of n keeps when a fraction rho is merged away (M = N - r).

    With n0 anchored tokens (all of them dst) the block keeps at least those.  Under the general
    rule only src tokens can be merged away: r = min(floor(rho * n), number of src).
    """
    r = int(math.floor(rho * n + 1e-9))
    if dst_frac > 0.0:
        return n - min(r, n - dst_count(n, rho, n0, dst_frac))
    return max(1, n - r, n0)


def dst_positions(n: int, k: int, n0: int = 0) -> list:
    """Block-local positions of the k dst tokens.

    The n0 anchored tokens at the front of the block are dst; the other k - n0 dst are evenly
    strided over the remaining n - n0 tokens, the first of them included (n0 = 0: evenly strided
    over the whole block).
    """
    assert n0 <= k <= n
    return list(range(n0)) + [n0 + (m * (n - n0)) // (k - n0) for m in range(k - n0)]


def row_norm(x: np.ndarray) -> np.ndarray:
    """RowNorm of Eq. 1: every row scaled to unit L2 norm (norm clamped at 1e-12)."""
    nrm = np.sqrt(np.sum(x * x, axis=1, dtype=x.dtype))
    return x / np.maximum(nrm, x.dtype.type(EPS_NORM))[:, None]


def match_block(xb: np.ndarray, k: int, n0: int = 0, kd: int = None):
    """Bipartite matching inside one block (Eq. 1, the best-match rule and the top-r selection).

    xb: [n, E] tokens of the block, which keeps k clusters of which the first kd (default: all k)
    are its dst tokens.  The r = n - k src tokens with the highest best-match similarity (ties:
    lower position first) merge into their best dst; every other src token stays a cluster of its
    own, numbered kd, kd+1, ... in ascending position.  Returns
      cluster[n]  cluster id m in 0..k-1 of every token (a dst is its own cluster),
      score[n]    cosine similarity of a src to its best dst (1.0 for dst tokens),
      gap[n]      how far the token is from deciding otherwise: best minus second-best similarity,
                  and (when not every src merges) the distance of its score to the score on the
                  other side of the selection boundary; inf for dst tokens.
    """
    n = xb.shape[0]
    kd = k if kd is None else kd
    dpos = dst_positions(n, kd, n0)
    is_dst = np.zeros(n, dtype=bool)
    is_dst[dpos] = True
    spos = np.flatnonzero(~is_dst)
    cluster = np.empty(n, dtype=np.int64)
    score = np.ones(n, dtype=xb.dtype)
    gap = np.full(n, np.inf, dtype=xb.dtype)
    cluster[dpos] = np.arange(kd)
    if spos.size:
        sim = row_norm(xb[spos]) @ row_norm(xb[dpos]).T           # Eq. 1, [n_src, n_dst]
        best = np.argmax(sim, axis=1)                            # first maximum = lowest m
        cluster[spos] = best
        score[spos] = sim[np.arange(spos.size), best]
        if kd > 1:
            rest = sim.copy()
            rest[np.arange(spos.size), best] = -np.inf
            gap[spos] = score[spos] - rest.max(axis=1)
        r = n - k
        if r < spos.size:
            # Sec. 3.2: only the r src tokens whose best similarity is highest merge
            order = np.lexsort((spos, -score[spos]))              # score descending, then position
            merged = np.zeros(spos.size, dtype=bool)
            merged[order[:r]] = True
            stay = spos[~merged]                                 # ascending position
            cluster[stay] = kd + np.arange(stay.size)
            s_sorted = score[spos][order]
            if 0 < r:
                other = np.where(merged, s_sorted[r], s_sorted[r - 1])   # first score across the boundary
                gap[spos] = np.minimum(gap[spos], np.abs(score[spos] - other))
    return cluster, score, gap


def cluster_owners(cluster: np.ndarray, n: int, k: int, kd: int, n0: int) -> list:
    """Block-local position of the token every cluster starts from: the dst token of clusters
    0..kd-1, the (single) unmerged src token of clusters kd..k-1."""
    owners = dst_positions(n, kd, n0)
    if k > kd:
        pos = {int(c): j for j, c in enumerate(cluster) if c >= kd}
        owners = owners + [pos[m] for m in range(kd, k)]
    return owners


def merged_layout(g: Geometry, blocks, rho: float):
    """Per block: number of clusters k_b and the first merged slot of the block.

    The merged sequence is [all specials] ++ [clusters of block 0] ++ ...
    Returns (k_list, offset_list, M).
    """
    ks, offs = [], []
    pos = g.n_prefix
    for (_, n), n0 in zip(blocks, anchor_sizes(g)):
        k = cluster_count(n, rho, n0, g.dst_frac)
        ks.append(k)
        offs.append(pos)
        pos += k
    return ks, offs, pos


def dst_counts(g: Geometry, blocks, rho: float) -> list:
    """Per block: how many of its clusters are dst tokens (all of them under Alg. 1's rule)."""
    return [dst_count(n, rho, n0, g.dst_frac) for (_, n), n0 in zip(blocks, anchor_sizes(g))]


def blockwise_tome(xr: np.ndarray, g: Geometry, blocks, rho: float):
    """Cluster assignment of one head's reordered tokens (Alg. 1, "BlockwiseToMe").

    xr: [L, E] reordered tokens of one head.  Returns
      assign[L]  slot of every reordered token in this head's merged sequence,
      score[L], gap[L]  as in match_block (specials: 1.0 / inf).
    """
    L = xr.shape[0]
    ks, offs, _ = merged_layout(g, blocks, rho)
    assign = np.empty(L, dtype=np.int64)
    score = np.ones(L, dtype=xr.dtype)
    gap = np.full(L, np.inf, dtype=xr.dtype)
    assign[:g.n_prefix] = np.arange(g.n_prefix)        # specials pass through
    for (start, n), k, off, n0, kd in zip(blocks, ks, offs, anchor_sizes(g), dst_counts(g, blocks, rho)):
        c, s, gp = match_block(xr[start:start + n], k, n0, kd)
        assign[start:start + n] = off + c
        score[start:start + n] = s
        gap[start:start + n] = gp
    return assign, score, gap


# --------------------------------------------------------------------------
# Sec. 3.2: merged token = mean of its constituents; Alg. 1 "BlockAggregate"
# --------------------------------------------------------------------------

def block_aggregate(xr: np.ndarray, assign: np.ndarray, g: Geometry, blocks, rho: float) -> np.ndarray:
    """Merged tokens [M, E] of one head: mean of the dst and of every src assigned to it.

    Summation order is fixed: the dst token first, then its src tokens in
    ascending reordered position.
    """
    ks, offs, M = merged_layout(g, blocks, rho)
    out = np.zeros((M, xr.shape[1]), dtype=xr.dtype)
    count = np.zeros(M, dtype=np.int64)
    out[:g.n_prefix] = xr[:g.n_prefix]
    count[:g.n_prefix] = 1
    for (start, n), k, off, n0, kd in zip(blocks, ks, offs, anchor_sizes(g), dst_counts(g, blocks, rho)):
        dpos = cluster_owners(assign[start:start + n] - off, n, k, kd, n0)
        dset = set(dpos)
        for m, j in enumerate(dpos):
            out[off + m] = xr[start + j]
            count[off + m] = 1
        for j in range(n):
            if j in dset:
                continue
            slot = assign[start + j]
            out[slot] += xr[start + j]
            count[slot] += 1
    return out / count[:, None].astype(xr.dtype)


# --------------------------------------------------------------------------
# Sec. 3.4 "Adaptive Outlier Filtering"; Alg. 2 "BlockAggregateQuantile" (queries only)
# --------------------------------------------------------------------------

def deviations(xr: np.ndarray, assign: np.ndarray, xm: np.ndarray) -> np.ndarray:
    """Sec. 3.4 step 2: L2 distance of every token to the merged token it belongs to; zero for
    a token that is not merged with any other token (its cluster has one member)."""
    size = np.bincount(assign, minlength=xm.shape[0])
    diff = xr - xm[assign]
    eps = np.sqrt(np.sum(diff * diff, axis=1, dtype=xr.dtype))
    return np.where(size[assign] >= 2, eps, xr.dtype.type(0))


def outlier_budget(total: int, frac: float) -> int:
    """Number of tokens the top-`frac` share of `total` tokens stands for (rounded down)."""
    return int(math.floor(frac * total + 1e-9))


def outlier_threshold(eps_all: np.ndarray, frac: float) -> float:
    """Sec. 3.4 step 3 / Alg. 2 "tau <- Quantile(eps, gamma)": the threshold above which a token
    is an outlier.  Read as an order statistic: tau is the largest deviation that is NOT among the
    top floor(frac * count) values, so that at most that many tokens lie strictly above it (fewer
    when values tie with tau)."""
    flat = np.sort(np.asarray(eps_all).ravel())
    d = outlier_budget(flat.size, frac)
    if d >= flat.size:
        return -math.inf
    return float(flat[flat.size - d - 1])


def remove_outliers(xr: np.ndarray, assign: np.ndarray, xm: np.ndarray, mask: np.ndarray,
                    g: Geometry, blocks, rho: float) -> np.ndarray:
    """Sec. 3.4 step 4: the merged tokens that lose a constituent are recomputed from the
    constituents that remain (same order: the dst token first if it remains, then ascending
    position).  A merged token that loses all its constituents becomes a zero row nobody reads."""
    ks, offs, M = merged_layout(g, blocks, rho)
    out = xm.copy()
    affected = np.unique(assign[mask])
    if affected.size == 0:
        return out
    aff = np.zeros(M, dtype=bool)
    aff[affected] = True
    acc = np.zeros((M, xr.shape[1]), dtype=xr.dtype)
    cnt = np.zeros(M, dtype=np.int64)
    for (start, n), k, off, n0, kd in zip(blocks, ks, offs, anchor_sizes(g), dst_counts(g, blocks, rho)):
        if not aff[off:off + k].any():
            continue
        dpos = cluster_owners(assign[start:start + n] - off, n, k, kd, n0)
        dset = set(dpos)
        for m, j in enumerate(dpos):
            if aff[off + m] and not mask[start + j]:
                acc[off + m] = xr[start + j]
                cnt[off + m] = 1
        for j in range(n):
            slot = assign[start + j]
            if j in dset or not aff[slot] or mask[start + j]:
                continue
            acc[slot] += xr[start + j]
            cnt[slot] += 1
    for slot in affected:
        out[slot] = acc[slot] / xr.dtype.type(cnt[slot]) if cnt[slot] else 0
    return out


def block_aggregate_quantile(qr_heads, assign_heads, g: Geometry, blocks, rho: float, frac: float):
    """Alg. 2 over all heads: merged queries with the outliers taken out, and the outlier mask.

    qr_heads / assign_heads: per head, reordered queries [L, E] and their cluster slots [L].
    Returns (qm_heads, mask_heads, eps_heads, tau).  The budget floor(frac * H * L) is shared by
    all heads (Sec. 3.4 step 3).
    """
    qm0 = [block_aggregate(qr, a, g, blocks, rho) for qr, a in zip(qr_heads, assign_heads)]
    eps = [deviations(qr, a, qm) for qr, a, qm in zip(qr_heads, assign_heads, qm0)]
    tau = outlier_threshold(np.concatenate(eps), frac)
    masks = [e > tau for e in eps]
    qm = [remove_outliers(qr, a, m0, mk, g, blocks, rho)
          for qr, a, m0, mk in zip(qr_heads, assign_heads, qm0, masks)]
    return qm, masks, eps, tau


# --------------------------------------------------------------------------
# Sec. 3.2 Eq. 3-4: attention over the reduced sequences
# --------------------------------------------------------------------------

def attention(qm: np.ndarray, km: np.ndarray, vm: np.ndarray, rows=None, chunk: int = 2048) -> np.ndarray:
    """softmax(qm km^T / sqrt(E)) vm for one head.

    `rows` selects query rows (rows are independent, so a subset is exact);
    queries are processed `chunk` rows at a time only to bound memory.
    """
    dt = qm.dtype
    if rows is not None:
        qm = qm[rows]
    scale = dt.type(1.0 / math.sqrt(qm.shape[1]))
    out = np.empty((qm.shape[0], vm.shape[1]), dtype=dt)
    for r0 in range(0, qm.shape[0], chunk):
        logits = (qm[r0:r0 + chunk] @ km.T) * scale
        logits = logits - logits.max(axis=1, keepdims=True)
        p = np.exp(logits)
        p = p / p.sum(axis=1, keepdims=True)
        out[r0:r0 + chunk] = p @ vm
    return out


# --------------------------------------------------------------------------
# Sec. 3.2 Eq. 5: unmerge
# --------------------------------------------------------------------------

def unmerge_by_cluster(om: np.ndarray, assign_q: np.ndarray) -> np.ndarray:
    """Every reordered token copies the output row of the merged query it belongs to."""
    return om[assign_q]


# --------------------------------------------------------------------------
# Head-uniform comparison variant (Sec. 2.3 / Sec. 3.2: one topology for all heads)
# --------------------------------------------------------------------------

def head_mean(x: np.ndarray) -> np.ndarray:
    """Metric token of the head-uniform variant: mean over heads, summed in head order."""
    acc = x[0].copy()
    for h in range(1, x.shape[0]):
        acc = acc + x[h]
    return acc / x.dtype.type(x.shape[0])


# --------------------------------------------------------------------------
# Alg. 1 end to end (outlier filter and the two projections left out)
# --------------------------------------------------------------------------

def layer_forward(q: np.ndarray, k: np.ndarray, v: np.ndarray, g: Geometry,
                  rho_q: float, rho_kv: float, variant: str = "headwise",
                  heads=None, dtype=np.float32, outlier_frac: float = 0.0):
    """Q, K, V [H, N, E] -> dict with O [N, len(heads)*E] and every intermediate.

    variant: "headwise" (the paper's method), "uniform" (one matching for all
    heads, from head-averaged tokens), or "none" (no merging).
    `heads` restricts the computation to a subset of heads (heads are
    independent except for the uniform variant's averaged metric and the
    outlier budget, which always use all heads).
    outlier_frac > 0 switches the adaptive outlier filtering of the queries on
    (Sec. 3.4, Alg. 2; Alg. 1 "BlockAggregateQuantile" and the second attention
    for the outlier queries): results gain "eps", "outlier_mask" (per head) and "tau".
    """
    H, N, E = q.shape
    assert N == g.N
    heads = list(range(H)) if heads is None else list(heads)
    q = q.astype(dtype, copy=False)
    k = k.astype(dtype, copy=False)
    v = v.astype(dtype, copy=False)
    pi, blocks = temporal_reorder(g)
    if variant == "none":
        rho_q = rho_kv = 0.0
    if variant == "uniform":
        uq = blockwise_tome(reorder(head_mean(q), pi), g, blocks, rho_q)
        uk = blockwise_tome(reorder(head_mean(k), pi), g, blocks, rho_kv)
    res = {"pi": pi, "blocks": blocks, "assign_q": [], "assign_k": [], "gap_q": [], "gap_k": [],
           "score_q": [], "score_k": [], "q_m": [], "k_m": [], "v_m": [], "o_m": []}
    filt = None
    if outlier_frac > 0.0 and variant != "none":
        # the outlier budget is shared by all heads, so the queries of every head are matched first
        qr_all = [reorder(q[h], pi) for h in range(H)]
        aq_all = [uq if variant == "uniform" else blockwise_tome(qr_all[h], g, blocks, rho_q)
                  for h in range(H)]
        qm_all, mask_all, eps_all, tau = block_aggregate_quantile(
            qr_all, [a[0] for a in aq_all], g, blocks, rho_q, outlier_frac)
        filt = (aq_all, qm_all, mask_all)
        res.update({"eps": [eps_all[h] for h in heads], "outlier_mask": [mask_all[h] for h in heads],
                    "tau": tau})
    cols = []
    for h in heads:
        qr, kr, vr = reorder(q[h], pi), reorder(k[h], pi), reorder(v[h], pi)
        if filt is not None:
            aq, sq, gq = filt[0][h]
        elif variant == "uniform":
            aq, sq, gq = uq
        else:
            aq, sq, gq = blockwise_tome(qr, g, blocks, rho_q)
        if variant == "uniform":
            ak, sk, gk = uk
        else:
            ak, sk, gk = blockwise_tome(kr, g, blocks, rho_kv)
        qm = filt[1][h] if filt is not None else block_aggregate(qr, aq, g, blocks, rho_q)
        km = block_aggregate(kr, ak, g, blocks, rho_kv)
        vm = block_aggregate(vr, ak, g, blocks, rho_kv)
        om = attention(qm, km, vm)
        o_r = unmerge_by_cluster(om, aq)
        if filt is not None and filt[2][h].any():
            # Alg. 1: the outlier queries attend on their own, un-merged
            o_r[filt[2][h]] = attention(qr[filt[2][h]], km, vm)
        o = inverse_reorder(o_r, pi)
        cols.append(o)
        for key, val in (("assign_q", aq), ("assign_k", ak), ("gap_q", gq), ("gap_k", gk),
                         ("score_q", sq), ("score_k", sk), ("q_m", qm), ("k_m", km),
                         ("v_m", vm), ("o_m", om)):
            res[key].append(val)
    res["O"] = np.concatenate(cols, axis=1)           # Eq. 7: heads side by side on channels
    res["heads"] = heads
    return res


def rep_map(assign: np.ndarray, pi: np.ndarray, g: Geometry, blocks, rho: float) -> np.ndarray:
    """Layout-independent form of an assignment: for every INPUT position i, the input
    position of the dst token (or itself, for specials) that token i was merged into."""
    ks, offs, M = merged_layout(g, blocks, rho)
    slot_owner = np.empty(M, dtype=np.int64)
    slot_owner[:g.n_prefix] = pi[:g.n_prefix]
    for (start, n), k, off, n0, kd in zip(blocks, ks, offs, anchor_sizes(g), dst_counts(g, blocks, rho)):
        for m, j in enumerate(cluster_owners(assign[start:start + n] - off, n, k, kd, n0)):
            slot_owner[off + m] = pi[start + j]
    rep = np.empty(g.N, dtype=np.int64)
    rep[pi] = slot_owner[assign]
    return rep
