/*
 * libhttm - HTTM (Head-wise Temporal Token Merging, arXiv 2511.21317) global-attention
 * layer for AMD MI355X (gfx950).  C ABI.
 *
 * The library computes the hot path of the paper's Algorithm 1 (App. D.1) between the QKV
 * projection and the output projection:
 *
 *   temporal reorder -> block-wise matching -> aggregation -> attention -> unmerge -> inverse reorder
 *
 * and, switched on through the geometry, the adaptive outlier filtering of the queries (Sec. 3.4,
 * Alg. 2: httm_geom_t.outlier_frac), first-frame anchoring (App. C.2), the paper's own block shape
 * (runs of n_s tokens x n_t frames, Sec. 4.1) and the general src/dst rule of Sec. 3.2 with top-r
 * selection (httm_geom_t.dst_frac).  HTTM_FLAG_LOG2_KEYS selects the faster stage-3 path: the
 * merged keys leave stage 2 with the logit scale folded in (same softmax, Eq. 3-4).
 *
 * Conventions common to every call
 *   - All tensor pointers are DEVICE pointers unless a parameter says "host".  Tensors are
 *     dense, row-major, 16-byte aligned, bf16 (bfloat16) unless stated otherwise.
 *   - The caller owns every tensor and the workspace.  The library owns only the plan and the
 *     small device index tables inside it (allocated in httm_plan_create, freed in
 *     httm_plan_destroy).  No other call allocates, frees or synchronises.
 *   - Every compute call is asynchronous on the HIP stream passed as `stream`
 *     (a hipStream_t cast to void*; NULL is the default stream).
 *   - Inputs are never modified.  In-place operation is not supported.  A plan with
 *     outlier_frac > 0 keeps the threshold and the outlier row offsets in its own device memory:
 *     calls that use such a plan must not overlap in time.
 *   - Return value: 0 (HTTM_OK) on success, a negative HTTM_E_* code otherwise.  Nothing
 *     aborts or throws across this boundary.  Argument checks happen on the host before
 *     any kernel is launched; a call that returns an error has launched nothing.
 *
 * Token layout (Sec. 3.2-3.3 of the paper; the frame layout follows VGGT):
 *   N = S * (n_special + Hp*Wp) tokens.  Token i = frame * (n_special + Hp*Wp) + slot;
 *   slots 0..n_special-1 are special tokens, slot n_special + y*Wp + x is patch (row y, col x).
 *   Per-head tensors are [H, N, d_head]; the layer output is [N, H*d_head].
 *
 * Reordered layout (Sec. 3.3, "Temporal Reordering"):
 *   [ all S*n_special specials in (frame, slot) order ] ++ [ merging blocks ].
 *   A merging block is a b x b window of patches stacked over T consecutive frames, blocks are
 *   ordered (frame group, window row, window col), tokens inside a block (frame, row, col).
 *   Windows at the right/bottom edge and the last frame group may be partial.
 *   (HTTM_FLAG_CHUNKED_BLOCKS: runs of b consecutive patch tokens of a frame instead of windows.)
 *
 * Merged layout (Sec. 3.2, "Merging", restricted to blocks as in Sec. 3.3 / Alg. 1):
 *   a block of n tokens keeps k = max(1, n - floor(rho*n + 1e-9)) clusters; its dst tokens are
 *   the block positions floor(m*n/k), m = 0..k-1; every other token (src) joins the dst with
 *   the highest cosine similarity (Eq. 1; lowest m on ties).  A merged token is the mean of
 *   its constituents.  The merged sequence of a head is
 *   [ specials, unmerged ] ++ [ the k clusters of block 0 ] ++ [ block 1 ] ...
 *   with length M = S*n_special + sum of k.  Q and K are matched independently per head
 *   (Eq. 2); V follows K's matches.
 *   (HTTM_FLAG_ANCHOR_FIRST_FRAME and dst_frac > 0 change which tokens are dst and how many
 *   clusters a block keeps; see there.)
 */
#ifndef HTTM_H
#define HTTM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HTTM_VERSION 100

#if defined(__GNUC__)
#define HTTM_API __attribute__((visibility("default")))
#else
#define HTTM_API
#endif

enum {
  HTTM_OK = 0,
  HTTM_E_INVALID_ARG = -1,        /* null pointer, misaligned pointer, non-positive size, bad enum */
  HTTM_E_UNSUPPORTED = -2,        /* d_head != 64, block of more than HTTM_MAX_BLOCK tokens, H > HTTM_MAX_HEADS,
                                     N >= 2^25 tokens per head */
  HTTM_E_WORKSPACE_TOO_SMALL = -3,
  HTTM_E_HIP = -4,                /* a HIP runtime call failed; see httm_last_hip_error() */
  HTTM_E_NO_DEVICE = -5,          /* no usable GPU */
  HTTM_E_OUT_OF_MEMORY = -6       /* host memory ran out while the index tables were built */
};

enum {
  HTTM_VARIANT_HEADWISE = 0,      /* the paper's method: every head matches on its own tokens (Sec. 3.2) */
  HTTM_VARIANT_UNIFORM = 1,       /* comparison: one matching for all heads, computed on the head-averaged
                                     tokens (the single topology for every head that Sec. 3.2 argues against) */
  HTTM_VARIANT_NONE = 2           /* no merging (rho ignored): plain multi-head attention, Eq. 3-4 with M = N */
};

/* First-frame anchoring (App. C.2, "Error Mitigation"): every patch token of frame 0 is a dst token,
 * so that similar tokens of the later frames of the first temporal group merge into them and
 * frame 0 itself is never merged away.  A block of the first group keeps max(k, n0) clusters, n0 its
 * frame-0 tokens; its other dst tokens are strided over the rest of the block.  Applies to Q and K. */
#define HTTM_FLAG_ANCHOR_FIRST_FRAME 1
/* Chunked spatial blocks (Sec. 4.1, "spatial block size n_s"): a spatial block is a run of b
 * consecutive patch tokens of a frame, in the frame's own (row-major) token order, the last run of a
 * frame partial - instead of a b x b window of the patch grid.  The paper's setting is b = 128, T = 30. */
#define HTTM_FLAG_CHUNKED_BLOCKS 2
/* Log2 keys: stage 2 multiplies the fp32 mean of every key cluster by log2(e) / sqrt(d_head) before
 * its one rounding to bf16, so that q . k' is the logit of Eq. 3 in base-2 units and stage 3 can use
 * the weights 2^(q . k') without a multiplication per score (httm_attention_log2; the same softmax,
 * Eq. 3-4).  A key that is a cluster of its own is rounded once where it would otherwise be copied.
 * With the flag, k_m of the stage-2 calls and of the layer's workspace holds these scaled keys, and
 * httm_layer_forward / httm_attention_outliers take the faster stage-3 path. */
#define HTTM_FLAG_LOG2_KEYS 4

#define HTTM_MAX_OUTLIER_FRAC 0.5
#define HTTM_MAX_BLOCK 4096       /* largest merging block (n_s*n_t tokens) the kernels accept; blocks of more
                                     than 512 tokens (the paper's 128 x 30 = 3840, Sec. 4.1) take a two-kernel path */
#define HTTM_MAX_HEADS 64

/* Problem description.  Plain data, filled by the caller. */
typedef struct httm_geom {
  int32_t S;          /* frames */
  int32_t Hp;         /* patch rows per frame */
  int32_t Wp;         /* patch columns per frame */
  int32_t n_special;  /* special tokens at the front of every frame (5 for VGGT); never merged */
  int32_t H;          /* attention heads */
  int32_t d_head;     /* channels per head; must be 64 */
  int32_t b;          /* spatial block edge in patches (n_s = b*b); with HTTM_FLAG_CHUNKED_BLOCKS: n_s itself */
  int32_t T;          /* temporal block length in frames (n_t) */
  double rho_q;       /* fraction of each block's query tokens merged away, 0 <= rho < 1 or 1 */
  double rho_kv;      /* the same for key/value tokens */
  int32_t variant;    /* HTTM_VARIANT_* */
  int32_t flags;      /* HTTM_FLAG_* bits; unknown bits are rejected */
  double outlier_frac; /* adaptive outlier filtering of the queries (Sec. 3.4): the share d of all H*N
                          query tokens - those that lie farthest from their merged token, over all
                          heads together - that is taken out of the merging again; 0 = off,
                          at most HTTM_MAX_OUTLIER_FRAC.  Ignored for HTTM_VARIANT_NONE. */
  double dst_frac;    /* 0: Alg. 1's rule - a block keeps k clusters, all of them dst tokens, and every src
                         merges.  > 0 (at most 1): the general rule of Sec. 3.2 - floor(dst_frac * n) tokens
                         of a block are dst (at least one), and only the r = min(floor(rho * n), number of
                         src) src tokens with the highest best-match similarity merge (ties: lower
                         position first); the other src stay clusters of their own, placed behind the
                         block's dst clusters in ascending position.  Any block size, both variants. */
} httm_geom_t;

/* Sizes derived from a geometry. */
typedef struct httm_sizes {
  int64_t N;                /* tokens per head */
  int64_t n_prefix;         /* S * n_special */
  int64_t n_blocks;         /* merging blocks per head */
  int64_t max_block;        /* tokens in the largest block */
  int64_t M_q;              /* merged query length per head */
  int64_t M_k;              /* merged key/value length per head */
  int64_t workspace_bytes;  /* what httm_layer_forward needs */
  int64_t outlier_cap;      /* floor(outlier_frac * H * N): the most outlier queries there can be (0 = off) */
} httm_sizes_t;

typedef struct httm_plan httm_plan_t;

/* ---- host-only helpers (no GPU needed) --------------------------------------------- */

HTTM_API int httm_version(void);
HTTM_API const char* httm_strerror(int code);
/* hipError_t of the most recent failing HIP call on this thread (0 if none). */
HTTM_API int httm_last_hip_error(void);

/* Fill *out from *g.  Host only. */
HTTM_API int httm_geom_sizes(const httm_geom_t* g, httm_sizes_t* out);

/* Write the index tables of a geometry into caller-provided HOST arrays (any may be NULL):
 *   pi[N]            input position of the token at reordered position j   (Alg. 1, TemporalReorder)
 *   block_start[n_blocks], block_n[n_blocks]   block extents in reordered coordinates
 *   block_kq[n_blocks], block_kk[n_blocks]     clusters kept per block for Q and for K/V
 *   block_offq[n_blocks], block_offk[n_blocks] first merged slot of the block, for Q and for K/V
 */
HTTM_API int httm_geom_tables(const httm_geom_t* g, int32_t* pi, int32_t* block_start, int32_t* block_n,
                     int32_t* block_kq, int32_t* block_kk, int32_t* block_offq, int32_t* block_offk);

/* The reorder inside every merging block in closed form, as the kernels that read tokens in the
 * caller's order use it instead of pi (Sec. 3.3: a block is a run of frames x grid rows x columns,
 * frame-major).  HOST arrays of n_blocks entries each, both required:
 *   block_src0[b]   input position of the block's first token
 *   block_dims[b]   n_x | (plane << 16): token r of the block is the input token
 *                   block_src0[b] + (r / plane) * tpf + ((r % plane) / n_x) * row_len + r % n_x,
 *                   tpf = n_special + Hp*Wp tokens per frame, row_len = Wp (Hp*Wp with
 *                   HTTM_FLAG_CHUNKED_BLOCKS) slots per row of the patch grid;
 *                   0 where the form does not reproduce pi (the kernels then read pi). */
HTTM_API int httm_geom_block_forms(const httm_geom_t* g, int32_t* block_src0, int32_t* block_dims);

/* ---- plan ---------------------------------------------------------------------------- */

/* Build the index tables of *g on the current HIP device.  Allocates a few int32 per token of
 * device memory (for HTTM_VARIANT_UNIFORM also 2*N*d_head floats for the head-averaged tokens; for
 * dst_frac > 0 on blocks of more than 512 tokens 2*H*N floats for the similarities the selection
 * reads when the caller passes no score arrays).  Synchronous.  The plan may be used by any number of
 * later calls, but two calls that use these buffers (or those of the outlier filter) must not run
 * concurrently: they share them. */
HTTM_API int httm_plan_create(const httm_geom_t* g, httm_plan_t** out);
/* A second plan of the same geometry with device buffers of its own (on the current device), for a
 * second stream: calls on the two plans may overlap freely.  Costs what httm_plan_create costs. */
HTTM_API int httm_plan_clone(const httm_plan_t* plan, httm_plan_t** out);
HTTM_API int httm_plan_destroy(httm_plan_t* plan);
HTTM_API int httm_plan_query(const httm_plan_t* plan, httm_sizes_t* out);

/* ---- stage 1: temporal reordering (Sec. 3.3; Alg. 1 "Reorder" / "InverseReorder") ----- */

/* direction 0: dst[h][j] = src[h][pi[j]]      (gather into block order)
 * direction 1: dst[h][pi[j]] = src[h][j]      (back to input order)
 * src, dst: [H, N, d_head] bf16, distinct buffers. */
HTTM_API int httm_reorder(const httm_plan_t* plan, const void* src, void* dst, int direction, void* stream);

/* ---- stage 2: block-wise matching and aggregation (Sec. 3.2 Eq. 1-2; Alg. 1
 *      "BlockwiseToMe" + "BlockAggregate") ------------------------------------------------- */

/* q_r, k_r, v_r : [H, N, d_head] bf16, REORDERED layout (output of httm_reorder).
 * q_m           : [H, M_q, d_head] bf16 out, merged queries.
 * k_m, v_m      : [H, M_k, d_head] bf16 out, merged keys / values (V merged with K's matches).
 * assign_q      : [H, N] int32 out; assign_q[h][j] = slot in 0..M_q-1 of reordered token j.
 * assign_k      : [H, N] int32 out; the same for keys.
 * score_q/k     : [H, N] float out or NULL; cosine similarity of token j to the dst it joined
 *                 (1.0 for dst and special tokens).
 * Similarities are fp32 sums of exact bf16 products; means are fp32 sums taken in a fixed
 * order (dst first, then src in ascending position) and rounded once to bf16, so results are
 * run-to-run identical. */
HTTM_API int httm_match_merge(const httm_plan_t* plan, const void* q_r, const void* k_r, const void* v_r,
                     void* q_m, void* k_m, void* v_m, int32_t* assign_q, int32_t* assign_k,
                     float* score_q, float* score_k, void* stream);

/* Stages 1 + 2 in one pass: the same computation on tensors in INPUT token order; the kernel
 * gathers each block's rows through pi, so no reordered copy of Q/K/V is ever written.
 * q, k, v : [H, N, d_head] bf16, input order.  Outputs exactly as httm_match_merge (assign_*
 * and score_* are indexed by REORDERED position j), bit-identical to
 * httm_reorder x3 followed by httm_match_merge. */
HTTM_API int httm_reorder_match_merge(const httm_plan_t* plan, const void* q, const void* k, const void* v,
                             void* q_m, void* k_m, void* v_m, int32_t* assign_q, int32_t* assign_k,
                             float* score_q, float* score_k, void* stream);

/* Un-blocked ("global") matching, the comparison point of Sec. 3.3 and Table 3: the whole sequence of
 * a head is one merging block.  kd = max(1, floor(dst_frac * N)) tokens at positions floor(m * N / kd)
 * are dst; Eq. 1 and the best-match rule over all N x kd pairs (about dst_frac * (1 - dst_frac) * N^2 *
 * d_head multiply-adds per head - the "0.19 N^2 d_head" of Sec. 3.3 at 25 %).  Matching only: it is
 * here to be timed against the block-local stage 2.
 * x        : [H, N, d_head] bf16, any token order.  N * kd pairs; N < 2^24 (else HTTM_E_UNSUPPORTED).
 * best_dst : [H, N] int32 out; index 0..kd-1 of the most similar dst (lowest index on exact ties);
 *            a dst token gets its own index.
 * sim      : [H, N] float out or NULL; that cosine similarity (1.0 for dst tokens). */
HTTM_API int httm_global_match(const void* x, int64_t N, int H, int d_head, double dst_frac,
                               int32_t* best_dst, float* sim, void* stream);

/* ---- stage 3: attention over the reduced sequences (Sec. 3.2 Eq. 3-4) ------------------- */

/* o = softmax(q k^T * scale) v, per head, non-causal, no mask.
 * Packed ragged layout: head h owns rows [q_offsets[h], q_offsets[h+1]) of q_m / o_m and rows
 * [k_offsets[h], k_offsets[h+1]) of k_m / v_m.  q_offsets, k_offsets are HOST arrays of H+1
 * non-decreasing int64 row indices (they are copied into the kernel arguments).
 * A head with no keys writes zeros; a head with no queries writes nothing.
 * d_head must be 64; H <= HTTM_MAX_HEADS; every head shorter than 2^24 rows.  bf16 in/out, fp32
 * softmax state and accumulation. */
HTTM_API int httm_attention(const void* q_m, const void* k_m, const void* v_m, void* o_m,
                   const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                   float scale, void* stream);

/* The same attention for keys that carry the logit scale (HTTM_FLAG_LOG2_KEYS):
 *   o = sum_j 2^(q . k'_j) v_j / sum_j 2^(q . k'_j)      (= Eq. 3-4 for k' = k * log2(e) / sqrt(d_head)).
 * Arguments and layout as for httm_attention, without `scale`.  Rows whose weights would leave the
 * fp32 range without a per-row shift are detected and recomputed with one, so the result is defined
 * for any finite input; the fast path covers row sums between 2^-64 and 2^64. */
HTTM_API int httm_attention_log2(const void* q_m, const void* k_log2, const void* v_m, void* o_m,
                                 const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                                 void* stream);

/* httm_attention_log2 with scratch memory (device, 16-byte aligned, scratch_bytes >=
 * httm_attention_scratch_bytes(H); its contents before and after the call are meaningless).  A
 * launch ends when its last workgroup ends, and a compute unit runs whole 256-row query tiles: T
 * tiles on C compute units take ceil(T / C) tile times.  With scratch, the T mod C tiles in excess
 * of a multiple of C - the partial last tiles of the heads first, then full tiles from the end - are
 * not run whole: their work is cut into equal shares over the keys, one or two per compute unit,
 * that run behind the whole tiles, and a second kernel adds the pieces of every tile up (in key
 * order: run-to-run identical), so that any tile count fills the chip.  Launches too short for the
 * split to pay (it costs about 15 us) run as without scratch.  The results agree with
 * httm_attention_log2 to fp32 rounding of the sums.  httm_layer_forward does the same with the
 * attn_split region of its workspace.
 * httm_attention_scratch is httm_attention with the same scratch and the same rule; there every
 * piece keeps the shift its sums are relative to, and the pieces of a row are brought to the
 * largest of their shifts before they are added. */
HTTM_API int64_t httm_attention_scratch_bytes(int H);
HTTM_API int httm_attention_log2_scratch(const void* q_m, const void* k_log2, const void* v_m, void* o_m,
                                         const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                                         void* scratch, int64_t scratch_bytes, void* stream);
HTTM_API int httm_attention_scratch(const void* q_m, const void* k_m, const void* v_m, void* o_m,
                                    const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                                    float scale, void* scratch, int64_t scratch_bytes, void* stream);

/* Host only (no GPU needed): how stage 3 with scratch cuts a launch with these head lengths on a
 * device of `compute_units` compute units - the very functions the kernels evaluate; for tests and
 * diagnostics.  HOST arrays:
 *   summary[8]  : tiles that run in pieces (0: none), shares, key tiles (of 64 keys) per share,
 *                 most tiles a share touches, slots of scratch (256 rows x 66 fp32 each), key tiles of
 *                 all split tiles together, full tiles that stay whole, partial tiles that are split
 *   segments    : or NULL; 5 int32 per slot (one workgroup each, at most max_segments): head, first
 *                 query row, key tiles [t0, t1) of the head's sequence (t0 >= t1: the slot is unused,
 *                 its workgroup has nothing to do), slot
 *   tiles       : or NULL; 4 int32 per split tile (at most max_tiles): head, first query row, first
 *                 and last share that left a piece of it (their slots are share + tile index) */
HTTM_API int httm_attention_split_plan(const int64_t* q_offsets, const int64_t* k_offsets, int H, int compute_units,
                                       int32_t* summary, int32_t* segments, int64_t max_segments,
                                       int32_t* tiles, int64_t max_tiles);

/* httm_attention_log2_scratch for callers that cannot allocate device memory and have no buffer to
 * pass: code that runs under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The scratch is an array of HTTM_STATIC_SCRATCH_BYTES inside the library's device code
 * (every GPU the library has run on holds its copy until the process ends); the call allocates and
 * frees nothing.  Arguments, layout and results as httm_attention_log2_scratch (bit-identical to
 * it).  A launch whose partial results need more than the array holds is refused with
 * HTTM_E_WORKSPACE_TOO_SMALL and nothing is launched: use httm_attention_log2_scratch with a buffer
 * of the caller, or httm_attention_log2, which needs none.  All calls on one GPU share the array:
 * two of them that overlap in time (two streams) race - serialise them.  Its contents between
 * calls are meaningless; every call writes what it later reads.  The first call on a device looks up
 * the array's address (not capturable: make one call before capturing). */
#define HTTM_STATIC_SCRATCH_BYTES (32ll << 20)
HTTM_API int httm_attention_log2_static(const void* q_m, const void* k_log2, const void* v_m, void* o_m,
                                        const int64_t* q_offsets, const int64_t* k_offsets, int H, int d_head,
                                        void* stream);

/* ---- stage 4: unmerge (Sec. 3.2 Eq. 5-7) and inverse reorder (Sec. 3.3) ------------------ */

/* o_m      : [H, M_q, d_head] bf16, attention output per merged query.
 * assign_q : [H, N] int32 from httm_match_merge.
 * fuse_inverse_reorder != 0:  out is [N, H*d_head] in INPUT token order, heads concatenated on
 *     channels:  out[pi[j]][h*d_head + c] = o_m[h][assign_q[h][j]][c].
 * fuse_inverse_reorder == 0:  out is [H, N, d_head] in REORDERED order:
 *     out[h][j] = o_m[h][assign_q[h][j]]   (follow with httm_reorder(..., 1, ...)).
 * A plan with outlier_frac > 0 is refused (HTTM_E_INVALID_ARG): the assignment its stage 2 writes
 * refers to rows of o_out as well, which only httm_unmerge_filtered takes. */
HTTM_API int httm_unmerge(const httm_plan_t* plan, const void* o_m, const int32_t* assign_q, void* out,
                 int fuse_inverse_reorder, void* stream);

/* ---- the whole layer (Alg. 1 between the two projections; with the outlier filter of Sec. 3.4
 *      when the plan's outlier_frac > 0) ---------------------------------------------------- */

/* q, k, v : [H, N, d_head] bf16 in INPUT token order.  out : [N, H*d_head] bf16.
 * workspace: at least httm_sizes_t.workspace_bytes bytes, 256-byte aligned.  After the call it
 * holds, in this order (each 256-byte aligned): q_m, k_m, v_m, o_m ([H, M, d_head] bf16),
 * assign_q, assign_k ([H, N] int32) and, with outlier filtering, eps_q, q_out, o_out - see
 * httm_workspace_layout.
 * The reorder is fused into the matching kernel's loads and the inverse reorder into the
 * unmerge kernel's stores; results are identical to calling the four stages one by one. */
HTTM_API int httm_layer_forward(const httm_plan_t* plan, const void* q, const void* k, const void* v,
                       void* out, void* workspace, size_t workspace_bytes, void* stream);

/* Byte offsets of the regions inside the workspace (host only).  eps_q, q_out and o_out have size
 * zero unless outlier filtering is on; attn_split (httm_attention_scratch_bytes(H) bytes) is the
 * scratch region of stage 3. */
typedef struct httm_workspace_layout {
  int64_t q_m, k_m, v_m, o_m, assign_q, assign_k, eps_q, q_out, o_out, attn_split, total;
} httm_workspace_layout_t;
HTTM_API int httm_workspace_layout(const httm_geom_t* g, httm_workspace_layout_t* out);

/* ---- adaptive outlier filtering of the merged queries (Sec. 3.4; Alg. 2
 *      "BlockAggregateQuantile"; Alg. 1, the second attention for the outlier queries) ------------
 * Only for plans with outlier_frac > 0 (else HTTM_E_INVALID_ARG).  The three calls replace stage 2,
 * add one attention pass and replace stage 4; httm_layer_forward runs them by itself.
 *
 * Sec. 3.4 step 2: the deviation of a query token is its L2 distance to its merged token (the
 * fp32 mean, before it is rounded to bf16), zero for a token that was not merged with another.
 * Step 3: with budget = outlier_cap, tau is the largest of the H*N deviations that is not among
 * the budget largest; a token whose deviation lies strictly above tau is an outlier (values that
 * tie with tau stay merged, so there can be fewer than budget).  Step 4: a merged query that loses
 * constituents is recomputed from those that remain (a zero row if none remains); an outlier
 * attends by itself with its original query row.
 *
 * The plan holds the threshold, the per-head counts and the row offsets on the device, so calls
 * that use one plan must not overlap in time. */

/* Stage 2 with the filter.  q, k, v, q_m, k_m, v_m, assign_k as for httm_reorder_match_merge.
 * assign_q : [H, N] int32 out; slot in 0..M_q-1, or -1 - r for an outlier whose query sits in row r
 *            of q_out.
 * eps_q    : [H, N] float out, the deviations.
 * q_out    : [outlier_cap, d_head] bf16 out; the outlier queries, grouped by head and, inside a
 *            head, in ascending reordered position. */
HTTM_API int httm_reorder_match_merge_filtered(const httm_plan_t* plan, const void* q, const void* k,
                                               const void* v, void* q_m, void* k_m, void* v_m,
                                               int32_t* assign_q, int32_t* assign_k, float* eps_q,
                                               void* q_out, void* stream);

/* o_out[r] = softmax(q_out[r] k_m[h]^T / 8) v_m[h] for every outlier row r, h the head it belongs to
 * (k_m as stage 2 of this plan wrote it: scaled keys with HTTM_FLAG_LOG2_KEYS).
 * k_m, v_m: [H, M_k, d_head] bf16; o_out: [outlier_cap, d_head] bf16 out. */
HTTM_API int httm_attention_outliers(const httm_plan_t* plan, const void* q_out, const void* k_m,
                                     const void* v_m, void* o_out, void* stream);

/* Stage 4 (inverse reorder fused) with assign_q as written by the filtered stage 2:
 * out[pi[j]][h*d_head ..] = assign_q[h][j] >= 0 ? o_m[h][assign_q[h][j]] : o_out[-1 - assign_q[h][j]]. */
HTTM_API int httm_unmerge_filtered(const httm_plan_t* plan, const void* o_m, const void* o_out,
                                   const int32_t* assign_q, void* out, void* stream);

/* Reads back what the last filtered stage 2 on this plan decided: *tau and counts[H] (outliers per
 * head).  Waits for the stream; for tests and diagnostics. */
HTTM_API int httm_outlier_stats(const httm_plan_t* plan, float* tau, int32_t* counts, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HTTM_H */
