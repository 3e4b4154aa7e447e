// Host-callable launchers of the gfx950 kernels.  Every launcher validates nothing: the C-ABI
// layer has checked shapes and pointers before it gets here.  All return hipError_t.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

#include "geometry.hpp"

namespace httm {

// ---- stage 1 -------------------------------------------------------------------------------
// direction 0: dst[h][j] = src[h][pi[j]];  direction 1: dst[h][pi[j]] = src[h][j].
hipError_t launch_reorder(const void* src, void* dst, const int32_t* pi_dev, int H, int64_t N,
                          int direction, hipStream_t stream);

// ---- stage 2 -------------------------------------------------------------------------------
struct MatchMergeStream {
  const void* x;        // [H, N, 64] bf16: the tensor that is matched (Q or K)
  const void* v;        // [H, N, 64] bf16 merged with x's matches, or nullptr
  void* xm;             // [H, M, 64] bf16 out
  void* vm;             // [H, M, 64] bf16 out (when v != nullptr)
  int32_t* assign;      // [H, N] out
  float* score;         // [H, N] out or nullptr
  const WorkItem* items;  // device
  int32_t n_items;
  int64_t M;
  const int32_t* preset;  // [N] cluster slot per reordered token shared by all heads, or nullptr
  const float* preset_score;  // [N] or nullptr
  float* eps;           // [H, N] out or nullptr: L2 distance of every token to its merged token
  float xm_scale;       // factor on the fp32 means of x before they are rounded to bf16 (1 = plain)
};
struct MatchMergeArgs {
  MatchMergeStream s[2];
  int32_t n_streams;
  const int32_t* pi;    // device; nullptr when x / v are already in reordered order
  int32_t tpf;          // with pi: tokens per frame and slots per row of the patch grid, the strides of
  int32_t row_len;      // the closed form of the reorder inside a work item (WorkItem.src0 / dims)
  int64_t N;
  int32_t H;
  int32_t max_block;
  int32_t max_k;        // most clusters any work item of any stream keeps
  int32_t top_r;        // some work item merges only its top-r src tokens (WorkItem.kd < k)
  WorkItem single;      // used instead of s[].items when those are nullptr (one work item, n_items = 1)
  int32_t chunks;       // big_match_kernel: chunks of 256 tokens per work item, and the item count the
  int32_t n_items_max;  // grid is laid out for (set by its launchers)
};
hipError_t launch_match_merge(const MatchMergeArgs& a, hipStream_t stream);
// The same for blocks of more than kSmallBlockMax tokens (two kernels; no preset mode).
constexpr int kSmallBlockMax = 512;
hipError_t launch_match_merge_big(const MatchMergeArgs& a, hipStream_t stream);
// General rule of Sec. 3.2 (a fixed share of dst tokens, WorkItem.kd < k): after a matching kernel has
// written, for every token, the slot of its most similar dst token (a dst token: its own slot) and
// that similarity, this kernel decides per work item which r = n - k src tokens merge - those with
// the highest similarity, ties by lower position - and gives every other src token a cluster of
// its own behind the dst clusters, in ascending position.  assign is rewritten in place.
struct TopRStream {
  int32_t* assign;        // [heads][head_stride]
  const float* score;     // [heads][head_stride]
  const WorkItem* items;
  int32_t n_items;
  int64_t head_stride;
};
struct TopRArgs {
  TopRStream s[2];
  int32_t n_streams;
};
hipError_t launch_top_r_select(const TopRArgs& a, int heads, hipStream_t stream);
// Un-blocked matching (the cost the merging blocks remove, paper Sec. 3.3): the whole sequence of a
// head is one block of N tokens with kd strided dst tokens.  best[h][j] = index 0..kd-1 of the dst
// most similar to token j (a dst token: its own index), sim[h][j] = that cosine similarity.
hipError_t launch_global_match(const void* x, int64_t N, int H, int32_t kd, int32_t* best, float* sim,
                               hipStream_t stream);

// ---- adaptive outlier filtering of the merged queries (paper Sec. 3.4, Alg. 2) ---------------
// State of the device-side selection of the threshold tau.
struct SelectState {
  uint32_t prefix1;  // the first 11 bits of tau's bit pattern
  uint32_t rank1;    // descending rank of tau among the values that share them
  float tau;         // the threshold: a deviation strictly above it marks an outlier
  uint32_t pad;
  uint32_t prefix2;  // the first 22 bits, and the rank among the values that share those
  uint32_t rank2;
  uint32_t pad2[2];
};
constexpr int kOutlierCountItems = 16;    // work items per workgroup of the kernel that counts the outliers,
constexpr int kOutlierCountItemsMin = 4;  // and when the items are long (blocks of more than 1024 tokens)
struct OutlierBuffers {      // all device memory, owned by the plan
  SelectState* state;
  uint32_t* hist;            // [3][2048] one histogram per pass of the select, zero between calls
  int32_t* counts;           // [H] outliers per head
  int32_t* offsets;          // [H + 1] first outlier row of every head in q_out / o_out
  int32_t* item_cnt;         // [H][n_items] outliers of a work item
  int32_t* wg_cnt;           // [H][n_items / kOutlierCountItemsMin + 1] the same summed per workgroup of the count kernel
  int32_t* item_base;        // [H][n_items] first outlier row of a work item, relative to its head
  int32_t* tiles;            // [1 + 2 * max_tiles]: n, then (head, first row) per attention tile
  int32_t max_tiles;
};
// tau = the largest of the H*N deviations that is not among the `budget` largest; then the
// outlier counts per (work item, head), their prefix offsets and the tile list of the second
// attention (`tile_rows` query rows per tile).
hipError_t launch_outlier_select(const float* eps, int H, int64_t N, int64_t budget,
                                 const WorkItem* items, int n_items, int max_block, const OutlierBuffers& b,
                                 int tile_rows, hipStream_t stream);
// Un-merge the outliers: recompute the merged queries that lose a constituent, give every
// outlier token a row in q_out and rewrite its assign_q entry as -1 - row.
struct RefineArgs {
  const void* x;          // [H, N, 64] bf16 queries (input order with pi, else reordered)
  void* xm;               // [H, M, 64] merged queries, updated in place
  int32_t* assign;        // [H, N], updated in place
  const float* eps;       // [H, N]
  void* q_out;            // [budget, 64] bf16
  const WorkItem* items;
  int32_t n_items;
  int64_t M;
  const int32_t* pi;
  int32_t tpf, row_len;   // as in MatchMergeArgs
  int64_t N;
  int32_t H;
  int32_t max_block;
  int32_t eager;          // request the token rows before testing the item for outliers
  OutlierBuffers b;
};
hipError_t launch_outlier_refine(const RefineArgs& a, hipStream_t stream);
// The same for blocks of more than kSmallBlockMax tokens (max_k: most clusters a work item keeps).
hipError_t launch_outlier_refine_big(const RefineArgs& a, int max_k, hipStream_t stream);

// Head-uniform variant: mean over heads of x[H, N, 64] (bf16) -> xbar[N, 64] (fp32), summed in
// head order; then block-wise matching of the fp32 tokens -> slot[N], score[N].
hipError_t launch_head_mean(const void* x, float* xbar, int H, int64_t N, hipStream_t stream);
hipError_t launch_match_f32(const float* xbar, const int32_t* pi, const WorkItem* items,
                            int32_t n_items, int32_t max_block, int32_t* slot, float* score,
                            hipStream_t stream);

// ---- stage 3 -------------------------------------------------------------------------------
constexpr int kAttnMaxHeads = HTTM_MAX_HEADS;
// log2_keys: the keys carry the factor scale * log2(e) already (stage 2 with
// MatchMergeStream.xm_scale), `scale` is ignored and the fast kernel runs first.
constexpr float kLog2KeyScale = 0.125f * 1.4426950408889634f;   // log2(e) / sqrt(d_head)
// `scratch` (device, 16-byte aligned, or nullptr): room for the fast kernel to run the partial last
// tile of every head in pieces over the keys (attention_scratch_bytes(H) bytes cover any lengths);
// without it, or when the launch is short, the partial tiles run whole.
hipError_t launch_attention(const void* q, const void* k, const void* v, void* o,
                            const int64_t* q_off_host, const int64_t* k_off_host, int H,
                            float scale, bool log2_keys, hipStream_t stream, void* scratch = nullptr,
                            int64_t scratch_bytes = 0);
// Bytes of scratch launch_attention would use for these head lengths if it had them (0: every tile
// runs whole), and the library's own scratch for callers that cannot allocate: a static device
// array of kAttnStaticScratchBytes, whose address on the current device *ptr receives.
constexpr int64_t kAttnStaticScratchBytes = 32ll << 20;
int64_t attention_scratch_need(const int64_t* q_off_host, const int64_t* k_off_host, int H);
hipError_t attention_static_scratch(void** ptr);
// Query rows and tiles are described by device memory (the outlier queries of Sec. 3.4, whose
// number per head is only known on the device): q / o rows of head h are
// [q_off_dev[h], q_off_dev[h+1]); tiles[0] tiles follow in `tiles` as (head, first row) pairs.
constexpr int kAttnDevTileRows = 256;
// Both in one launch: the host-described sequences (q, o) and, appended to the grid, the
// device-described query rows (q2, o2) against the same keys / values.
hipError_t launch_attention_both(const void* q, const void* k, const void* v, void* o,
                                 const int64_t* q_off_host, const int64_t* k_off_host, int H, float scale,
                                 const void* q2, void* o2, const int32_t* q2_off_dev, const int32_t* tiles,
                                 int max_tiles, bool log2_keys, hipStream_t stream, void* scratch = nullptr,
                                 int64_t scratch_bytes = 0);
hipError_t launch_attention_dev_tiles(const void* q, const void* k, const void* v, void* o,
                                      const int32_t* q_off_dev, const int32_t* tiles, int max_tiles,
                                      const int64_t* k_off_host, int H, float scale, bool log2_keys,
                                      hipStream_t stream);

// ---- stage 4 -------------------------------------------------------------------------------
// fused != 0: out[pi[j]][h*64 + c] = o_m[h][assign[h][j]][c]  (out is [N, H*64])
// fused == 0: out[h][j][c]         = o_m[h][assign[h][j]][c]  (out is [H, N, 64])
// A negative assign entry a refers to row -1 - a of `o_out` (an outlier query's own output row).
hipError_t launch_unmerge(const void* o_m, const int32_t* assign, const int32_t* pi_dev, void* out,
                          int H, int64_t N, int64_t M_q, int fused, hipStream_t stream,
                          const void* o_out = nullptr);

}  // namespace httm
