// Host-side index tables of an HTTM geometry: the temporal reordering permutation
// (paper Sec. 3.3), the merging-block list and the merged-sequence layout (Sec. 3.2, Alg. 1).
#pragma once
#include <cstdint>
#include <vector>

#include "../../include/httm.h"

namespace httm {

// One unit of matching/aggregation work, identical for every head: a run of `n` consecutive
// reordered tokens that keeps `k` clusters whose merged slots start at `moff`.
// Real merging blocks have k <= n; the special-token prefix is cut into pseudo-blocks with
// k == n (every token its own cluster), which the same kernels handle as plain copies.
// The first `n0` tokens of the run are dst tokens whatever the ratio (first-frame anchoring,
// paper App. C.2); the remaining k - n0 dst tokens are strided over the other n - n0.
struct WorkItem {
  int32_t start;  // first reordered position
  int32_t n;      // tokens
  int32_t k;      // clusters kept
  int32_t moff;   // first merged slot
  int32_t n0;     // leading tokens that are always dst
  int32_t kd;     // clusters 0..kd-1 are the dst tokens; kd == k unless only the top-r src merge
  // Closed form of the reorder inside the item, for kernels that read tokens in the caller's order
  // (paper Sec. 3.3: a block is a run of frames x rows x columns of the patch grid, frame-major):
  // token r of the item is the input token src0 + f * tpf + y * row_len + x with
  // f = r / plane, y = (r % plane) / nx, x = r % nx, nx = dims & 0xFFFF, plane = dims >> 16
  // (tpf = tokens per frame, row_len = slots per row of the patch grid).  dims == 0: no closed form
  // (the special-token prefix), the reorder table pi is read instead.
  int32_t src0;
  int32_t dims;
};

// Scratch of stage 3 that covers any launch (attention_split.hpp: kAttnScratchBytes; a slot of
// 256 rows x 66 fp32 for each of the at most 512 + 255 - 1 segments).
inline int64_t attention_scratch_bytes(int) { return (int64_t)(512 + 255) * 256 * (64 + 2) * 4; }

struct HostTables {
  int64_t N = 0, n_prefix = 0, n_blocks = 0, max_block = 0;
  int64_t M_q = 0, M_k = 0;
  std::vector<int32_t> pi;           // reordered position -> input position
  std::vector<int32_t> block_start;  // per real block
  std::vector<int32_t> block_n;
  std::vector<int32_t> block_kq, block_kk, block_offq, block_offk;
  std::vector<int32_t> block_src0, block_dims;  // WorkItem.src0 / dims of every real block (with pi only)
  std::vector<WorkItem> items_q, items_k;  // prefix pseudo-blocks followed by the real blocks
};

constexpr int kPrefixChunk = 64;  // tokens per pseudo-block of the special prefix

// Validate a geometry (returns an HTTM_E_* code).
int check_geom(const httm_geom_t& g);

// Clusters kept by a block of n tokens at merge ratio rho, at least its n0 anchored tokens; *kd
// (if given) receives how many of them are dst tokens (Sec. 3.2; dst_frac = 0: all of them).
int32_t clusters_kept(int32_t n, double rho, int32_t n0 = 0, double dst_frac = 0.0, int32_t* kd = nullptr);

// Outlier queries there can be at most (0 when the filter is off).
int64_t outlier_budget(const httm_geom_t& g, int64_t N);

// Build every table.  `with_pi` = false skips the O(N) permutation (sizes only).
int build_tables(const httm_geom_t& g, bool with_pi, HostTables* out);

inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

int workspace_layout(const httm_geom_t& g, const HostTables& t, httm_workspace_layout_t* out);

}  // namespace httm
