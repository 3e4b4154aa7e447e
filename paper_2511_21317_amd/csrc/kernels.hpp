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
};
struct MatchMergeArgs {
  MatchMergeStream s[2];
  int32_t n_streams;
  const int32_t* pi;    // device; nullptr when x / v are already in reordered order
  int64_t N;
  int32_t H;
  int32_t max_block;
};
hipError_t launch_match_merge(const MatchMergeArgs& a, hipStream_t stream);

// Head-uniform variant: mean over heads of x[H, N, 64] (bf16) -> xbar[N, 64] (fp32), summed in
// head order; then block-wise matching of the fp32 tokens -> slot[N], score[N].
hipError_t launch_head_mean(const void* x, float* xbar, int H, int64_t N, hipStream_t stream);
hipError_t launch_match_f32(const float* xbar, const int32_t* pi, const WorkItem* items,
                            int32_t n_items, int32_t max_block, int32_t* slot, float* score,
                            hipStream_t stream);

// ---- stage 3 -------------------------------------------------------------------------------
constexpr int kAttnMaxHeads = HTTM_MAX_HEADS;
hipError_t launch_attention(const void* q, const void* k, const void* v, void* o,
                            const int64_t* q_off_host, const int64_t* k_off_host, int H,
                            float scale, hipStream_t stream);

// ---- stage 4 -------------------------------------------------------------------------------
// fused != 0: out[pi[j]][h*64 + c] = o_m[h][assign[h][j]][c]  (out is [N, H*64])
// fused == 0: out[h][j][c]         = o_m[h][assign[h][j]][c]  (out is [H, N, 64])
hipError_t launch_unmerge(const void* o_m, const int32_t* assign, const int32_t* pi_dev, void* out,
                          int H, int64_t N, int64_t M_q, int fused, hipStream_t stream);

}  // namespace httm
