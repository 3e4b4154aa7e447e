// Stage 2 for merging blocks that do not fit one LDS tile (more than 512 tokens; the paper's own
// setting is n_b = n_s * n_t = 128 * 30 = 3840, Sec. 4.1).  Same computation as match_merge.hip
// (Sec. 3.2 Eq. 1 and the best-match rule inside a block, Sec. 3.3; mean of the constituents,
// Alg. 1 "BlockwiseToMe" / "BlockAggregate"), cut in two kernels:
//
//   big_match_kernel      one workgroup per (256 tokens of a work item, head, stream).  The tokens sit
//                         in registers as MFMA B operands; the dst tokens of the item stream through
//                         LDS in tiles of 64 (gathered through pi, double buffered), each tile giving
//                         a [64 dst x 256 tokens] block of raw dot products on the matrix cores, scaled
//                         by 1/||d|| and folded into a running (best score, lowest index) per token.
//                         It is the score half of a flash-attention kernel with an arg-max in place
//                         of the softmax.
//   big_aggregate_kernel  one workgroup of 1024 threads per (work item, head, stream).  Cluster sizes
//                         with integer LDS atomics, a prefix sum, the members of every cluster placed
//                         with a second integer atomic and then put into ascending position by
//                         counting (the lists, and so the sums, are the same from run to run); the
//                         member LISTS fit in LDS even though the rows do not, and one thread per
//                         (cluster, 16-byte chunk) gathers its members' rows from global memory, adds
//                         them in fp32 and rounds once.
#include <type_traits>

#include "dev_common.hpp"
#include "kernels.hpp"

namespace httm {

namespace {

struct PairSel {
  bf16x2 lo, hi;
};
__device__ __forceinline__ PairSel pair_selectors() {
  // (1, 0) and (0, 1) as bf16 pairs, pinned in vector registers (see match_merge.hip)
  uint32_t slo = 0x00003f80u, shi = 0x3f800000u;
  asm volatile("" : "+v"(slo), "+v"(shi));
  return {__builtin_bit_cast(bf16x2, slo), __builtin_bit_cast(bf16x2, shi)};
}

__device__ __forceinline__ float sum8(float x) {
  int v = __builtin_bit_cast(int, x);
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false));
  v = __builtin_bit_cast(int, x);
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false));
  v = __builtin_bit_cast(int, x);
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false));
  return x;
}

__device__ __forceinline__ float chunk_sumsq(const bf16x8 w, float ss) {
  const bf16x2 pr[4] = {__builtin_shufflevector(w, w, 0, 1), __builtin_shufflevector(w, w, 2, 3),
                        __builtin_shufflevector(w, w, 4, 5), __builtin_shufflevector(w, w, 6, 7)};
#pragma unroll
  for (int q = 0; q < 4; ++q) ss = __builtin_amdgcn_fdot2_f32_bf16(pr[q], pr[q], ss, false);
  return ss;
}

constexpr int kBmWaves = 4;
constexpr int kBmThreads = 64 * kBmWaves;
// 32-token tiles per wave.  (Three or four would spread the per-dst-tile work over more scores, but the
// operands they keep in registers cost a resident wave: 1.29 / 1.31 / 1.56 ms for stage 2 at 3840-token
// blocks with 2 / 3 / 4.)
constexpr int kBmQt = 2;
constexpr int kBmTokens = 32 * kBmQt * kBmWaves;   // tokens per workgroup
constexpr int kBmDstTile = 64;

// WIDE: the work item may be a whole sequence (un-blocked matching): positions are computed with
// 64-bit products and integer divisions where they are needed, and a workgroup takes 256 consecutive
// positions, dst tokens included.  Merging blocks (at most HTTM_MAX_BLOCK tokens) are handled with
// less index arithmetic, which would otherwise cost more than the arithmetic on the scores: the
// division-free maps of BlockMap, the source rows of all dst tokens of the block looked up once into
// LDS, and workgroups that take 256 consecutive SRC tokens (a dst token has no match to look for, so
// a block with 30 % dst tokens has 30 % fewer scores).
template <bool WIDE>
__global__ __launch_bounds__(kBmThreads) __attribute__((amdgpu_waves_per_eu(2, 4)))
void big_match_kernel(const MatchMergeArgs a) {
  __shared__ __align__(16) unsigned char s_d[2][kBmDstTile * kLdsRowBytes];
  __shared__ __align__(16) float s_dinv[2][kBmDstTile];
  __shared__ uint32_t s_rows[WIDE ? 1 : HTTM_MAX_BLOCK];   // source row of the dst token of every cluster

  // blockIdx -> (work item, head, stream) group and its chunk of 256 tokens.  All chunks of a group
  // stream the same dst tokens, and workgroups go round-robin to the 8 XCDs (each with its own L2),
  // so the chunks of a group are made consecutive workgroups of ONE XCD: XCD x walks the groups
  // x, x + 8, ... and inside a group its a.chunks chunks.
  const int xcd = blockIdx.x & 7, pos = blockIdx.x >> 3;
  const int group = (pos / a.chunks) * 8 + xcd, chunk = pos % a.chunks;
  const int n_heads = a.H;
  const int item = group % a.n_items_max, hs = group / a.n_items_max;
  if (hs >= n_heads * a.n_streams) return;
  const int sidx = hs / n_heads;
  const int64_t h = hs % n_heads;
  const MatchMergeStream& s = a.s[sidx];
  if (item >= s.n_items) return;
  const WorkItem it = s.items ? s.items[item] : a.single;
  // k: the dst tokens of the item (all its clusters under Alg. 1's rule; with a fixed dst share the
  // clusters behind them are the src tokens that stay unmerged, numbered by the selection kernel)
  const int n = it.n, k = it.kd, n0 = it.n0;
  const int t0 = chunk * kBmTokens;
  if (t0 >= n) return;
  const BlockMap bm(n, k, n0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int64_t N = a.N;
  const char* __restrict__ x = (const char*)s.x + h * N * kRowBytes;
  const int32_t* __restrict__ pi = a.pi;
  int32_t* __restrict__ assign = s.assign + h * N + it.start;
  float* __restrict__ score = s.score ? s.score + h * N + it.start : nullptr;

  if (k == n) {   // nothing to merge: every token is its own cluster
    for (int t = t0 + tid; t < n && t < t0 + kBmTokens; t += kBmThreads) {
      assign[t] = it.moff + t;
      if (score) score[t] = 1.0f;
    }
    return;
  }
  // tokens this workgroup matches: positions [t0, t0 + kBmTokens) (WIDE) or the src tokens of those ranks
  const int n_tok = WIDE ? n : n - k;
  if constexpr (!WIDE) {
    // the entries of the dst tokens themselves: chunk c writes those of the clusters [c, c + 1) * kBmTokens
    for (int m = t0 + tid; m < k && m < t0 + kBmTokens; m += kBmThreads) {
      const int p = bm.dst_position(m);
      assign[p] = it.moff + m;
      if (score) score[p] = 1.0f;
    }
    if (t0 >= n_tok) return;
    for (int m2 = tid; m2 < k; m2 += kBmThreads) {
      const int p = bm.dst_position(m2);
      s_rows[m2] = pi ? (uint32_t)pi[it.start + p] : (uint32_t)(it.start + p);
    }
  }

  // ---- this wave's 64 tokens as B operands: lane -> token column, 8 channels per k-step ---------
  bf16x8 bx[kBmQt][4];
  float invn[kBmQt], bias[kBmQt];
  int tpos[kBmQt];
#pragma unroll
  for (int qt = 0; qt < kBmQt; ++qt) {
    const int tok = t0 + wave * (32 * kBmQt) + qt * 32 + l32;
    const int tokc = tok < n_tok ? tok : n_tok - 1;
    if constexpr (WIDE) tpos[qt] = tokc;
    else tpos[qt] = bm.src_position(tokc);
    const uint32_t src = pi ? (uint32_t)pi[it.start + tpos[qt]] : (uint32_t)(it.start + tpos[qt]);
    float ss = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bx[qt][ks] = *(const bf16x8*)(x + src * kRowBytes + ks * 32 + half * 16);
      ss = chunk_sumsq(bx[qt][ks], ss);
    }
    ss += __shfl_xor(ss, 32);
    const float nrm = sqrtf(ss);
    invn[qt] = 1.0f / fmaxf(nrm, 1e-12f);
    bias[qt] = nrm * 1.001f;   // score + bias >= 0 for every dst: |<x, d>| / ||d|| <= ||x||
  }
  if constexpr (!WIDE) __syncthreads();   // s_rows complete

  // ---- dst tiles: thread (row r0 / r0 + 32, chunk c) moves two 16-byte pieces per tile -----------
  const int r0 = tid >> 3, c16 = (tid & 7) * 16;
  const int n_tiles = (k + kBmDstTile - 1) / kBmDstTile;
  u32x4 dreg[2];
  auto dst_src_row = [&](int m) -> uint32_t {   // source row of the dst token of cluster m (clamped)
    const int mc = m < k ? m : k - 1;
    if constexpr (WIDE) {
      const int p = dst_position_any(mc, n, k, n0);
      return pi ? (uint32_t)pi[it.start + p] : (uint32_t)(it.start + p);
    } else {
      return s_rows[mc];
    }
  };
  uint32_t srow[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) srow[i] = dst_src_row(r0 + 32 * i);
#pragma unroll
  for (int i = 0; i < 2; ++i) dreg[i] = *(const u32x4*)(x + srow[i] * kRowBytes + c16);
  if (n_tiles > 1) {
#pragma unroll
    for (int i = 0; i < 2; ++i) srow[i] = dst_src_row(kBmDstTile + r0 + 32 * i);
  }

  // Running arg-max.  A score s = <x, d> / ||d|| is kept as the key (s + bias) with its four lowest
  // mantissa bits replaced by 15 - r, r the accumulator register it came from: the keys are
  // non-negative floats, so a plain float maximum orders them by score and, among scores that agree
  // to 2^-19, by the lower dst index - two vector instructions per score (fma, and-or) plus the
  // maximum tree, instead of scale, compare and two selects.
  float bestk[kBmQt];
  int bd0[kBmQt];
#pragma unroll
  for (int qt = 0; qt < kBmQt; ++qt) {
    bestk[qt] = -1.0f;
    bd0[qt] = 0;
  }
  for (int j = 0; j < n_tiles; ++j) {
    const int buf = j & 1;
    // rows of tile j: registers -> LDS, and 1/||d|| from the 8 lanes that share a row
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r = r0 + 32 * i;
      *(u32x4*)(&s_d[buf][r * kLdsRowBytes + c16]) = dreg[i];
      const float ss = sum8(chunk_sumsq(__builtin_bit_cast(bf16x8, dreg[i]), 0.f));
      if ((tid & 7) == 0)
        s_dinv[buf][r] = j * kBmDstTile + r < k ? __builtin_amdgcn_rsqf(fmaxf(ss, 1e-24f)) : __builtin_nanf("");
    }
    // tile j+1 on its way while tile j is used; the source rows of tile j+2 behind it
    if (j + 1 < n_tiles) {
#pragma unroll
      for (int i = 0; i < 2; ++i) dreg[i] = *(const u32x4*)(x + srow[i] * kRowBytes + c16);
      if (j + 2 < n_tiles) {
#pragma unroll
        for (int i = 0; i < 2; ++i) srow[i] = dst_src_row((j + 2) * kBmDstTile + r0 + 32 * i);
      }
    }
    __syncthreads();
#pragma unroll
    for (int step = 0; step < 2; ++step) {
      const int d0 = j * kBmDstTile + step * 32;
      if (d0 >= k) break;
      bf16x8 ad[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        ad[ks] = *(const bf16x8*)(&s_d[buf][(step * 32 + l32) * kLdsRowBytes + ks * 32 + half * 16]);
#pragma unroll
      for (int qt = 0; qt < kBmQt; ++qt) {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad[ks], bx[qt][ks], acc, 0, 0, 0);
        // acc[r] = <dst d0 + 8*(r/4) + 4*half + r%4, token l32 of tile qt>; rows past k have a NaN
        // scale, and a maximum never returns the NaN operand
        float stepk = -1.0f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 dv = *(const f32x4*)(&s_dinv[buf][step * 32 + 8 * g + 4 * half]);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const uint32_t u = __float_as_uint(fmaf(acc[4 * g + q], dv[q], bias[qt]));
            stepk = fmaxf(stepk, __uint_as_float((u & ~15u) | (uint32_t)(15 - (4 * g + q))));
          }
        }
        // strict comparison of the scores without the index bits: an earlier step keeps a tie
        if (__uint_as_float(__float_as_uint(stepk) & ~15u) > __uint_as_float(__float_as_uint(bestk[qt]) & ~15u)) {
          bestk[qt] = stepk;
          bd0[qt] = d0;
        }
      }
    }
    // (the next iteration writes the other buffer; the one after it this buffer again, and by then
    // every wave has passed the next barrier)
  }

#pragma unroll
  for (int qt = 0; qt < kBmQt; ++qt) {
    const int r = 15 - (int)(__float_as_uint(bestk[qt]) & 15u);
    int bmq = bd0[qt] + 8 * (r >> 2) + 4 * half + (r & 3);
    float bestq = __uint_as_float(__float_as_uint(bestk[qt]) & ~15u);
    const float ob = __shfl_xor(bestq, 32);
    const int om = __shfl_xor(bmq, 32);
    if (ob > bestq || (ob == bestq && om < bmq)) {
      bestq = ob;
      bmq = om;
    }
    const int tok = t0 + wave * (32 * kBmQt) + qt * 32 + l32;
    if (half == 0 && tok < n_tok) {
      int c = -1;
      if constexpr (WIDE) c = cluster_at(tok, n, k, n0);   // (a src token by construction otherwise)
      float sc = 1.0f;
      if (c < 0) {
        c = bmq;
        sc = (bestq - bias[qt]) * invn[qt];
      }
      assign[tpos[qt]] = it.moff + c;
      if (score) score[tpos[qt]] = sc;
    }
  }
}

// ---- top-r selection -----------------------------------------------------------------------------
// One workgroup of 1024 threads per (work item, head, stream), up to four tokens per thread (token t =
// round * 1024 + thread, so ascending position is (round, wave, lane) order).  The r-th largest
// similarity of the item's src tokens comes from a radix select on an order-preserving image of the
// floats (4 passes of 8 bits, LDS histogram, integer counts only); similarities that tie with it are
// taken in ascending position.
constexpr int kSelThreads = 1024;
constexpr int kSelRounds = HTTM_MAX_BLOCK / kSelThreads;

__global__ __launch_bounds__(kSelThreads) void top_r_select_kernel(const TopRArgs a) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sel[2];
  __shared__ int s_part[kSelThreads / 64];
  const TopRStream& s = a.s[blockIdx.z];
  if ((int)blockIdx.x >= s.n_items) return;
  const WorkItem it = s.items[blockIdx.x];
  const int n = it.n, k = it.k, kd = it.kd, n0 = it.n0;
  if (kd >= k) return;                 // every src token merges: the matching kernel's entries stand
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int32_t* __restrict__ assign = s.assign + (int64_t)blockIdx.y * s.head_stride + it.start;
  const float* __restrict__ score = s.score + (int64_t)blockIdx.y * s.head_stride + it.start;
  const int r = n - k, n_src = n - kd;   // src tokens that merge, src tokens there are (r < n_src here)
  bool is_src[kSelRounds];
  uint32_t key[kSelRounds];
#pragma unroll
  for (int i = 0; i < kSelRounds; ++i) {
    const int t = i * kSelThreads + tid;
    is_src[i] = t < n && cluster_at(t, n, kd, n0) < 0;
    key[i] = 0;
    if (is_src[i]) {
      const uint32_t u = __float_as_uint(score[t]);
      key[i] = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    }
  }
  // ascending-position rank of the flagged tokens: exclusive count over (round, wave, lane)
  auto rank_in_order = [&](const bool (&flag)[kSelRounds], int (&rank)[kSelRounds]) {
    int base = 0;
#pragma unroll
    for (int i = 0; i < kSelRounds; ++i) {
      const unsigned long long b = __ballot(flag[i]);
      if (lane == 0) s_part[wave] = __popcll(b);
      __syncthreads();
      int before = 0, total = 0;
      for (int w = 0; w < kSelThreads / 64; ++w) {
        before += w < wave ? s_part[w] : 0;
        total += s_part[w];
      }
      rank[i] = base + before + __builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, 0u));
      base += total;
      __syncthreads();
    }
  };
  bool merged[kSelRounds];
#pragma unroll
  for (int i = 0; i < kSelRounds; ++i) merged[i] = false;
  if (r > 0) {
    uint32_t prefix = 0, rank = (uint32_t)(r - 1);   // descending rank of the last key taken
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < kSelRounds; ++i)
        if (is_src[i] && (pass == 0 || (key[i] >> (shift + 8)) == prefix)) atomicAdd(&hist[(key[i] >> shift) & 255u], 1u);
      __syncthreads();
      if (wave == 0) {
        uint32_t hb[4], mine = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          hb[i] = hist[lane * 4 + i];
          mine += hb[i];
        }
        uint32_t incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
          const uint32_t up = (uint32_t)__shfl_up((int)incl, d);
          if (lane >= d) incl += up;
        }
        uint32_t above = (uint32_t)__shfl((int)incl, 63) - incl;   // keys in the bins of higher lanes
#pragma unroll
        for (int i = 3; i >= 0; --i) {
          if (rank >= above && rank < above + hb[i]) {
            sel[0] = (prefix << 8) | (uint32_t)(lane * 4 + i);
            sel[1] = rank - above;
          }
          above += hb[i];
        }
      }
      __syncthreads();
      prefix = sel[0];
      rank = sel[1];
      __syncthreads();
    }
    // `prefix` is the key of the last src taken; rank + 1 of the keys equal to it are taken
    bool eq[kSelRounds];
    int er[kSelRounds];
#pragma unroll
    for (int i = 0; i < kSelRounds; ++i) eq[i] = is_src[i] && key[i] == prefix;
    rank_in_order(eq, er);
#pragma unroll
    for (int i = 0; i < kSelRounds; ++i) merged[i] = is_src[i] && (key[i] > prefix || (eq[i] && er[i] <= (int)rank));
  }
  bool stay[kSelRounds];
  int idx[kSelRounds];
#pragma unroll
  for (int i = 0; i < kSelRounds; ++i) stay[i] = is_src[i] && !merged[i];
  rank_in_order(stay, idx);
#pragma unroll
  for (int i = 0; i < kSelRounds; ++i)
    if (stay[i]) assign[i * kSelThreads + tid] = it.moff + kd + idx[i];
  (void)n_src;
}

// ---- aggregation ---------------------------------------------------------------------------------

constexpr int kBaWaves = 16;
constexpr int kBaThreads = 64 * kBaWaves;

// What the REFINE instantiation needs on top of the stream description (Sec. 3.4 step 4).
struct RefineExtra {
  const SelectState* state;   // tau
  const int32_t* offsets;     // [H + 1] first outlier row of a head
  const int32_t* item_base;   // [H][n_items] first outlier row of a work item inside its head
  void* q_out;                // [budget, 64] bf16
};

// Dynamic LDS: s_src[nmax] int32 | s_off[kmax + 1] int32 | s_cur[kmax] int32 | s_any[nmax] u16 |
//              s_cl[nmax] int16 | s_list[nmax] u16 | s_aff[kmax] u8 | s_dout[kmax] u8
//
// REFINE = false: first aggregation of one stream (X and, for the K stream, V); the workgroups of the
//                 last stream, which carries V and takes twice as long, are dispatched first, so the
//                 launch ends on the short ones.
// REFINE = true : the un-merging of the outliers for the query stream a.s[0] (see
//                 outlier_refine_kernel in match_merge.hip for the rules): tokens whose deviation lies
//                 above tau get a row of q_out and a negative assign entry, and only the clusters that
//                 lose a constituent are summed again.
template <bool REFINE>
__global__ __launch_bounds__(kBaThreads) void big_aggregate_kernel(const MatchMergeArgs a, const RefineExtra rx,
                                                                   int nmax, int kmax) {
  extern __shared__ __align__(16) unsigned char lds[];
  int32_t* s_src = (int32_t*)lds;
  int32_t* s_off = s_src + nmax;
  int32_t* s_cur = s_off + kmax + 1;
  uint16_t* s_any = (uint16_t*)(s_cur + kmax);                 // members of every cluster, in any order
  int16_t* s_cl = (int16_t*)(s_any + nmax + (nmax & 1));
  uint16_t* s_list = (uint16_t*)(s_cl + nmax + (nmax & 1));    // the same in the order of the sums
  uint8_t* s_aff = (uint8_t*)(s_list + nmax + (nmax & 1));
  uint8_t* s_dout = s_aff + kmax;
  __shared__ int s_part[kBaWaves];

  const MatchMergeStream& s = a.s[REFINE ? 0 : gridDim.z - 1 - blockIdx.z];
  if ((int)blockIdx.x >= s.n_items) return;
  const WorkItem it = s.items[blockIdx.x];
  const int n = it.n, k = it.k, kd = it.kd;
  if (REFINE && k == n) return;   // nothing was merged here: no deviation, no outlier
  // position of the dst token of cluster m; the clusters kd .. k-1 are single src tokens that did not
  // merge (general rule of Sec. 3.2): they have no dst token, their only member comes first anyway
  const BlockMap bm(n, kd, it.n0);
  auto dst_of = [&](int m) { return m < kd ? bm.dst_position(m) : -1; };
  const int64_t h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t N = a.N, M = s.M;
  const char* __restrict__ x = (const char*)s.x + h * N * kRowBytes;
  const char* __restrict__ v = (!REFINE && s.v) ? (const char*)s.v + h * N * kRowBytes : nullptr;
  u32x4* __restrict__ xm = (u32x4*)s.xm + (h * M + it.moff) * kRowChunks;
  u32x4* __restrict__ vm = v ? (u32x4*)s.vm + (h * M + it.moff) * kRowChunks : nullptr;
  int32_t* __restrict__ assign = s.assign + h * N + it.start;

  // ---- clusters of the tokens; in REFINE mode the outliers leave ---------------------------------------
  if (REFINE) {
    const float tau = rx.state->tau;
    const float* __restrict__ eps = s.eps + h * N + it.start;
    bool any = false;
    for (int t = tid; t < n; t += kBaThreads) {
      int cl = assign[t] - it.moff;
      if (cl < 0 || cl >= k) cl = -1;              // not a slot of this item: left alone
      const bool out = cl >= 0 && eps[t] > tau;
      s_cl[t] = (int16_t)(out ? -2 - cl : cl);     // outliers remember the cluster they leave
      any = any || out;
    }
    if (!__syncthreads_or(any)) return;
  } else if (s.preset) {
    // head-uniform variant: the clusters were computed once on the head-averaged tokens
    float* __restrict__ score = s.score ? s.score + h * N + it.start : nullptr;
    for (int t = tid; t < n; t += kBaThreads) {
      const int32_t slot = s.preset[it.start + t];
      assign[t] = slot;
      if (score) score[t] = s.preset_score ? s.preset_score[it.start + t] : 1.0f;
      s_cl[t] = (int16_t)(slot - it.moff);
    }
  } else {
    for (int t = tid; t < n; t += kBaThreads) s_cl[t] = (int16_t)(assign[t] - it.moff);
  }
  for (int m = tid; m <= k; m += kBaThreads) s_off[m] = 0;
  for (int m = tid; m < k; m += kBaThreads) {
    s_aff[m] = 0;
    s_dout[m] = 0;
  }
  __syncthreads();
  for (int t = tid; t < n; t += kBaThreads) {
    s_src[t] = a.pi ? a.pi[it.start + t] : it.start + t;
    const int cl = s_cl[t];
    if (cl >= 0) atomicAdd(&s_off[cl + 1], 1);    // integer counts: order does not matter
    if (REFINE && cl <= -2) {
      const int left = -2 - cl;
      s_aff[left] = 1;
      if (dst_of(left) == t) s_dout[left] = 1;
    }
  }
  __syncthreads();

  if (REFINE) {
    // rows of q_out in ascending position: the head's range, then this item's share, then the rank
    int base = rx.offsets[h] + rx.item_base[h * s.n_items + blockIdx.x];
    for (int t0 = 0; t0 < n; t0 += kBaThreads) {
      const int t = t0 + tid;
      const bool out = t < n && s_cl[t] <= -2;
      const unsigned long long ob = __ballot(out);
      if (lane == 0) s_part[wave] = __popcll(ob);
      __syncthreads();
      int before = 0, total = 0;
      for (int w = 0; w < kBaWaves; ++w) {
        before += w < wave ? s_part[w] : 0;
        total += s_part[w];
      }
      if (out) {
        const int row = base + before +
                        __builtin_amdgcn_mbcnt_hi((uint32_t)(ob >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ob, 0u));
        assign[t] = -1 - row;
        const u32x4* __restrict__ srcrow = (const u32x4*)(x + (uint32_t)s_src[t] * kRowBytes);
        u32x4* __restrict__ dst = (u32x4*)rx.q_out + (int64_t)row * kRowChunks;
        u32x4 r8[kRowChunks];
#pragma unroll
        for (int c = 0; c < kRowChunks; ++c) r8[c] = srcrow[c];
#pragma unroll
        for (int c = 0; c < kRowChunks; ++c) dst[c] = r8[c];
      }
      base += total;
      __syncthreads();
    }
  }

  // inclusive prefix over s_off[1..k]  ->  s_off[m] = first list entry of cluster m
  {
    const int per = (k + kBaThreads - 1) / kBaThreads;
    const int i0 = 1 + tid * per, i1 = i0 + per <= k + 1 ? i0 + per : k + 1;
    int sum = 0;
    for (int i = i0; i < i1; ++i) sum += s_off[i];
    int incl = sum;   // inclusive scan over the wave, then over the 16 wave totals
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d);
      if (lane >= d) incl += up;
    }
    if (lane == 63) s_part[wave] = incl;
    __syncthreads();
    int base = incl - sum;
    for (int w = 0; w < wave; ++w) base += s_part[w];
    for (int i = i0; i < i1; ++i) {
      base += s_off[i];
      s_off[i] = base;
    }
  }
  __syncthreads();
  for (int m = tid; m < k; m += kBaThreads) s_cur[m] = s_off[m];
  __syncthreads();

  // ---- member lists -------------------------------------------------------------------------------------------
  // Every token takes a slot of its cluster's range with an integer LDS atomic (any order), then finds
  // its place in the order of the sums by counting the members that precede it: ascending position,
  // re-ordered so that the dst token comes first (the order of match_merge.hip); plain ascending if
  // the dst token has left.  The result does not depend on the order of the atomics, so it is the
  // same from run to run; the work per token is the size of its cluster.
  for (int t = tid; t < n; t += kBaThreads) {
    const int cl = s_cl[t];
    if (cl >= 0) s_any[atomicAdd(&s_cur[cl], 1)] = (uint16_t)t;
  }
  __syncthreads();
  for (int t = tid; t < n; t += kBaThreads) {
    const int cl = s_cl[t];
    if (cl < 0) continue;
    const int first = s_off[cl], len = s_off[cl + 1] - first;
    int rank = 0;
    for (int j = 0; j < len; ++j) rank += (int)s_any[first + j] < t;
    const int dp = (REFINE && s_dout[cl]) ? -1 : dst_of(cl);
    const int fin = t == dp ? 0 : (t < dp ? rank + 1 : rank);
    s_list[first + fin] = (uint16_t)t;
  }
  __syncthreads();

  // ---- aggregation: thread (cluster m, 16-byte chunk c) gathers its members' rows ---------------------------
  // Four members at a time, all loads of a batch (X and V) issued before the first add; a batch that
  // runs past the end of the list loads nothing for the missing members and adds zeros.
  const PairSel sel = pair_selectors();
  auto add_chunk = [&](float (&acc)[8], const bf16x8 w) {
    const bf16x2 pr[4] = {__builtin_shufflevector(w, w, 0, 1), __builtin_shufflevector(w, w, 2, 3),
                          __builtin_shufflevector(w, w, 4, 5), __builtin_shufflevector(w, w, 6, 7)};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc[2 * q] = __builtin_amdgcn_fdot2_f32_bf16(pr[q], sel.lo, acc[2 * q], false);
      acc[2 * q + 1] = __builtin_amdgcn_fdot2_f32_bf16(pr[q], sel.hi, acc[2 * q + 1], false);
    }
  };
  auto finish = [&](const float (&acc)[8], float cnt, float (&mean)[8], float f) -> u32x4 {
    const float rcnt = 1.0f / cnt;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      // correctly rounded quotient: one Newton step on the product with the reciprocal
      const float qv = acc[q] * rcnt;
      mean[q] = fmaf(fmaf(-qv, cnt, acc[q]), rcnt, qv);
    }
    u32x4 o;
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = pack_bf16x2(mean[2 * q] * f, mean[2 * q + 1] * f);
    return o;
  };
  // The rows come through buffer loads: the four offsets of a batch first (a missing member gets the
  // offset one past the head's rows, for which the load returns zeros), then the loads in a straight
  // line.  A load inside a branch, or one whose address is computed between the loads, makes the
  // compiler wait for all earlier loads before its first use, which would run the batch one row at
  // a time; so the loop exists twice, with and without V, instead of testing v inside.
  const uint32_t head_bytes = (uint32_t)N * kRowBytes;
  const __amdgpu_buffer_rsrc_t x_rows = __builtin_amdgcn_make_buffer_rsrc((void*)x, 0, (int)head_bytes, kRawBufferWord3);
  const __amdgpu_buffer_rsrc_t v_rows =
      __builtin_amdgcn_make_buffer_rsrc((void*)(v ? v : x), 0, (int)head_bytes, kRawBufferWord3);
  auto sum_members = [&](auto with_v, int beg, int end, int c, float (&acc)[8], float (&accv)[8]) {
    constexpr bool kWithV = decltype(with_v)::value;
    for (int idx = beg; idx < end; idx += 4) {
      uint32_t off[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int token = s_list[idx + u < end ? idx + u : beg];
        const uint32_t o = (uint32_t)s_src[token] * kRowBytes + c * 16;
        off[u] = idx + u < end ? o : head_bytes;
      }
      u32x4 w[4], wv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) w[u] = __builtin_amdgcn_raw_buffer_load_b128(x_rows, (int)off[u], 0, 0);
      if constexpr (kWithV) {
#pragma unroll
        for (int u = 0; u < 4; ++u) wv[u] = __builtin_amdgcn_raw_buffer_load_b128(v_rows, (int)off[u], 0, 0);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) add_chunk(acc, __builtin_bit_cast(bf16x8, w[u]));
      if constexpr (kWithV) {
#pragma unroll
        for (int u = 0; u < 4; ++u) add_chunk(accv, __builtin_bit_cast(bf16x8, wv[u]));
      }
    }
  };
  for (int mc = tid; mc < k * kRowChunks; mc += kBaThreads) {
    const int m = mc >> 3, c = mc & 7;
    if (REFINE && !s_aff[m]) continue;
    const int beg = s_off[m], end = s_off[m + 1];
    float acc[8], accv[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = accv[q] = 0.f;
    if (v)
      sum_members(std::true_type{}, beg, end, c, acc, accv);
    else
      sum_members(std::false_type{}, beg, end, c, acc, accv);
    if (REFINE && end == beg) {   // every constituent has left: a zero row nobody reads
      xm[mc] = u32x4{0, 0, 0, 0};
      continue;
    }
    const float cnt = (float)(end - beg);
    float mean[8], meanv[8];
    xm[mc] = finish(acc, cnt, mean, REFINE ? 1.0f : s.xm_scale);
    if (v) vm[mc] = finish(accv, cnt, meanv, 1.0f);
    if (!REFINE && s.eps) {
      // Sec. 3.4 step 2: L2 distance of every constituent to the fp32 mean; zero if nothing was merged
      float* __restrict__ eps = s.eps + h * N + it.start;
      // (the members' rows again, four at a time like the sums above)
      for (int i2 = beg; i2 < end; i2 += 4) {
        int j[4];
        uint32_t off[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          j[u] = s_list[i2 + u < end ? i2 + u : beg];
          const uint32_t o = (uint32_t)s_src[j[u]] * kRowBytes + c * 16;
          off[u] = i2 + u < end ? o : head_bytes;
        }
        u32x4 w4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w4[u] = __builtin_amdgcn_raw_buffer_load_b128(x_rows, (int)off[u], 0, 0);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bf16x8 w = __builtin_bit_cast(bf16x8, w4[u]);
          float d2 = 0.f;
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const float df = (float)w[q] - mean[q];
            d2 = fmaf(df, df, d2);
          }
          d2 = sum8(d2);
          if (c == 0 && i2 + u < end) eps[j[u]] = end - beg >= 2 ? sqrtf(d2) : 0.f;
        }
      }
    }
  }
}

size_t big_aggregate_lds(int nmax, int kmax) {
  const size_t n2 = (size_t)nmax + (nmax & 1);
  return (size_t)nmax * 4 + ((size_t)kmax + 1) * 4 + (size_t)kmax * 4 + 3 * n2 * 2 + 2 * (size_t)kmax;
}

template <bool REFINE>
hipError_t allow_big_lds() {
  static bool done = false;
  if (done) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute((const void*)big_aggregate_kernel<REFINE>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
  done = e == hipSuccess;
  return e;
}

}  // namespace

hipError_t launch_top_r_select(const TopRArgs& a, int heads, hipStream_t stream) {
  int n_items = 0;
  for (int i = 0; i < a.n_streams; ++i) n_items = a.s[i].n_items > n_items ? a.s[i].n_items : n_items;
  if (n_items == 0 || heads == 0) return hipSuccess;
  hipLaunchKernelGGL(top_r_select_kernel, dim3((unsigned)n_items, (unsigned)heads, (unsigned)a.n_streams),
                     dim3(kSelThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_match_merge_big(const MatchMergeArgs& a, hipStream_t stream) {
  int n_items = 0, preset = 0;
  for (int i = 0; i < a.n_streams; ++i) {
    n_items = a.s[i].n_items > n_items ? a.s[i].n_items : n_items;
    preset |= a.s[i].preset != nullptr;
  }
  if (n_items == 0 || a.H == 0) return hipSuccess;
  const int nmax = a.max_block;
  const int kmax = a.max_k > 0 ? a.max_k : a.max_block;
  hipError_t e;
  if (!preset) {
    MatchMergeArgs m = a;
    m.chunks = (nmax + kBmTokens - 1) / kBmTokens;
    m.n_items_max = n_items;
    const int64_t groups = (int64_t)n_items * a.H * a.n_streams;
    const unsigned mgrid = (unsigned)(8 * ((groups + 7) / 8) * m.chunks);
    hipLaunchKernelGGL(big_match_kernel<false>, dim3(mgrid), dim3(kBmThreads), 0, stream, m);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.top_r) {
      // general rule of Sec. 3.2: which src tokens merge, and the clusters of those that do not
      TopRArgs t = {};
      t.n_streams = a.n_streams;
      for (int i = 0; i < a.n_streams; ++i) {
        if (!a.s[i].score) return hipErrorInvalidValue;     // the selection needs every token's similarity
        t.s[i] = {a.s[i].assign, a.s[i].score, a.s[i].items, a.s[i].n_items, a.N};
      }
      e = launch_top_r_select(t, a.H, stream);
      if (e != hipSuccess) return e;
    }
  }
  e = allow_big_lds<false>();
  if (e != hipSuccess) return e;
  dim3 agrid((unsigned)n_items, (unsigned)a.H, (unsigned)a.n_streams);
  hipLaunchKernelGGL(big_aggregate_kernel<false>, agrid, dim3(kBaThreads), big_aggregate_lds(nmax, kmax), stream,
                     a, RefineExtra{}, nmax, kmax);
  return hipGetLastError();
}

hipError_t launch_global_match(const void* x, int64_t N, int H, int32_t kd, int32_t* best, float* sim,
                               hipStream_t stream) {
  if (N == 0 || H == 0) return hipSuccess;
  MatchMergeArgs a = {};
  a.n_streams = 1;
  a.pi = nullptr;
  a.N = N;
  a.H = H;
  a.max_block = (int32_t)N;
  a.single = {0, (int32_t)N, kd, 0, 0, kd, 0, 0};
  a.s[0].x = x;
  a.s[0].assign = best;
  a.s[0].score = sim;
  a.s[0].items = nullptr;
  a.s[0].n_items = 1;
  a.chunks = (int32_t)((N + kBmTokens - 1) / kBmTokens);
  a.n_items_max = 1;
  // (one group per head: the groups of 8 consecutive heads run side by side on the 8 XCDs)
  const unsigned grid = (unsigned)(8 * ((H + 7) / 8) * a.chunks);
  hipLaunchKernelGGL(big_match_kernel<true>, dim3(grid), dim3(kBmThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_outlier_refine_big(const RefineArgs& r, int max_k, hipStream_t stream) {
  if (r.n_items == 0 || r.H == 0) return hipSuccess;
  MatchMergeArgs a = {};
  a.n_streams = 1;
  a.pi = r.pi;
  a.N = r.N;
  a.H = r.H;
  a.max_block = r.max_block;
  a.max_k = max_k;
  a.s[0].x = r.x;
  a.s[0].xm = r.xm;
  a.s[0].assign = r.assign;
  a.s[0].items = r.items;
  a.s[0].n_items = r.n_items;
  a.s[0].M = r.M;
  a.s[0].eps = const_cast<float*>(r.eps);
  const RefineExtra rx = {r.b.state, r.b.offsets, r.b.item_base, r.q_out};
  const int nmax = r.max_block, kmax = max_k > 0 ? max_k : r.max_block;
  hipError_t e = allow_big_lds<true>();
  if (e != hipSuccess) return e;
  dim3 grid((unsigned)r.n_items, (unsigned)r.H);
  hipLaunchKernelGGL(big_aggregate_kernel<true>, grid, dim3(kBaThreads), big_aggregate_lds(nmax, kmax), stream, a,
                     rx, nmax, kmax);
  return hipGetLastError();
}

}  // namespace httm
