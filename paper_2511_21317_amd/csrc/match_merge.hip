// Stage 2: block-wise bipartite matching (paper Sec. 3.2 Eq. 1 and the best-match rule,
// restricted to merging blocks as in Sec. 3.3 / Alg. 1 "BlockwiseToMe") and aggregation of the
// merged tokens (Sec. 3.2, mean of the constituents; Alg. 1 "BlockAggregate").
//
// One workgroup handles one (work item, head, stream); stream 0 is Q, stream 1 is K with V riding
// on K's matches (Eq. 2 and the sentence after it).  The kernel reads every token row once and
// writes the merged rows and one int32 per token; what bounds it is the issue of vector
// instructions inside a chain of dependent steps (four workgroups per CU), not the memory system.
//
// Inside a workgroup:
//   0. all rows of x are requested at once (straight-line buffer loads, see row_offsets); while
//      they are on their way the table of the dst tokens is built;
//   1. the rows go to LDS (144-byte padded rows), and 1/||x|| in fp32 comes from the registers
//      that staged them (the 8 lanes of a row add their partial sums of squares);
//   2. similarities are raw dot products from v_mfma_f32_32x32x16_bf16 (products of two bf16 are
//      exact in fp32, accumulation is fp32), computed transposed - D * X^T - so that a lane holds
//      one token's scores against 16 of 32 dst tokens; scaling by 1/||d|| and the arg-max run in
//      registers, the two half-waves are combined with one cross-lane exchange.  Lowest cluster
//      id wins exact ties;
//   3. for the K stream the rows of v are requested now (their staging registers were free for the
//      matching) and arrive during 4;
//   4. the tokens are ordered by (cluster, position) with a stable counting sort built from wave
//      ballots (no atomics, so the order is fixed and results are run-to-run identical); one
//      thread per (cluster, 16-byte chunk) then adds the dst and its src tokens in ascending
//      position in fp32, divides by the member count and rounds once to bf16;
//   5. the rows of v replace the rows of x in LDS and the aggregation of 4 runs again with the
//      same clusters.
// Work items with k == n (special-token prefix, or merge ratio 0) skip 1-5 and copy rows.
#include "dev_common.hpp"
#include "kernels.hpp"

namespace httm {

namespace {

// members of a cluster whose rows the aggregation requests together.  Every lane of a wave runs as
// many rounds as the largest cluster among its 8 needs, so a round of 4 wastes more vector issue
// slots than it saves LDS round trips now that a round is one round trip (measured at cfg 5, fused
// launch: 1 -> 0.409, 2 -> 0.391, 3 -> 0.409, 4 -> 0.405, 6 -> 0.47, 8 -> 0.56 ms)
constexpr int kAggBatch = 2;

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel primitives only (no LDS round
// trips): shifts by 1, 2, 4 and 8 inside each row of 16 lanes (a lane without a source adds 0), then
// the last lane of row 0 / 2 is added to row 1 / 3, and the last lane of row 1 to rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 -> rows 1, 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 -> rows 2, 3
  return v;
}

// Selectors (1, 0) and (0, 1) as bf16 pairs, pinned in vector registers: as an instruction
// literal the pair (1, 0) is not taken as two bf16 halves by v_dot2c_f32_bf16 (measured: wrong
// sums), from a register it is.
struct PairSelectors {
  bf16x2 lo, hi;
};
__device__ __forceinline__ PairSelectors make_pair_selectors() {
  uint32_t slo = 0x00003f80u, shi = 0x3f800000u;
  asm volatile("" : "+v"(slo), "+v"(shi));
  return {__builtin_bit_cast(bf16x2, slo), __builtin_bit_cast(bf16x2, shi)};
}

// acc[0..7] += the 8 bf16 channels of one 16-byte row chunk.  One v_dot2 per channel: the pair
// (x_lo, x_hi) against (1, 0) or (0, 1) adds exactly one bf16 value to the fp32 accumulator.
__device__ __forceinline__ void add_row_chunk(float (&acc)[8], const bf16x8 w, const PairSelectors& sel) {
  const bf16x2 sel_lo = sel.lo, sel_hi = sel.hi;
  const bf16x2 pr[4] = {__builtin_shufflevector(w, w, 0, 1), __builtin_shufflevector(w, w, 2, 3),
                        __builtin_shufflevector(w, w, 4, 5), __builtin_shufflevector(w, w, 6, 7)};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    acc[2 * q] = __builtin_amdgcn_fdot2_f32_bf16(pr[q], sel_lo, acc[2 * q], false);
    acc[2 * q + 1] = __builtin_amdgcn_fdot2_f32_bf16(pr[q], sel_hi, acc[2 * q + 1], false);
  }
}

// Sum of x over the aligned group of 8 lanes a lane belongs to, returned in all 8 lanes; data-parallel
// primitives only (no LDS): lane^1 and lane^2 inside a quad, then the mirrored lane of the other quad
// (which by then holds that quad's sum).
__device__ __forceinline__ float sum_over_8_lanes(float x) {
  int v = __builtin_bit_cast(int, x);
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  v = __builtin_bit_cast(int, x);
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  v = __builtin_bit_cast(int, x);
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  return x;
}

// a / b for a small positive integer-valued b, correctly rounded: one Newton step on the product
// with the hardware reciprocal (the residual is exact thanks to the fma).
__device__ __forceinline__ float div_by_count(float a, float b, float rb) {
  const float q = a * rb;
  const float r = fmaf(-q, b, a);
  return fmaf(r, rb, q);
}

// 8 bf16 values times f, rounded to bf16 again.
__device__ __forceinline__ u32x4 scale_chunk(u32x4 w, float f) {
  u32x4 o;
#pragma unroll
  for (int q = 0; q < 4; ++q)
    o[q] = pack_bf16x2(__uint_as_float(w[q] << 16) * f, __uint_as_float(w[q] & 0xFFFF0000u) * f);
  return o;
}

// ---- requests for the token rows of a work item -------------------------------------------------
// One thread stages ITER 16-byte chunks: chunk (tid & 7) of the rows (tid >> 3) + (NT / 8) * i.
// First the byte offsets of all of them inside one head's tensor (when the tokens are still in the
// caller's order: from the closed form of the reorder, or one index load each), then all row loads
// back to back: the counter of outstanding loads is kept in issue order, so a wait for an index
// placed between the row loads would make the rows arrive one round trip after the other.  The rows
// are read with buffer loads - a descriptor of the head's tensor in scalar registers plus a 32-bit
// byte offset per lane (N < 2^25 is checked on the host) - because a slot past the item's last row
// can then be given the offset N * 128, which the descriptor's range check turns into zeros without
// a memory access: the requests are straight-line code.
template <int NT, int ITER>
__device__ __forceinline__ void row_offsets(const int32_t* __restrict__ pi, int tpf, int row_len, const WorkItem& it,
                                            int tid, uint32_t head_bytes, uint32_t (&off)[ITER]) {
  const int n = it.n;
  if (pi && it.dims) {
    // the reorder in closed form: row r of the item is frame r / plane, grid row (r % plane) / nx,
    // column r % nx of the block; the quotients of these small integers are exact in fp32 with the
    // half added (the true quotient of r + 1/2 is at least 1 / (2 * plane) away from every integer)
    const int nx = it.dims & 0xFFFF, plane = it.dims >> 16;
    const float r_plane = 1.0f / (float)plane, r_nx = 1.0f / (float)nx;
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int row = (tid + i * NT) >> 3;
      const int f = (int)(((float)row + 0.5f) * r_plane);
      const int rem = row - f * plane;
      const int y = (int)(((float)rem + 0.5f) * r_nx);
      off[i] = (uint32_t)(it.src0 + f * tpf + y * row_len + (rem - y * nx));
    }
  } else if (pi) {
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int row = (tid + i * NT) >> 3;
      off[i] = row < n ? (uint32_t)pi[it.start + row] : 0u;
    }
  } else {
#pragma unroll
    for (int i = 0; i < ITER; ++i) off[i] = (uint32_t)(it.start + ((tid + i * NT) >> 3));
  }
#pragma unroll
  for (int i = 0; i < ITER; ++i)
    off[i] = ((tid + i * NT) >> 3) < n ? off[i] * kRowBytes + (tid & 7) * 16 : head_bytes;
}

template <int ITER>
__device__ __forceinline__ void request_rows(const void* head_base, uint32_t head_bytes, const uint32_t (&off)[ITER],
                                             u32x4 (&dst)[ITER]) {
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)head_base, 0, (int)head_bytes, kRawBufferWord3);
#pragma unroll
  for (int i = 0; i < ITER; ++i) dst[i] = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off[i], 0, kBufferNonTemporal);
}

// TOPR: work items may have fewer dst tokens (WorkItem.kd) than clusters (k): the general rule of
// Sec. 3.2, where only the n - k src tokens with the highest best-match similarity merge and the
// other src tokens stay clusters of their own (a separate instantiation, so that the usual one
// pays nothing for it).
template <int NW, int MAXN, bool TOPR = false>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(4, 8)))
void match_merge_kernel(const MatchMergeArgs a) {
  constexpr int NT = 64 * NW;
  constexpr int ITER = MAXN * kRowChunks / NT;
  static_assert(MAXN * kRowChunks % NT == 0, "tile must divide among the threads");
  static_assert(NT == MAXN, "one thread per token");

  // (row MAXN stays zero: the aggregation reads it for the slots of a round that have no member)
  __shared__ __align__(16) unsigned char tile[(MAXN + 1) * kLdsRowBytes];
  // phase A (matching): inverse norms of all tokens / of the dst tokens
  // phase B (aggregation): member lists - the same storage, the phases are separated by barriers
  // (TOPR: the selection's 256-bin histogram and a few words, between the two phases)
  constexpr int kUnionA = MAXN * 8, kUnionB = MAXN * 4 + 8 + NW * MAXN, kUnionT = TOPR ? 1024 + 8 + 4 * NW : 0;
  constexpr int kUnionAB = kUnionA > kUnionB ? kUnionA : kUnionB;
  __shared__ __align__(16) unsigned char s_union[kUnionAB > kUnionT ? kUnionAB : kUnionT];
  __shared__ uint16_t s_dpos[MAXN];
  __shared__ int16_t s_cl[MAXN];
  float* s_invn = (float*)s_union;                    // [MAXN]
  float* s_dinv = s_invn + MAXN;                      // [MAXN]
  uint16_t* s_list = (uint16_t*)s_union;              // [MAXN]    tokens ordered by (cluster, position)
  uint16_t* s_off = s_list + MAXN;                    // [MAXN+1]  first list entry of every cluster
  uint8_t* s_wcnt = (uint8_t*)(s_off + MAXN + 4);     // [NW][MAXN] members of cluster m inside wave w (<= 64)

  // (the last stream first: it is the one with v, whose workgroups live longest - the launch should
  // not end on them)
  const MatchMergeStream& s = a.s[a.n_streams - 1 - blockIdx.z];
  if ((int)blockIdx.x >= s.n_items) return;
  const WorkItem it = s.items[blockIdx.x];
  const int64_t h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = it.n, k = it.k;
  const int64_t N = a.N, M = s.M;
  // wave-uniform bases; the per-lane byte offsets below fit 32 bits (N < 2^25 is checked on the host)
  const char* __restrict__ x = (const char*)s.x + h * N * kRowBytes;
  const char* __restrict__ v = s.v ? (const char*)s.v + h * N * kRowBytes : nullptr;
  u32x4* __restrict__ xm = (u32x4*)s.xm + (h * M + it.moff) * kRowChunks;
  u32x4* __restrict__ vm = s.v ? (u32x4*)s.vm + (h * M + it.moff) * kRowChunks : nullptr;
  int32_t* __restrict__ assign = s.assign + h * N + it.start;
  float* __restrict__ score = s.score ? s.score + h * N + it.start : nullptr;

  // ---- the rows of x, all requested up front ---------------------------------------------------
  // The rows of v are requested after the matching (their registers are free until then) and
  // arrive while the clusters are sorted and x is aggregated.
  const uint32_t head_bytes = (uint32_t)N * (uint32_t)kRowBytes;
  uint32_t off[ITER];
  row_offsets<NT, ITER>(a.pi, a.tpf, a.row_len, it, tid, head_bytes, off);
  u32x4 xr[ITER], vr[ITER];
  request_rows<ITER>(x, head_bytes, off, xr);
  auto request_v_rows = [&]() { request_rows<ITER>(v, head_bytes, off, vr); };

  // ---- nothing to merge: copy ----------------------------------------------------------------
  if (k == n && (!TOPR || it.kd == n)) {
    if (v) request_v_rows();
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int e = tid + i * NT;
      if ((e >> 3) < n) {
        xm[e] = s.xm_scale == 1.0f ? xr[i] : scale_chunk(xr[i], s.xm_scale);
        if (v) vm[e] = vr[i];
      }
    }
    if (tid < n) {
      assign[tid] = it.moff + tid;
      if (score) score[tid] = 1.0f;
      if (s.eps) s.eps[h * N + it.start + tid] = 0.f;
    }
    return;
  }

  // ---- 1. the table of the dst tokens, while the rows are on their way ------------------------------
  const int kd = TOPR ? it.kd : k;   // dst tokens = clusters 0 .. kd-1
  s_cl[tid] = -1;
  if (tid < kLdsRowBytes / 16) *(u32x4*)(tile + MAXN * kLdsRowBytes + tid * 16) = u32x4{0, 0, 0, 0};
  __syncthreads();
  for (int m = tid; m < kd; m += NT) {
    const int p = dst_position(m, n, kd, it.n0);
    s_dpos[m] = (uint16_t)p;
    s_cl[p] = (int16_t)m;
  }
  // pad the last 32-wide dst tile with NaN: a NaN score never compares greater, so the arg-max
  // below needs no bounds test
  if (!s.preset)
    for (int m = kd + tid; m < ((kd + 31) & ~31); m += NT) s_dinv[m] = __builtin_nanf("");
  __syncthreads();

  // ---- 2. rows to LDS, and their inverse norms ---------------------------------------------------
  // (slots past the item's last row hold zeros and are written as well: the tile has MAXN rows)
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int e = tid + i * NT;
    *(u32x4*)(tile + (e >> 3) * kLdsRowBytes + (e & 7) * 16) = xr[i];
  }
  if (!s.preset) {
    // inverse norms, from the registers: the 8 lanes that hold the chunks of a row add their sums
    // of squares; of the ITER rows a group of 8 lanes holds, lane c finishes the c-th (one square
    // root and one division per thread) and, if the row is a dst token, files it under its cluster
    static_assert(ITER == kRowChunks, "one row per lane of a group");
    float mine = 0.f;
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const bf16x8 w = __builtin_bit_cast(bf16x8, xr[i]);
      const bf16x2 pr[4] = {__builtin_shufflevector(w, w, 0, 1), __builtin_shufflevector(w, w, 2, 3),
                            __builtin_shufflevector(w, w, 4, 5), __builtin_shufflevector(w, w, 6, 7)};
      float ss = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) ss = __builtin_amdgcn_fdot2_f32_bf16(pr[q], pr[q], ss, false);
      ss = sum_over_8_lanes(ss);
      if ((tid & 7) == i) mine = ss;
    }
    const int row = (tid >> 3) + (NT >> 3) * (tid & 7);
    if (row < n) {
      const float invn = 1.0f / fmaxf(sqrtf(mine), 1e-12f);
      s_invn[row] = invn;
      const int c = s_cl[row];
      if (c >= 0) s_dinv[c] = invn;
    }
  }
  __syncthreads();

  const int l32 = lane & 31, half = lane >> 5;
  int my_cl = -1;  // cluster of token `tid`

  if (s.preset) {
    // Head-uniform variant: the clusters were computed once on the head-averaged tokens.
    if (tid < n) {
      const int32_t slot = s.preset[it.start + tid];
      my_cl = slot - it.moff;
      assign[tid] = slot;
      if (score) score[tid] = s.preset_score ? s.preset_score[it.start + tid] : 1.0f;
      // (general rule: a src token that did not merge is the only member of a cluster behind the dst ones)
      if (TOPR && my_cl >= kd) s_dpos[my_cl] = (uint16_t)tid;
    }
    if (TOPR) __syncthreads();
  } else {
    // ---- 3. similarities and arg-max -----------------------------------------------------------
    // Wave w owns the tokens 64w .. 64w+63, i.e. the two 32-token tiles 2w and 2w+1.
    // The two tiles go through the dst tiles side by side: they share the dst operand and the dst
    // norms, and their dependent chains of LDS reads overlap.
    const int ndt = (kd + 31) >> 5;
    float my_sc = 1.0f;                // similarity of token `tid` to the dst it would join
    if (wave * 64 < n) {
      int tok[2];
      const unsigned char* xrow[2];
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        tok[sub] = (wave * 2 + sub) * 32 + l32;
        xrow[sub] = tile + (tok[sub] < n ? tok[sub] : n - 1) * kLdsRowBytes + half * 16;
      }
      float best[2] = {-INFINITY, -INFINITY};
      int bm[2] = {0, 0};
      for (int dt = 0; dt < ndt; ++dt) {
        asm volatile("" ::: "memory");   // keeps the reads of the token operands inside the loop: registers
        const int m = dt * 32 + l32;
        const int drow = s_dpos[m < kd ? m : kd - 1];
        f32x16 acc[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][r] = acc[1][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8 ad = *(const bf16x8*)(tile + drow * kLdsRowBytes + ks * 32 + half * 16);
#pragma unroll
          for (int sub = 0; sub < 2; ++sub)
            acc[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad, *(const bf16x8*)(xrow[sub] + ks * 32), acc[sub], 0, 0, 0);
        }
        // acc[sub][r] = <dst row, token>, dst row = dt*32 + 8*(r/4) + 4*half + r%4, token = l32 of the tile.
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int mb = dt * 32 + 8 * g + 4 * half;
          const f32x4 dv = *(const f32x4*)(s_dinv + mb);   // mb is a multiple of 4: aligned
#pragma unroll
          for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
              const float sc = acc[sub][4 * g + q] * dv[q];
              if (sc > best[sub]) {
                best[sub] = sc;
                bm[sub] = mb + q;
              }
            }
          }
        }
      }
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const float ob = __shfl_xor(best[sub], 32);
        const int om = __shfl_xor(bm[sub], 32);
        if (ob > best[sub] || (ob == best[sub] && om < bm[sub])) {
          best[sub] = ob;
          bm[sub] = om;
        }
      }
      // lanes 0..31 publish tile 0 and lanes 32..63 tile 1, so that afterwards thread `tid` holds
      // the result of token `tid`
      const int t = half ? tok[1] : tok[0];
      if (t < n) {
        int c = s_cl[t];
        float sc = 1.0f;
        if (c < 0) {
          c = half ? bm[1] : bm[0];
          sc = (half ? best[1] : best[0]) * s_invn[t];
        }
        my_cl = c;
        my_sc = sc;
        if (!TOPR) {
          assign[t] = it.moff + c;
          if (score) score[t] = sc;
        }
      }
    }
    __syncthreads();   // everybody is done with s_invn / s_dinv

    if (TOPR) {
      // ---- 3b. top-r selection (Sec. 3.2): of the n - kd src tokens only the r = n - k with the
      // highest similarity merge (ties: lower position first).  The r-th largest key is found by a
      // radix select over the block (4 passes of 8 bits, LDS histogram); keys that tie with it are
      // taken in ascending position; every other src token becomes a cluster of its own.
      uint32_t* hist = (uint32_t*)s_union;   // [256]; s_invn / s_dinv are dead now
      uint32_t* sel = hist + 256;            // [0] prefix found so far, [1] rank inside it
      int* s_wsum = (int*)(sel + 2);         // [NW] per-wave counts
      const int r = n - k, n_src = n - kd;
      const bool is_src = tid < n && s_cl[tid] < 0;
      uint32_t key = 0;                      // order-preserving image of the similarity
      if (is_src) {
        const uint32_t u = __float_as_uint(my_sc);
        key = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      }
      bool merged = is_src && r > 0;
      if (r > 0 && r < n_src) {
        uint32_t prefix = 0, rank = (uint32_t)(r - 1);   // descending rank of the last key taken
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
          const int shift = 24 - 8 * pass;
          for (int b = tid; b < 256; b += NT) hist[b] = 0;
          __syncthreads();
          if (is_src && (pass == 0 || (key >> (shift + 8)) == prefix)) atomicAdd(&hist[(key >> shift) & 255u], 1u);
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
        }
        // `prefix` is the key of the last src taken; rank + 1 of the keys equal to it are taken
        const bool eq = is_src && key == prefix;
        const unsigned long long eb = __ballot(eq);
        if (lane == 0) s_wsum[wave] = __popcll(eb);
        __syncthreads();
        int er = __builtin_amdgcn_mbcnt_hi((uint32_t)(eb >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)eb, 0u));
        for (int w = 0; w < wave; ++w) er += s_wsum[w];
        merged = is_src && (key > prefix || (eq && er <= (int)rank));
        __syncthreads();   // s_wsum is reused below
      }
      const bool stay = is_src && !merged;
      const unsigned long long sb = __ballot(stay);
      if (lane == 0) s_wsum[wave] = __popcll(sb);
      __syncthreads();
      if (stay) {
        int idx = __builtin_amdgcn_mbcnt_hi((uint32_t)(sb >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)sb, 0u));
        for (int w = 0; w < wave; ++w) idx += s_wsum[w];
        my_cl = kd + idx;
        // (its similarity to the dst it did not join stays the reported score)
        s_dpos[my_cl] = (uint16_t)tid;
      }
      if (tid < n) {
        assign[tid] = it.moff + my_cl;
        if (score) score[tid] = my_sc;
      }
      __syncthreads();   // s_dpos of the new clusters is visible; the union is free for phase 4
    }
  }

  if (v) request_v_rows();

  // ---- 4. stable counting sort of the tokens by cluster -----------------------------------------
  // Rank of a token among the tokens of its cluster inside its wave, and per-wave cluster sizes.
  // The set of lanes that hold the same cluster id is built bit by bit from wave ballots
  // (log2(k) rounds instead of one round per cluster).
  int my_rank = 0;
  for (int m = lane; m < k; m += 64) s_wcnt[wave * MAXN + m] = 0;   // each wave clears its own row
  {
    unsigned long long same = __ballot(my_cl >= 0);
    for (int bit = 0; (1 << bit) < k; ++bit) {
      const bool set = (my_cl >> bit) & 1;
      const unsigned long long b = __ballot(set);
      same &= set ? b : ~b;
    }
    if (my_cl >= 0) {
      my_rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // same wave wrote the zeros above
    if (my_cl >= 0 && my_rank == 0) s_wcnt[wave * MAXN + my_cl] = (uint8_t)__popcll(same);
  }
  __syncthreads();
  {
    // First list entry of every cluster.  Every wave computes all of them and writes them (the same
    // values from every wave): a wave reads back only what it wrote itself, so no barrier is needed
    // before the lists are filled, and nobody waits for one wave's scan.
    int carry = 0;
    for (int m0 = 0; m0 < k; m0 += 64) {
      const int m = m0 + lane;
      int tot = 0;
      if (m < k) {
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += s_wcnt[w * MAXN + m];
      }
      const int incl = wave_inclusive_scan(tot);
      if (m < k) s_off[m] = (uint16_t)(carry + incl - tot);
      carry += __builtin_amdgcn_readlane(incl, 63);
    }
    if (lane == 0) s_off[k] = (uint16_t)carry;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  }
  if (my_cl >= 0) {
    // position among the members of the cluster in ascending token order ...
    int rank = my_rank;
    for (int w = 0; w < wave; ++w) rank += s_wcnt[w * MAXN + my_cl];
    // ... re-ordered so that the dst token comes first and the src tokens keep their order
    const int dp = s_dpos[my_cl];
    const int pos = tid == dp ? 0 : rank + (dp < tid ? 0 : 1);
    s_list[s_off[my_cl] + pos] = (uint16_t)tid;
  }
  __syncthreads();

  // ---- 5. aggregation: thread (cluster m, 16-byte chunk c) -----------------------------------------
  const PairSelectors sel = make_pair_selectors();
  // chunk c of the merged row of cluster m, mc = 8 * m + c, from the rows the tile holds (x: first)
  auto merged_row = [&](const int mc, const bool first) -> u32x4 {
    const int m = mc >> 3, c = mc & 7;
    const int beg = s_off[m], end = s_off[m + 1];
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    // members in list order: the dst token, then its src tokens in ascending position
    const unsigned char* col = tile + c * 16;
    // kAggBatch members per round: their rows are requested together, and with them the list
    // entries of the next round, so that a round costs one LDS round trip.  A slot past the end of
    // the cluster reads the tile's zero row - one select on the row number instead of four on the
    // row's registers, and the list is read without a clamp (the entries behind a cluster's end are
    // other clusters' members or, behind the last one, the words that follow the list in LDS:
    // read, never used).  The kernel is bound by vector instruction issue; these loops are most of it.
    int jj[kAggBatch];
#pragma unroll
    for (int u = 0; u < kAggBatch; ++u) {
      const int e = s_list[beg + u];
      jj[u] = beg + u < end ? e : MAXN;
    }
    for (int idx = beg; idx < end; idx += kAggBatch) {
      bf16x8 w[kAggBatch];
#pragma unroll
      for (int u = 0; u < kAggBatch; ++u) w[u] = *(const bf16x8*)(col + jj[u] * kLdsRowBytes);
#pragma unroll
      for (int u = 0; u < kAggBatch; ++u) {
        const int e = s_list[idx + kAggBatch + u];
        jj[u] = idx + kAggBatch + u < end ? e : MAXN;
      }
#pragma unroll
      for (int u = 0; u < kAggBatch; ++u) add_row_chunk(acc, w[u], sel);
    }
    const float cnt = (float)(end - beg);
    const float rcnt = 1.0f / cnt;
    float mean[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) mean[q] = div_by_count(acc[q], cnt, rcnt);
    const float f = first ? s.xm_scale : 1.0f;   // 1 unless the keys carry the logit scale
    u32x4 o;
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = pack_bf16x2(mean[2 * q] * f, mean[2 * q + 1] * f);
    if (s.eps && first) {
      // Sec. 3.4 step 2: L2 distance of every constituent to the merged token (the fp32 mean);
      // zero where nothing was merged.  The 8 lanes of a cluster hold 8 channels each.
      float* __restrict__ eps = s.eps + h * N + it.start;
      // (the members again, kAggBatch per round with the next list entries on their way, like the sums)
      const bool merged = end - beg >= 2;
      int ej[kAggBatch];
#pragma unroll
      for (int u = 0; u < kAggBatch; ++u) {
        const int e = s_list[beg + u];
        ej[u] = beg + u < end ? e : MAXN;
      }
      for (int i2 = beg; i2 < end; i2 += kAggBatch) {
        bf16x8 w[kAggBatch];
        int cur[kAggBatch];
#pragma unroll
        for (int u = 0; u < kAggBatch; ++u) {
          cur[u] = ej[u];
          w[u] = *(const bf16x8*)(col + ej[u] * kLdsRowBytes);
        }
#pragma unroll
        for (int u = 0; u < kAggBatch; ++u) {
          const int e = s_list[i2 + kAggBatch + u];
          ej[u] = i2 + kAggBatch + u < end ? e : MAXN;
        }
#pragma unroll
        for (int u = 0; u < kAggBatch; ++u) {
          float d2 = 0.f;
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const float df = (float)w[u][q] - mean[q];
            d2 = fmaf(df, df, d2);
          }
          d2 = sum_over_8_lanes(d2);
          if (c == 0 && cur[u] != MAXN) eps[cur[u]] = merged ? __builtin_amdgcn_sqrtf(d2) : 0.f;
        }
      }
    }
    return o;
  };
  auto v_rows_to_lds = [&]() {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int e = tid + i * NT;
      *(u32x4*)(tile + (e >> 3) * kLdsRowBytes + (e & 7) * 16) = vr[i];
    }
  };
  const int n_out = k * kRowChunks;
  if (v && n_out <= NT) {
    // One merged row chunk per thread (the usual case): it is stored only after the rows of v have
    // gone to LDS - behind a store, the wait for those rows would wait for the store as well.
    u32x4 o = {0, 0, 0, 0};
    if (tid < n_out) o = merged_row(tid, true);
    v_rows_to_lds();
    if (tid < n_out) xm[tid] = o;
    __syncthreads();
  } else {
    for (int mc = tid; mc < n_out; mc += NT) xm[mc] = merged_row(mc, true);
    if (v) {
      v_rows_to_lds();
      __syncthreads();
    }
  }
  if (v) {
    for (int mc = tid; mc < n_out; mc += NT) vm[mc] = merged_row(mc, false);
  }
}

// ---- un-merging the outliers (Sec. 3.4 step 4; Alg. 2, second loop) ---------------------------------
//
// One workgroup per (work item, head), queries only.  Tokens whose deviation lies above tau leave
// their cluster: the merged tokens that lose a constituent are recomputed from the constituents
// that remain (dst first if it remains, then ascending position - the order of the first
// aggregation), a merged token that loses all of them becomes a zero row, and every outlier gets a
// row of its own in q_out; its assign entry becomes -1 - row.  Work items without an outlier
// return before they load a single token row.
template <int NW, int MAXN>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(4, 8)))
void outlier_refine_kernel(const RefineArgs a) {
  constexpr int NT = 64 * NW;
  constexpr int ITER = MAXN * kRowChunks / NT;
  static_assert(NT == MAXN, "one thread per token");
  __shared__ __align__(16) unsigned char tile[MAXN * kLdsRowBytes];
  __shared__ uint16_t s_list[MAXN];
  __shared__ uint16_t s_off[MAXN + 4];
  __shared__ uint8_t s_wcnt[NW * MAXN];
  __shared__ uint16_t s_dpos[MAXN];
  __shared__ uint8_t s_affected[MAXN];   // cluster m lost a constituent
  __shared__ uint8_t s_dst_out[MAXN];    // the dst token of cluster m is an outlier
  __shared__ int s_wout[NW];             // outliers per wave

  if ((int)blockIdx.x >= a.n_items) return;
  const WorkItem it = a.items[blockIdx.x];
  const int n = it.n, k = it.k;
  if (k == n) return;                    // nothing was merged here: no deviation, no outlier
  const int64_t h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t N = a.N, M = a.M;
  int32_t* __restrict__ assign = a.assign + h * N + it.start;
  // The token rows are requested before it is known whether the item has an outlier at all when
  // outliers are dense (`eager`: at least one per largest block on average), so that the row
  // latency does not queue behind the latency of the deviations; otherwise after the test.
  const char* __restrict__ x = (const char*)a.x + h * N * kRowBytes;
  const uint32_t head_bytes = (uint32_t)N * (uint32_t)kRowBytes;
  u32x4 xr[ITER];
  uint32_t off[ITER];
  if (a.eager) {
    row_offsets<NT, ITER>(a.pi, a.tpf, a.row_len, it, tid, head_bytes, off);
    request_rows<ITER>(x, head_bytes, off, xr);
  }
  const float tau = a.b.state->tau;
  int cl = tid < n ? assign[tid] - it.moff : -1;   // cluster before the filter
  if (cl >= k) cl = -1;                            // (an entry that is not a slot of this item is left alone)
  const bool is_out = cl >= 0 && a.eps[h * N + it.start + tid] > tau;
  if (!__syncthreads_or(is_out)) return;
  if (!a.eager) {
    row_offsets<NT, ITER>(a.pi, a.tpf, a.row_len, it, tid, head_bytes, off);
    request_rows<ITER>(x, head_bytes, off, xr);
  }

  // ---- rows to LDS ---------------------------------------------------------------------------------
  for (int m = tid; m < k; m += NT) {
    // (clusters kd .. k-1 are single src tokens that did not merge: they never lose a constituent)
    s_dpos[m] = (uint16_t)(m < it.kd ? dst_position(m, n, it.kd, it.n0) : 0xFFFF);
    s_affected[m] = 0;
    s_dst_out[m] = 0;
  }
  for (int m = lane; m < k; m += 64) s_wcnt[wave * MAXN + m] = 0;
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int e = tid + i * NT;
    const int row = e >> 3, c = e & 7;
    if (row < n) *(u32x4*)(tile + row * kLdsRowBytes + c * 16) = xr[i];
  }
  __syncthreads();

  // ---- outliers: rows in q_out, new assign entries, affected clusters ----------------------------------
  const unsigned long long ob = __ballot(is_out);
  if (lane == 0) s_wout[wave] = __popcll(ob);
  if (is_out) {
    s_affected[cl] = 1;
    if (s_dpos[cl] == tid) s_dst_out[cl] = 1;
  }
  __syncthreads();
  if (is_out) {
    // rows of q_out: the head's range, then this work item's share of it, then ascending position
    int r = __builtin_amdgcn_mbcnt_hi((uint32_t)(ob >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)ob, 0u));
    for (int w = 0; w < wave; ++w) r += s_wout[w];
    const int row = a.b.offsets[h] + a.b.item_base[h * a.n_items + blockIdx.x] + r;
    assign[tid] = -1 - row;
    u32x4* __restrict__ dst = (u32x4*)a.q_out + (int64_t)row * kRowChunks;
#pragma unroll
    for (int c = 0; c < kRowChunks; ++c) dst[c] = *(const u32x4*)(tile + tid * kLdsRowBytes + c * 16);
  }
  const int my_cl = is_out ? -1 : cl;   // members that remain

  // ---- stable counting sort of the remaining members by cluster (as in the first aggregation) ------
  int my_rank = 0;
  {
    unsigned long long same = __ballot(my_cl >= 0);
    for (int bit = 0; (1 << bit) < k; ++bit) {
      const bool set = (my_cl >> bit) & 1;
      const unsigned long long b = __ballot(set);
      same &= set ? b : ~b;
    }
    if (my_cl >= 0) {
      my_rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(same >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)same, 0u));
      if (my_rank == 0) s_wcnt[wave * MAXN + my_cl] = (uint8_t)__popcll(same);
    }
  }
  __syncthreads();
  {
    // First list entry of every cluster.  Every wave computes all of them and writes them (the same
    // values from every wave): a wave reads back only what it wrote itself, so no barrier is needed
    // before the lists are filled, and nobody waits for one wave's scan.
    int carry = 0;
    for (int m0 = 0; m0 < k; m0 += 64) {
      const int m = m0 + lane;
      int tot = 0;
      if (m < k) {
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += s_wcnt[w * MAXN + m];
      }
      const int incl = wave_inclusive_scan(tot);
      if (m < k) s_off[m] = (uint16_t)(carry + incl - tot);
      carry += __builtin_amdgcn_readlane(incl, 63);
    }
    if (lane == 0) s_off[k] = (uint16_t)carry;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  }
  if (my_cl >= 0) {
    int rank = my_rank;
    for (int w = 0; w < wave; ++w) rank += s_wcnt[w * MAXN + my_cl];
    const int dp = s_dpos[my_cl];
    // dst first and the src tokens in ascending position; plain ascending if the dst has left
    const int pos = s_dst_out[my_cl] ? rank : (tid == dp ? 0 : rank + (dp < tid ? 0 : 1));
    s_list[s_off[my_cl] + pos] = (uint16_t)tid;
  }
  __syncthreads();

  // ---- the affected merged tokens again ---------------------------------------------------------------------
  const PairSelectors sel = make_pair_selectors();
  u32x4* __restrict__ xm = (u32x4*)a.xm + (h * M + it.moff) * kRowChunks;
  for (int mc = tid; mc < k * kRowChunks; mc += NT) {
    const int m = mc >> 3, c = mc & 7;
    if (!s_affected[m]) continue;
    const int beg = s_off[m], end = s_off[m + 1];
    float acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] = 0.f;
    const unsigned char* col = tile + c * 16;
    for (int idx = beg; idx < end; ++idx)
      add_row_chunk(acc, *(const bf16x8*)(col + s_list[idx] * kLdsRowBytes), sel);
    u32x4 o = {0, 0, 0, 0};
    if (end > beg) {
      const float cnt = (float)(end - beg);
      const float rcnt = 1.0f / cnt;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        o[q] = pack_bf16x2(div_by_count(acc[2 * q], cnt, rcnt), div_by_count(acc[2 * q + 1], cnt, rcnt));
    }
    xm[mc] = o;
  }
}

// ---- head-uniform comparison variant -------------------------------------------------------------

// xbar[i][c] = (x[0][i][c] + x[1][i][c] + ... ) / H, added in head order, fp32.
__global__ __launch_bounds__(256) void head_mean_kernel(const u32x4* __restrict__ x,
                                                        float* __restrict__ xbar, int H, int64_t N) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (row, chunk)
  if (e >= N * kRowChunks) return;
  float acc[8];
  {
    const u32x4 w = x[e];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc[2 * q] = bf16_lo(w[q]);
      acc[2 * q + 1] = bf16_hi(w[q]);
    }
  }
  for (int h = 1; h < H; ++h) {
    const u32x4 w = x[(int64_t)h * N * kRowChunks + e];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      acc[2 * q] += bf16_lo(w[q]);
      acc[2 * q + 1] += bf16_hi(w[q]);
    }
  }
  const float fh = (float)H;
  f32x4 lo = {acc[0] / fh, acc[1] / fh, acc[2] / fh, acc[3] / fh};
  f32x4 hi = {acc[4] / fh, acc[5] / fh, acc[6] / fh, acc[7] / fh};
  f32x4* o = (f32x4*)(xbar + e * 8);
  o[0] = lo;
  o[1] = hi;
}

constexpr int kF32Stride = 68;  // floats per LDS row (272 B: 16-byte aligned, odd granule count)
constexpr int kF32Tile = 64;    // dst tokens per LDS tile

// Block-wise matching of fp32 tokens (the head-averaged tokens of the head-uniform variant, one
// "head's" worth): one workgroup per (work item, 256 of its tokens), one thread per token with the
// token in registers; the item's dst tokens pass through LDS in tiles of 64 and every thread takes
// its fp32 FMA dot products with them in ascending cluster order (first maximum wins).  Any block
// size; writes the slot of the most similar dst token (a dst token: its own slot) and the similarity.
__global__ __launch_bounds__(256) void match_f32_kernel(const float* __restrict__ xbar,
                                                        const int32_t* __restrict__ pi,
                                                        const WorkItem* __restrict__ items,
                                                        int32_t* __restrict__ slot,
                                                        float* __restrict__ score) {
  __shared__ __align__(16) float s_d[kF32Tile * kF32Stride];
  __shared__ float s_dinv[kF32Tile];
  const WorkItem it = items[blockIdx.x];
  const int n = it.n, kd = it.kd, n0 = it.n0, tid = threadIdx.x;
  if ((int)blockIdx.y * 256 >= n) return;
  const int t = blockIdx.y * 256 + tid;
  if (kd == n) {
    if (t < n) {
      slot[it.start + t] = it.moff + t;
      score[it.start + t] = 1.0f;
    }
    return;
  }
  const int tc = t < n ? t : n - 1;
  const int64_t src = pi ? (int64_t)pi[it.start + tc] : (int64_t)(it.start + tc);
  float xr[kDHead];
#pragma unroll
  for (int c = 0; c < kDHead / 4; ++c) {
    const f32x4 w = *(const f32x4*)(xbar + src * kDHead + c * 4);
#pragma unroll
    for (int q = 0; q < 4; ++q) xr[c * 4 + q] = w[q];
  }
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < kDHead; ++q) ss = fmaf(xr[q], xr[q], ss);
  const float invn = 1.0f / fmaxf(sqrtf(ss), 1e-12f);
  float best = -INFINITY;
  int bm = 0;
  for (int m0 = 0; m0 < kd; m0 += kF32Tile) {
#pragma unroll
    for (int i = 0; i < kF32Tile * 16 / 256; ++i) {
      const int e = tid + i * 256, row = e >> 4, c = e & 15;
      const int m = m0 + row < kd ? m0 + row : kd - 1;
      const int p = dst_position(m, n, kd, n0);
      const int64_t sd = pi ? (int64_t)pi[it.start + p] : (int64_t)(it.start + p);
      *(f32x4*)(s_d + row * kF32Stride + c * 4) = *(const f32x4*)(xbar + sd * kDHead + c * 4);
    }
    __syncthreads();
    if (tid < kF32Tile) {
      float ds = 0.f;
      for (int q = 0; q < kDHead; ++q) ds = fmaf(s_d[tid * kF32Stride + q], s_d[tid * kF32Stride + q], ds);
      s_dinv[tid] = 1.0f / fmaxf(sqrtf(ds), 1e-12f);
    }
    __syncthreads();
    const int lim = kd - m0 < kF32Tile ? kd - m0 : kF32Tile;
    for (int mm = 0; mm < lim; ++mm) {
      float dot = 0.f;
#pragma unroll
      for (int q = 0; q < kDHead; ++q) dot = fmaf(xr[q], s_d[mm * kF32Stride + q], dot);
      const float sim = dot * s_dinv[mm];
      if (sim > best) {
        best = sim;
        bm = m0 + mm;
      }
    }
    __syncthreads();
  }
  if (t < n) {
    int c = cluster_at(t, n, kd, n0);
    float sc = 1.0f;
    if (c < 0) {
      c = bm;
      sc = best * invn;
    }
    slot[it.start + t] = it.moff + c;
    score[it.start + t] = sc;
  }
}

}  // namespace

hipError_t launch_match_merge(const MatchMergeArgs& a, hipStream_t stream) {
  int n_items = 0;
  for (int i = 0; i < a.n_streams; ++i) n_items = a.s[i].n_items > n_items ? a.s[i].n_items : n_items;
  if (n_items == 0 || a.H == 0) return hipSuccess;
  if (a.max_block > kSmallBlockMax) return launch_match_merge_big(a, stream);
  dim3 grid((unsigned)n_items, (unsigned)a.H, (unsigned)a.n_streams);
  if (a.top_r) {
    if (a.max_block <= 64)
      hipLaunchKernelGGL((match_merge_kernel<1, 64, true>), grid, dim3(64), 0, stream, a);
    else if (a.max_block <= 256)
      hipLaunchKernelGGL((match_merge_kernel<4, 256, true>), grid, dim3(256), 0, stream, a);
    else
      hipLaunchKernelGGL((match_merge_kernel<8, 512, true>), grid, dim3(512), 0, stream, a);
    return hipGetLastError();
  }
  if (a.max_block <= 64)
    hipLaunchKernelGGL((match_merge_kernel<1, 64>), grid, dim3(64), 0, stream, a);
  else if (a.max_block <= 256)
    hipLaunchKernelGGL((match_merge_kernel<4, 256>), grid, dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL((match_merge_kernel<8, 512>), grid, dim3(512), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_outlier_refine(const RefineArgs& a, hipStream_t stream) {
  if (a.n_items == 0 || a.H == 0) return hipSuccess;
  dim3 grid((unsigned)a.n_items, (unsigned)a.H);
  if (a.max_block <= 64)
    hipLaunchKernelGGL((outlier_refine_kernel<1, 64>), grid, dim3(64), 0, stream, a);
  else if (a.max_block <= 256)
    hipLaunchKernelGGL((outlier_refine_kernel<4, 256>), grid, dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL((outlier_refine_kernel<8, 512>), grid, dim3(512), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_head_mean(const void* x, float* xbar, int H, int64_t N, hipStream_t stream) {
  if (N == 0) return hipSuccess;
  const int64_t total = N * kRowChunks;
  hipLaunchKernelGGL(head_mean_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                     (const u32x4*)x, xbar, H, N);
  return hipGetLastError();
}

hipError_t launch_match_f32(const float* xbar, const int32_t* pi, const WorkItem* items,
                            int32_t n_items, int32_t max_block, int32_t* slot, float* score,
                            hipStream_t stream) {
  if (n_items == 0) return hipSuccess;
  const int mb = max_block < kPrefixChunk ? kPrefixChunk : max_block;
  hipLaunchKernelGGL(match_f32_kernel, dim3((unsigned)n_items, (unsigned)((mb + 255) / 256)), dim3(256), 0, stream,
                     xbar, pi, items, slot, score);
  return hipGetLastError();
}

}  // namespace httm
