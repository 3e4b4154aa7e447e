// Stage 2: block-wise bipartite matching (paper Sec. 3.2 Eq. 1 and the best-match rule,
// restricted to merging blocks as in Sec. 3.3 / Alg. 1 "BlockwiseToMe") and aggregation of the
// merged tokens (Sec. 3.2, mean of the constituents; Alg. 1 "BlockAggregate").
//
// One workgroup handles one (work item, head, stream); stream 0 is Q, stream 1 is K with V riding
// on K's matches (Eq. 2 and the sentence after it).  The kernel is bound by HBM bandwidth: it
// reads every token row once and writes the merged rows and one int32 per token.  All global
// loads of the workgroup are issued before anything else happens so that each wave has up to
// 16 independent 16-byte loads per lane in flight.
//
// Inside a workgroup:
//   1. the block's rows go to LDS (144-byte padded rows);
//   2. one thread per token computes 1/||x|| in fp32;
//   3. similarities are raw dot products from v_mfma_f32_32x32x16_bf16 (products of two bf16 are
//      exact in fp32, accumulation is fp32), computed transposed - D * X^T - so that a lane holds
//      one token's scores against 16 of 32 dst tokens; scaling by 1/||d|| and the arg-max run in
//      registers, the two half-waves are combined with one cross-lane exchange.  Lowest cluster
//      id wins exact ties;
//   4. every cluster is summed by one wave, lane = channel, dst first and then its src tokens in
//      ascending position (the member set comes from a wave ballot, so the order is fixed and
//      results are run-to-run identical), divided by the member count and rounded once to bf16;
//   5. for the K stream the V rows, held in registers since the start, replace the K rows in LDS
//      and step 4 runs again with the same clusters.
// Work items with k == n (special-token prefix, or merge ratio 0) skip 1-5 and copy rows.
#include "dev_common.hpp"
#include "kernels.hpp"

namespace httm {

namespace {

template <int NW, int MAXN>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(4, 8))) void match_merge_kernel(const MatchMergeArgs a) {
  constexpr int NT = 64 * NW;
  constexpr int ITER = MAXN * kRowChunks / NT;
  constexpr int NC = MAXN / 64;
  static_assert(MAXN * kRowChunks % NT == 0, "tile must divide among the threads");

  __shared__ __align__(16) unsigned char tile[MAXN * kLdsRowBytes];
  __shared__ float s_invn[MAXN];
  __shared__ float s_dinv[MAXN];
  __shared__ int32_t s_dpos[MAXN];
  __shared__ int32_t s_cl[MAXN];

  const MatchMergeStream& s = a.s[blockIdx.z];
  if ((int)blockIdx.x >= s.n_items) return;
  const WorkItem it = s.items[blockIdx.x];
  const int64_t h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = it.n, k = it.k;
  const int64_t N = a.N, M = s.M;
  const u32x4* __restrict__ x = (const u32x4*)s.x + h * N * kRowChunks;
  const u32x4* __restrict__ v = s.v ? (const u32x4*)s.v + h * N * kRowChunks : nullptr;
  u32x4* __restrict__ xm = (u32x4*)s.xm + (h * M + it.moff) * kRowChunks;
  u32x4* __restrict__ vm = s.v ? (u32x4*)s.vm + (h * M + it.moff) * kRowChunks : nullptr;
  int32_t* __restrict__ assign = s.assign + h * N + it.start;
  float* __restrict__ score = s.score ? s.score + h * N + it.start : nullptr;

  // ---- all global loads up front -----------------------------------------------------------
  u32x4 xr[ITER], vr[ITER];
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int e = tid + i * NT;
    const int row = e >> 3, c = e & 7;
    if (row < n) {
      const int64_t src = a.pi ? (int64_t)a.pi[it.start + row] : (int64_t)(it.start + row);
      xr[i] = __builtin_nontemporal_load(&x[src * kRowChunks + c]);
      if (v) vr[i] = __builtin_nontemporal_load(&v[src * kRowChunks + c]);
    }
  }

  // ---- nothing to merge: copy ----------------------------------------------------------------
  if (k == n) {
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int e = tid + i * NT;
      if ((e >> 3) < n) {
        xm[e] = xr[i];
        if (v) vm[e] = vr[i];
      }
    }
    for (int t = tid; t < n; t += NT) {
      assign[t] = it.moff + t;
      if (score) score[t] = 1.0f;
    }
    return;
  }

  // ---- 1. rows to LDS ------------------------------------------------------------------------
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    const int e = tid + i * NT;
    const int row = e >> 3, c = e & 7;
    if (row < n) *(u32x4*)(tile + row * kLdsRowBytes + c * 16) = xr[i];
  }
  for (int t = tid; t < n; t += NT) s_cl[t] = -1;
  __syncthreads();

  const int l32 = lane & 31, half = lane >> 5;

  if (s.preset) {
    // Head-uniform variant: the clusters were computed once on the head-averaged tokens.
    for (int m = tid; m < k; m += NT) s_dpos[m] = (m * n) / k;
    for (int t = tid; t < n; t += NT) {
      const int32_t slot = s.preset[it.start + t];
      s_cl[t] = slot - it.moff;
      assign[t] = slot;
      if (score) score[t] = s.preset_score ? s.preset_score[it.start + t] : 1.0f;
    }
    __syncthreads();
  } else {
    // ---- 2. inverse norms --------------------------------------------------------------------
    for (int t = tid; t < n; t += NT) {
      float ss = 0.f;
#pragma unroll
      for (int c = 0; c < kRowChunks; ++c) {
        const u32x4 w = *(const u32x4*)(tile + t * kLdsRowBytes + c * 16);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float lo = bf16_lo(w[q]), hi = bf16_hi(w[q]);
          ss = fmaf(lo, lo, ss);
          ss = fmaf(hi, hi, ss);
        }
      }
      s_invn[t] = 1.0f / fmaxf(sqrtf(ss), 1e-12f);
    }
    __syncthreads();
    for (int m = tid; m < k; m += NT) {
      const int p = (m * n) / k;  // dst position of cluster m
      s_dpos[m] = p;
      s_dinv[m] = s_invn[p];
      s_cl[p] = m;
    }
    __syncthreads();

    // ---- 3. similarities and arg-max -----------------------------------------------------------
    const int ntt = (n + 31) >> 5, ndt = (k + 31) >> 5;
    for (int tt = wave; tt < ntt; tt += NW) {
      const int tok = tt * 32 + l32;
      const int tokc = tok < n ? tok : n - 1;
      bf16x8 bx[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        bx[ks] = *(const bf16x8*)(tile + tokc * kLdsRowBytes + ks * 32 + half * 16);
      float best = -INFINITY;
      int bm = 0;
      for (int dt = 0; dt < ndt; ++dt) {
        const int m = dt * 32 + l32;
        const int drow = s_dpos[m < k ? m : k - 1];
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8 ad = *(const bf16x8*)(tile + drow * kLdsRowBytes + ks * 32 + half * 16);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ad, bx[ks], acc, 0, 0, 0);
        }
        // acc[r] = <dst row, token>, dst row = dt*32 + 8*(r/4) + 4*half + r%4, token = l32.
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int mm = dt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
          if (mm < k) {
            const float sc = acc[r] * s_dinv[mm];
            if (sc > best) {
              best = sc;
              bm = mm;
            }
          }
        }
      }
      const float ob = __shfl_xor(best, 32);
      const int om = __shfl_xor(bm, 32);
      if (ob > best || (ob == best && om < bm)) {
        best = ob;
        bm = om;
      }
      if (half == 0 && tok < n) {
        int c = s_cl[tok];
        float sc = 1.0f;
        if (c < 0) {
          c = bm;
          sc = best * s_invn[tok];
          s_cl[tok] = c;
        }
        assign[tok] = it.moff + c;
        if (score) score[tok] = sc;
      }
    }
    __syncthreads();
  }

  // ---- 4./5. aggregation ---------------------------------------------------------------------
  int clr[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int t = lane + 64 * c;
    clr[c] = t < n ? s_cl[t] : -1;
  }
  const int64_t head_rows = (h * M + it.moff) * kDHead;
  for (int pass = 0; pass < 2; ++pass) {
    uint16_t* __restrict__ out = (uint16_t*)(pass == 0 ? s.xm : s.vm) + head_rows;
    for (int m = wave; m < k; m += NW) {
      const int dp = s_dpos[m];
      float acc = bf16_bits_to_f32(*(const uint16_t*)(tile + dp * kLdsRowBytes + lane * 2));
      int cnt = 1;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        if (c * 64 < n) {
          unsigned long long mask = __ballot(clr[c] == m && (lane + 64 * c) != dp);
          while (mask) {
            const int j = __ffsll((long long)mask) - 1 + 64 * c;
            acc += bf16_bits_to_f32(*(const uint16_t*)(tile + j * kLdsRowBytes + lane * 2));
            ++cnt;
            mask &= mask - 1;
          }
        }
      }
      out[m * kDHead + lane] = f32_to_bf16_bits(acc / (float)cnt);
    }
    if (pass == 1 || v == nullptr) break;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
      const int e = tid + i * NT;
      const int row = e >> 3, c = e & 7;
      if (row < n) *(u32x4*)(tile + row * kLdsRowBytes + c * 16) = vr[i];
    }
    __syncthreads();
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

// Block-wise matching of fp32 tokens (one head's worth): one thread per token, fp32 FMA dots.
__global__ __launch_bounds__(256) void match_f32_kernel(const float* __restrict__ xbar,
                                                        const int32_t* __restrict__ pi,
                                                        const WorkItem* __restrict__ items,
                                                        int32_t max_block,
                                                        int32_t* __restrict__ slot,
                                                        float* __restrict__ score) {
  extern __shared__ __align__(16) float lds_f[];
  float* tile = lds_f;                                   // [max_block][kF32Stride]
  float* s_invn = tile + (size_t)max_block * kF32Stride;  // [max_block]
  int32_t* s_dpos = (int32_t*)(s_invn + max_block);      // [max_block]
  int32_t* s_cl = s_dpos + max_block;                    // [max_block]
  const WorkItem it = items[blockIdx.x];
  const int n = it.n, k = it.k, tid = threadIdx.x;
  if (k == n) {
    for (int t = tid; t < n; t += 256) {
      slot[it.start + t] = it.moff + t;
      score[it.start + t] = 1.0f;
    }
    return;
  }
  for (int e = tid; e < n * 16; e += 256) {
    const int row = e >> 4, c = e & 15;
    const int64_t src = pi ? (int64_t)pi[it.start + row] : (int64_t)(it.start + row);
    *(f32x4*)(tile + row * kF32Stride + c * 4) = *(const f32x4*)(xbar + src * kDHead + c * 4);
  }
  for (int t = tid; t < n; t += 256) s_cl[t] = -1;
  __syncthreads();
  for (int t = tid; t < n; t += 256) {
    float ss = 0.f;
    for (int c = 0; c < kDHead; ++c) ss = fmaf(tile[t * kF32Stride + c], tile[t * kF32Stride + c], ss);
    s_invn[t] = 1.0f / fmaxf(sqrtf(ss), 1e-12f);
  }
  __syncthreads();
  for (int m = tid; m < k; m += 256) {
    const int p = (m * n) / k;
    s_dpos[m] = p;
    s_cl[p] = m;
  }
  __syncthreads();
  for (int t = tid; t < n; t += 256) {
    int c = s_cl[t];
    float sc = 1.0f;
    if (c < 0) {
      float xr[kDHead];
#pragma unroll
      for (int q = 0; q < kDHead; ++q) xr[q] = tile[t * kF32Stride + q];
      float best = -INFINITY;
      int bm = 0;
      for (int m = 0; m < k; ++m) {
        const int dp = s_dpos[m];
        float dot = 0.f;
#pragma unroll
        for (int q = 0; q < kDHead; ++q) dot = fmaf(xr[q], tile[dp * kF32Stride + q], dot);
        const float sim = dot * s_invn[dp];
        if (sim > best) {
          best = sim;
          bm = m;
        }
      }
      c = bm;
      sc = best * s_invn[t];
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
  dim3 grid((unsigned)n_items, (unsigned)a.H, (unsigned)a.n_streams);
  if (a.max_block <= 64)
    hipLaunchKernelGGL((match_merge_kernel<1, 64>), grid, dim3(64), 0, stream, a);
  else if (a.max_block <= 256)
    hipLaunchKernelGGL((match_merge_kernel<4, 256>), grid, dim3(256), 0, stream, a);
  else
    hipLaunchKernelGGL((match_merge_kernel<8, 512>), grid, dim3(512), 0, stream, a);
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
  int mb = max_block < kPrefixChunk ? kPrefixChunk : max_block;
  const size_t lds = (size_t)mb * (kF32Stride * 4 + 12);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)match_f32_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(match_f32_kernel, dim3((unsigned)n_items), dim3(256), lds, stream, xbar, pi,
                     items, mb, slot, score);
  return hipGetLastError();
}

}  // namespace httm
