// Stage 1 (temporal reordering, paper Sec. 3.3) and stage 4 (unmerge, Sec. 3.2 Eq. 5-7, with the
// inverse reordering of Sec. 3.3 fused into the store addresses).
//
// Both are pure data movement of 128-byte token rows and are bound by HBM bandwidth.  A row is
// moved by 8 adjacent lanes, 16 bytes each, so every wavefront load/store instruction touches
// whole 128-byte lines; each thread keeps four independent rows in flight.
#include "dev_common.hpp"
#include "kernels.hpp"

namespace httm {

namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerPass = kThreads / kRowChunks;  // 32
constexpr int kUnroll = 4;
constexpr int kRowsPerWg = kRowsPerPass * kUnroll;   // 128

template <int DIR>
__global__ __launch_bounds__(kThreads) void reorder_kernel(const u32x4* __restrict__ src,
                                                           u32x4* __restrict__ dst,
                                                           const int32_t* __restrict__ pi,
                                                           int64_t N) {
  const int c = threadIdx.x & 7;
  const int r = threadIdx.x >> 3;
  const int64_t head_base = (int64_t)blockIdx.y * N * kRowChunks;
  const int64_t j0 = (int64_t)blockIdx.x * kRowsPerWg + r;
  // All loads are unconditional (a slot past the last token reads token N-1 again and stores
  // nothing): a load inside a branch is followed by a wait for everything outstanding, and the
  // kUnroll rows of a thread would arrive one round trip after the other.
  int32_t idx[kUnroll];
  u32x4 val[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int64_t j = j0 + u * kRowsPerPass;
    idx[u] = pi[j < N ? j : N - 1];
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int64_t j = j0 + u * kRowsPerPass;
    const int64_t row = DIR == 0 ? (int64_t)idx[u] : (j < N ? j : N - 1);
    val[u] = __builtin_nontemporal_load(&src[head_base + row * kRowChunks + c]);
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int64_t j = j0 + u * kRowsPerPass;
    if (j < N) {
      const int64_t row = DIR == 0 ? j : (int64_t)idx[u];
      __builtin_nontemporal_store(val[u], &dst[head_base + row * kRowChunks + c]);
    }
  }
}

// out[h][j] = o_m[h][assign[h][j]]  (reordered layout, one head per blockIdx.y).
__global__ __launch_bounds__(kThreads) void unmerge_rows_kernel(const u32x4* __restrict__ o_m,
                                                                const int32_t* __restrict__ assign,
                                                                u32x4* __restrict__ out, int64_t N,
                                                                int64_t M_q,
                                                                const u32x4* __restrict__ o_out) {
  const int c = threadIdx.x & 7;
  const int r = threadIdx.x >> 3;
  const int64_t h = blockIdx.y;
  const int64_t j0 = (int64_t)blockIdx.x * kRowsPerWg + r;
  int32_t idx[kUnroll];
  u32x4 val[kUnroll];
  // (unconditional loads, as in reorder_kernel: one address per row, chosen before the load)
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int64_t j = j0 + u * kRowsPerPass;
    idx[u] = assign[h * N + (j < N ? j : N - 1)];
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const u32x4* p = idx[u] >= 0 ? &o_m[(h * M_q + idx[u]) * kRowChunks + c]
                                 : &o_out[(int64_t)(-1 - idx[u]) * kRowChunks + c];   // an outlier's own row
    val[u] = *p;
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const int64_t j = j0 + u * kRowsPerPass;
    if (j < N) __builtin_nontemporal_store(val[u], &out[(h * N + j) * kRowChunks + c]);
  }
}

// Fused unmerge + inverse reorder + head concatenation.
// A workgroup owns kTok consecutive REORDERED tokens and all heads: the [H][kTok] tile of
// assignments is read with whole-line loads into LDS, then every (token, head) row is copied
// from o_m to out[pi[j]][h*64 ...].  For a fixed token the H rows are adjacent in `out`, so a
// workgroup writes H*128 contiguous bytes per token.
constexpr int kTok = 32;

__global__ __launch_bounds__(kThreads) void unmerge_fused_kernel(const u32x4* __restrict__ o_m,
                                                                 const int32_t* __restrict__ assign,
                                                                 const int32_t* __restrict__ pi,
                                                                 u32x4* __restrict__ out, int H,
                                                                 int64_t N, int64_t M_q,
                                                                 const u32x4* __restrict__ o_out) {
  extern __shared__ int32_t lds[];
  int32_t* s_assign = lds;             // [H][kTok]
  int32_t* s_pi = lds + H * kTok;      // [kTok]
  // Workgroups go round-robin to the 8 XCDs; give every XCD a contiguous range of token tiles so
  // that the tiles of one merging block, which read the same few rows of o_m, share one L2.
  const int per_xcd = gridDim.x >> 3;
  const int64_t tile = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  const int64_t j0 = tile * kTok;
  if (j0 >= N) return;
  for (int e = threadIdx.x; e < H * kTok; e += kThreads) {
    const int h = e / kTok, t = e % kTok;
    const int64_t j = j0 + t;
    s_assign[e] = j < N ? assign[(int64_t)h * N + j] : 0;
  }
  if (threadIdx.x < kTok) {
    const int64_t j = j0 + threadIdx.x;
    s_pi[threadIdx.x] = j < N ? pi[j] : 0;
  }
  __syncthreads();
  const int c = threadIdx.x & 7;
  const int total = kTok * H;  // (token, head) rows of this tile, token-major
  for (int e0 = threadIdx.x >> 3; e0 < total; e0 += kRowsPerPass * kUnroll) {
    u32x4 val[kUnroll];
    // (unconditional loads, as in reorder_kernel; a slot without a row reads row 0 of head 0)
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int e = e0 + u * kRowsPerPass;
      const int t = e / H, h = e % H;
      const bool valid = e < total && j0 + t < N;
      const int32_t sl = valid ? s_assign[h * kTok + t] : 0;   // negative: row -1 - sl of the outlier outputs
      const u32x4* p = sl >= 0 ? &o_m[((int64_t)(valid ? h : 0) * M_q + sl) * kRowChunks + c]
                               : &o_out[(int64_t)(-1 - sl) * kRowChunks + c];
      val[u] = *p;
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int e = e0 + u * kRowsPerPass;
      if (e < total) {
        const int t = e / H, h = e % H;
        if (j0 + t < N)
          __builtin_nontemporal_store(
              val[u], &out[((int64_t)s_pi[t] * H + h) * kRowChunks + c]);
      }
    }
  }
}

}  // namespace

hipError_t launch_reorder(const void* src, void* dst, const int32_t* pi_dev, int H, int64_t N,
                          int direction, hipStream_t stream) {
  if (N == 0 || H == 0) return hipSuccess;
  dim3 grid((unsigned)((N + kRowsPerWg - 1) / kRowsPerWg), (unsigned)H);
  if (direction == 0)
    hipLaunchKernelGGL(reorder_kernel<0>, grid, dim3(kThreads), 0, stream, (const u32x4*)src,
                       (u32x4*)dst, pi_dev, N);
  else
    hipLaunchKernelGGL(reorder_kernel<1>, grid, dim3(kThreads), 0, stream, (const u32x4*)src,
                       (u32x4*)dst, pi_dev, N);
  return hipGetLastError();
}

hipError_t launch_unmerge(const void* o_m, const int32_t* assign, const int32_t* pi_dev, void* out,
                          int H, int64_t N, int64_t M_q, int fused, hipStream_t stream,
                          const void* o_out) {
  if (N == 0 || H == 0) return hipSuccess;
  if (fused) {
    dim3 grid((unsigned)(((N + kTok - 1) / kTok + 7) / 8 * 8));
    const size_t lds = (size_t)(H * kTok + kTok) * sizeof(int32_t);
    hipLaunchKernelGGL(unmerge_fused_kernel, grid, dim3(kThreads), lds, stream, (const u32x4*)o_m,
                       assign, pi_dev, (u32x4*)out, H, N, M_q, (const u32x4*)o_out);
  } else {
    dim3 grid((unsigned)((N + kRowsPerWg - 1) / kRowsPerWg), (unsigned)H);
    hipLaunchKernelGGL(unmerge_rows_kernel, grid, dim3(kThreads), 0, stream, (const u32x4*)o_m,
                       assign, (u32x4*)out, N, M_q, (const u32x4*)o_out);
  }
  return hipGetLastError();
}

}  // namespace httm
