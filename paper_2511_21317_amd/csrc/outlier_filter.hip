// Adaptive outlier filtering of the merged queries, device-wide part (paper Sec. 3.4 step 3;
// Alg. 2 "tau <- Quantile(eps, gamma)" and the marking of the outliers).
//
// The H*N deviations are non-negative floats, so their bit patterns order like the values.  The
// threshold - the largest deviation outside the budget of the `budget` largest ones - is found by
// a three-pass radix select on the bit pattern (11 + 11 + 10 bits): a pass histograms the digit
// of every value that matches the digits fixed so far (LDS atomics, then one global atomic per
// non-empty bin) and a one-workgroup kernel walks the histogram from the top to the wanted
// rank.  Integer counts only, so the result does not depend on the order of the atomics.
// Then one pass counts the values above the threshold per (work item, head), a prefix sum per
// head gives every work item the first outlier row it owns (no atomics: the rows of q_out are
// the same from run to run), and one wave turns the head totals into row offsets and into the
// tile list of the second attention.
#include "dev_common.hpp"
#include "kernels.hpp"

namespace httm {

namespace {

constexpr int kBins = 2048;
constexpr int kSelThreads = 256;

template <int PASS>
__device__ __forceinline__ bool digit_of(uint32_t key, uint32_t prefix, uint32_t* digit) {
  if (PASS == 0) {
    *digit = key >> 21;
    return true;
  }
  if (PASS == 1) {
    *digit = (key >> 10) & 0x7FFu;
    return (key >> 21) == prefix;
  }
  *digit = key & 0x3FFu;
  return (key >> 10) == prefix;
}

template <int PASS>
__global__ __launch_bounds__(kSelThreads) void select_hist_kernel(const uint32_t* __restrict__ keys,
                                                                  int64_t total,
                                                                  const SelectState* __restrict__ st,
                                                                  uint32_t* __restrict__ hist) {
  __shared__ uint32_t s_hist[kBins];
  for (int b = threadIdx.x; b < kBins; b += kSelThreads) s_hist[b] = 0;
  __syncthreads();
  const uint32_t prefix = PASS == 0 ? 0u : st->prefix;
  // 16-byte loads; `keys` is 16-byte aligned and the tail is handled by the last threads
  const int64_t n4 = total >> 2;
  const int64_t stride = (int64_t)gridDim.x * kSelThreads;
  for (int64_t i = (int64_t)blockIdx.x * kSelThreads + threadIdx.x; i < n4; i += stride) {
    const u32x4 w = ((const u32x4*)keys)[i];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint32_t d;
      if (digit_of<PASS>(w[q], prefix, &d)) atomicAdd(&s_hist[d], 1u);
    }
  }
  if (blockIdx.x == 0) {
    for (int64_t i = (n4 << 2) + threadIdx.x; i < total; i += kSelThreads) {
      uint32_t d;
      if (digit_of<PASS>(keys[i], prefix, &d)) atomicAdd(&s_hist[d], 1u);
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < kBins; b += kSelThreads) {
    const uint32_t c = s_hist[b];
    if (c) atomicAdd(&hist[b], c);
  }
}

// One workgroup.  Finds the bin that holds the value of descending rank st->rank (0 = largest),
// extends the prefix by that digit, and leaves the histogram zeroed for the next pass / call.
template <int PASS>
__global__ __launch_bounds__(kSelThreads) void select_pick_kernel(uint32_t* __restrict__ hist,
                                                                  SelectState* __restrict__ st,
                                                                  uint32_t budget) {
  constexpr int PER = kBins / kSelThreads;
  __shared__ uint32_t s_part[kSelThreads];
  const int t = threadIdx.x;
  uint32_t h[PER], mine = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    h[i] = hist[t * PER + i];
    hist[t * PER + i] = 0;
    mine += h[i];
  }
  s_part[t] = mine;
  __syncthreads();
  uint32_t above = 0;   // values in the bins of the threads above this one
  for (int u = t + 1; u < kSelThreads; ++u) above += s_part[u];
  const uint32_t rank = PASS == 0 ? budget : st->rank;
  const uint32_t prefix = PASS == 0 ? 0u : st->prefix;
  __syncthreads();      // everybody has read the old state
#pragma unroll
  for (int i = PER - 1; i >= 0; --i) {
    if (rank >= above && rank < above + h[i]) {
      const uint32_t digit = (uint32_t)(t * PER + i);
      const uint32_t np = PASS == 0 ? digit : (prefix << (PASS == 1 ? 11 : 10)) | digit;
      st->prefix = np;
      st->rank = rank - above;
      if (PASS == 2) st->tau = __uint_as_float(np);
    }
    above += h[i];
  }
}

// item_cnt[h][i] = number of deviations above tau among the tokens of work item i of head h.
// One wave per (item, head).
__global__ __launch_bounds__(256) void outlier_count_kernel(const float* __restrict__ eps, int64_t N,
                                                            const WorkItem* __restrict__ items, int n_items,
                                                            const SelectState* __restrict__ st,
                                                            int32_t* __restrict__ item_cnt) {
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= n_items) return;
  const int lane = threadIdx.x & 63;
  const float tau = st->tau;
  const WorkItem it = items[item];
  const float* e = eps + (int64_t)blockIdx.y * N + it.start;
  int c = 0;
  for (int t = lane; t < it.n; t += 64) c += e[t] > tau ? 1 : 0;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d);
  if (lane == 0) item_cnt[(int64_t)blockIdx.y * n_items + item] = c;
}

// One workgroup per head: exclusive prefix sum of the head's item counts, in place, so that every
// work item knows the first outlier row it owns (relative to its head); counts[h] = the head's total.
__global__ __launch_bounds__(256) void outlier_scan_kernel(int32_t* __restrict__ item_cnt, int n_items,
                                                           int32_t* __restrict__ counts) {
  __shared__ int s_part[256];
  int32_t* c = item_cnt + (int64_t)blockIdx.x * n_items;
  const int t = threadIdx.x;
  const int per = (n_items + 255) / 256;
  const int i0 = t * per, i1 = i0 + per < n_items ? i0 + per : n_items;
  int sum = 0;
  for (int i = i0; i < i1; ++i) sum += c[i];
  s_part[t] = sum;
  __syncthreads();
  int base = 0;
  for (int u = 0; u < t; ++u) base += s_part[u];
  for (int i = i0; i < i1; ++i) {
    const int v = c[i];
    c[i] = base;
    base += v;
  }
  if (t == 255) counts[blockIdx.x] = base;
}

// One wave: first outlier row of every head, and the (head, first row) list of the second
// attention's query tiles.  Lane h looks after head h (H <= 64).
__global__ __launch_bounds__(64) void outlier_offsets_kernel(const int32_t* __restrict__ counts,
                                                             int32_t* __restrict__ offsets,
                                                             int32_t* __restrict__ tiles, int H,
                                                             int tile_rows, int max_tiles) {
  const int h = threadIdx.x;
  int32_t off = 0, first_tile = 0, mine = 0;
  for (int g = 0; g < H; ++g) {
    const int32_t c = counts[g];
    if (g < h) {
      off += c;
      first_tile += (c + tile_rows - 1) / tile_rows;
    }
    if (g == h) mine = c;
  }
  if (h < H) {
    offsets[h] = off;
    int nt = first_tile;
    for (int32_t r = 0; r < mine && nt < max_tiles; r += tile_rows, ++nt) {
      tiles[1 + 2 * nt] = h;
      tiles[2 + 2 * nt] = r;
    }
    if (h == H - 1) {
      offsets[H] = off + mine;
      tiles[0] = nt < max_tiles ? nt : max_tiles;
    }
  }
}

}  // namespace

hipError_t launch_outlier_select(const float* eps, int H, int64_t N, int64_t budget,
                                 const WorkItem* items, int n_items, const OutlierBuffers& b,
                                 int tile_rows, hipStream_t stream) {
  const int64_t total = (int64_t)H * N;
  if (total == 0) return hipSuccess;
  const uint32_t* keys = (const uint32_t*)eps;
  // Few workgroups: each ends with one global atomic per non-empty bin, and the values crowd into
  // a handful of bins in the first pass, so the number of workgroups is what serialises there.
  int64_t want = (total / 4 + kSelThreads - 1) / kSelThreads;
  const unsigned grid = (unsigned)(want < 1 ? 1 : (want > 256 ? 256 : want));
  hipLaunchKernelGGL(select_hist_kernel<0>, dim3(grid), dim3(kSelThreads), 0, stream, keys, total, b.state, b.hist);
  hipLaunchKernelGGL(select_pick_kernel<0>, dim3(1), dim3(kSelThreads), 0, stream, b.hist, b.state, (uint32_t)budget);
  hipLaunchKernelGGL(select_hist_kernel<1>, dim3(grid), dim3(kSelThreads), 0, stream, keys, total, b.state, b.hist);
  hipLaunchKernelGGL(select_pick_kernel<1>, dim3(1), dim3(kSelThreads), 0, stream, b.hist, b.state, (uint32_t)budget);
  hipLaunchKernelGGL(select_hist_kernel<2>, dim3(grid), dim3(kSelThreads), 0, stream, keys, total, b.state, b.hist);
  hipLaunchKernelGGL(select_pick_kernel<2>, dim3(1), dim3(kSelThreads), 0, stream, b.hist, b.state, (uint32_t)budget);
  hipLaunchKernelGGL(outlier_count_kernel, dim3((unsigned)((n_items + 3) / 4), (unsigned)H), dim3(256), 0,
                     stream, eps, N, items, n_items, b.state, b.item_base);
  hipLaunchKernelGGL(outlier_scan_kernel, dim3((unsigned)H), dim3(256), 0, stream, b.item_base, n_items,
                     b.counts);
  hipLaunchKernelGGL(outlier_offsets_kernel, dim3(1), dim3(64), 0, stream, b.counts, b.offsets, b.tiles, H,
                     tile_rows, b.max_tiles);
  return hipGetLastError();
}

}  // namespace httm
