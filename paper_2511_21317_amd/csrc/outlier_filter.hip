// Adaptive outlier filtering of the merged queries, device-wide part (paper Sec. 3.4 step 3;
// Alg. 2 "tau <- Quantile(eps, gamma)" and the marking of the outliers).
//
// The H*N deviations are non-negative floats, so their bit patterns order like the values.  The
// threshold - the largest deviation outside the budget of the `budget` largest ones - is found by
// a three-pass radix select on the bit pattern (11 + 11 + 10 bits): a pass histograms the digit
// of every value that matches the digits fixed so far (LDS atomics, then one global atomic per
// non-empty bin).  Walking a histogram from the top to the wanted rank is the prologue of the NEXT
// kernel - every workgroup does it for itself, from the finished histogram of the launch before -
// so the select costs three launches, not six.  Integer counts only: the result does not depend
// on the order of the atomics.  Then one pass counts the values above the threshold per (work
// item, head), and one kernel with a workgroup per head gives every work item the first outlier
// row it owns (a prefix sum, no atomics: the rows of q_out are the same from run to run), turns
// the head totals into row offsets and into the tile list of the second attention, and clears
// the histograms for the next call.
#include "dev_common.hpp"
#include "kernels.hpp"

namespace httm {

namespace {

constexpr int kBins = 2048;
constexpr int kSelThreads = 256;
// threads per workgroup of the histogram passes: few workgroups (see launch_outlier_select), so many
// threads each - a thread then has one round of loads to wait for instead of four
constexpr int kHistThreads = 1024;

__device__ __forceinline__ uint32_t wave_inclusive_scan_u32(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(v, d);
    if (lane >= d) v += up;
  }
  return v;
}

// All NTHR threads of a workgroup: the bin of `hist` (kBins counts, bin = digit) that holds the
// value of descending rank `rank` (0 = the largest), and the rank inside that bin.
template <int NTHR>
__device__ __forceinline__ void pick_digit(const uint32_t* __restrict__ hist, uint32_t rank, uint32_t* digit,
                                           uint32_t* rank_in_bin) {
  constexpr int PER = kBins / NTHR;
  __shared__ uint32_t s_wave[NTHR / 64];
  __shared__ uint32_t s_res[2];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  uint32_t h[PER], mine = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    h[i] = hist[t * PER + i];
    mine += h[i];
  }
  const uint32_t incl = wave_inclusive_scan_u32(mine);
  const uint32_t wave_total = __shfl(incl, 63);
  if (lane == 63) s_wave[wave] = incl;
  if (t == 0) s_res[0] = s_res[1] = 0;
  __syncthreads();
  uint32_t above = wave_total - incl;   // values in the bins of the threads above this one
  for (int w = wave + 1; w < NTHR / 64; ++w) above += s_wave[w];
#pragma unroll
  for (int i = PER - 1; i >= 0; --i) {
    if (rank >= above && rank < above + h[i]) {
      s_res[0] = (uint32_t)(t * PER + i);
      s_res[1] = rank - above;
    }
    above += h[i];
  }
  __syncthreads();
  *digit = s_res[0];
  *rank_in_bin = s_res[1];
}

// The digits decided before pass PASS and the rank among the values that share them, from the
// histogram of the pass before (pass 0: nothing decided, the rank is the budget).  Workgroup 0
// leaves them in the state, where the next launch starts from.
template <int PASS>
__device__ __forceinline__ void select_prologue(const uint32_t* __restrict__ hist, SelectState* __restrict__ st,
                                                uint32_t budget, bool writer, uint32_t* prefix, uint32_t* rank) {
  if (PASS == 0) {
    *prefix = 0;
    *rank = budget;
    return;
  }
  uint32_t digit;
  if (PASS == 1) {
    pick_digit<kHistThreads>(hist, budget, &digit, rank);
    *prefix = digit;
    if (writer && threadIdx.x == 0) {
      st->prefix1 = *prefix;
      st->rank1 = *rank;
    }
  } else {
    pick_digit<kHistThreads>(hist + kBins, st->rank1, &digit, rank);
    *prefix = (st->prefix1 << 11) | digit;
    if (writer && threadIdx.x == 0) {
      st->prefix2 = *prefix;
      st->rank2 = *rank;
    }
  }
}

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
__global__ __launch_bounds__(kHistThreads) void select_hist_kernel(const uint32_t* __restrict__ keys,
                                                                  int64_t total, SelectState* __restrict__ st,
                                                                  uint32_t* __restrict__ hist, uint32_t budget) {
  __shared__ uint32_t s_hist[kBins];
  for (int b = threadIdx.x; b < kBins; b += kHistThreads) s_hist[b] = 0;
  uint32_t prefix, rank;
  select_prologue<PASS>(hist, st, budget, blockIdx.x == 0, &prefix, &rank);
  __syncthreads();
  // 16-byte loads; `keys` is 16-byte aligned and the tail is handled by the last threads
  const int64_t n4 = total >> 2;
  const int64_t stride = (int64_t)gridDim.x * kHistThreads;
  // (four independent loads per round: a thread has some 17 of them to do, and one at a time each
  // would cost a trip to memory)
  for (int64_t i = (int64_t)blockIdx.x * kHistThreads + threadIdx.x; i < n4; i += 4 * stride) {
    u32x4 w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) w[u] = ((const u32x4*)keys)[i + u * stride < n4 ? i + u * stride : i];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (i + u * stride >= n4) break;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        uint32_t d;
        if (digit_of<PASS>(w[u][q], prefix, &d)) atomicAdd(&s_hist[d], 1u);
      }
    }
  }
  if (blockIdx.x == 0) {
    for (int64_t i = (n4 << 2) + threadIdx.x; i < total; i += kHistThreads) {
      uint32_t d;
      if (digit_of<PASS>(keys[i], prefix, &d)) atomicAdd(&s_hist[d], 1u);
    }
  }
  __syncthreads();
  uint32_t* __restrict__ out = hist + PASS * kBins;
  for (int b = threadIdx.x; b < kBins; b += kHistThreads) {
    const uint32_t c = s_hist[b];
    if (c) atomicAdd(&out[b], c);
  }
}

// item_cnt[h][i] = number of deviations above tau among the tokens of work item i of head h, and
// wg_cnt[h][w] = their sum over the work items of workgroup w.  The prologue takes the last
// digit of tau from the third histogram.  One wave per (item, head) at a time, `items_per_wg` items
// per workgroup (fewer when the items are long, so that a wave does not walk several of them).
__global__ __launch_bounds__(kSelThreads) void outlier_count_kernel(const float* __restrict__ eps, int64_t N,
                                                                    const WorkItem* __restrict__ items, int n_items,
                                                                    SelectState* __restrict__ st,
                                                                    const uint32_t* __restrict__ hist,
                                                                    int32_t* __restrict__ item_cnt,
                                                                    int32_t* __restrict__ wg_cnt, int items_per_wg) {
  __shared__ int s_sum[kSelThreads / 64];
  uint32_t digit, rank_in_bin;
  pick_digit<kSelThreads>(hist + 2 * kBins, st->rank2, &digit, &rank_in_bin);
  const float tau = __uint_as_float((st->prefix2 << 10) | digit);
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) st->tau = tau;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int wave_sum = 0;
  for (int i = wave; i < items_per_wg; i += kSelThreads / 64) {
    const int item = blockIdx.x * items_per_wg + i;
    if (item >= n_items) break;
    const WorkItem it = items[item];
    const float* e = eps + (int64_t)blockIdx.y * N + it.start;
    int c = 0;
    for (int t = lane; t < it.n; t += 256) {   // four independent loads per round
      float v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = e[t + 64 * u < it.n ? t + 64 * u : t];
#pragma unroll
      for (int u = 0; u < 4; ++u) c += (t + 64 * u < it.n && v[u] > tau) ? 1 : 0;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d);
    if (lane == 0) item_cnt[(int64_t)blockIdx.y * n_items + item] = c;
    wave_sum += c;
  }
  if (lane == 0) s_sum[wave] = wave_sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    int tot = 0;
    for (int w = 0; w < kSelThreads / 64; ++w) tot += s_sum[w];
    wg_cnt[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = tot;
  }
}

// One workgroup per head h:
//  - item_base[h][i] = exclusive prefix sum of item_cnt[h][.], so that every work item knows the first
//    outlier row it owns (relative to its head);
//  - its share of the three histograms cleared for the next call;
//  - workgroup 0: the head totals from the sums of the count kernel's workgroups, the first outlier
//    row of every head and the (head, first row) list of the second attention's query tiles.
__global__ __launch_bounds__(kSelThreads) void outlier_offsets_kernel(const int32_t* __restrict__ item_cnt,
                                                                      int32_t* __restrict__ item_base, int n_items,
                                                                      int H, uint32_t* __restrict__ hist,
                                                                      const int32_t* __restrict__ wg_cnt, int n_wg,
                                                                      int32_t* __restrict__ counts,
                                                                      int32_t* __restrict__ offsets,
                                                                      int32_t* __restrict__ tiles, int tile_rows,
                                                                      int max_tiles) {
  __shared__ int s_part[kSelThreads / 64];
  __shared__ int s_slice[kSelThreads];
  __shared__ int s_total[HTTM_MAX_HEADS];
  const int t = threadIdx.x, h = blockIdx.x;
  if (h == 0) {
    // thread t adds a slice of head t % H (H <= 64: at least four slices), thread g < H the slices of head g
    const int slices = kSelThreads / H, g = t % H, sl = t / H;
    int sum = 0;
    if (sl < slices)
      for (int i = sl; i < n_wg; i += slices) sum += wg_cnt[(int64_t)g * n_wg + i];
    s_slice[t] = sum;
    __syncthreads();
    if (t < H) {
      int tot = 0;
      for (int u = 0; u < slices; ++u) tot += s_slice[u * H + t];
      s_total[t] = tot;
      counts[t] = tot;
    }
    __syncthreads();
  }
  for (int b = h * kSelThreads + t; b < 3 * kBins; b += H * kSelThreads) hist[b] = 0;
  // prefix sum over this head's work items
  {
    const int32_t* c = item_cnt + (int64_t)h * n_items;
    int32_t* o = item_base + (int64_t)h * n_items;
    const int per = (n_items + kSelThreads - 1) / kSelThreads;
    const int i0 = t * per, i1 = i0 + per < n_items ? i0 + per : n_items;
    int sum = 0;
    for (int i = i0; i < i1; ++i) sum += c[i];
    const int incl = (int)wave_inclusive_scan_u32((uint32_t)sum);
    if ((t & 63) == 63) s_part[t >> 6] = incl;
    __syncthreads();
    int base = incl - sum;
    for (int w = 0; w < (t >> 6); ++w) base += s_part[w];
    for (int i = i0; i < i1; ++i) {
      o[i] = base;
      base += c[i];
    }
  }
  if (h != 0) return;
  // first outlier row and first tile of every head (lane g of the first wave looks after head g),
  // then the tile list with all threads
  __shared__ int s_first[HTTM_MAX_HEADS + 1];
  if (t < 64) {
    int32_t off = 0, first_tile = 0, mine = 0;
    for (int g = 0; g < H; ++g) {
      const int32_t c = s_total[g];
      if (g < t) {
        off += c;
        first_tile += (c + tile_rows - 1) / tile_rows;
      }
      if (g == t) mine = c;
    }
    if (t < H) {
      offsets[t] = off;
      s_first[t] = first_tile;
      if (t == H - 1) {
        offsets[H] = off + mine;
        const int nt = first_tile + (mine + tile_rows - 1) / tile_rows;
        s_first[H] = nt < max_tiles ? nt : max_tiles;
        tiles[0] = s_first[H];
      }
    }
  }
  __syncthreads();
  for (int nt = t; nt < s_first[H]; nt += kSelThreads) {
    int g = 0;
    while (g + 1 < H && s_first[g + 1] <= nt) ++g;
    tiles[1 + 2 * nt] = g;
    tiles[2 + 2 * nt] = (nt - s_first[g]) * tile_rows;
  }
}

}  // namespace

hipError_t launch_outlier_select(const float* eps, int H, int64_t N, int64_t budget,
                                 const WorkItem* items, int n_items, int max_block, const OutlierBuffers& b,
                                 int tile_rows, hipStream_t stream) {
  const int64_t total = (int64_t)H * N;
  if (total == 0) return hipSuccess;
  const uint32_t* keys = (const uint32_t*)eps;
  // Few workgroups: each ends with one global atomic per non-empty bin, and the values crowd into
  // a handful of bins in the first pass, so the number of workgroups is what serialises there.
  int64_t want = (total / 4 + kHistThreads - 1) / kHistThreads;
  const unsigned grid = (unsigned)(want < 1 ? 1 : (want > 256 ? 256 : want));
  const uint32_t bud = (uint32_t)budget;
  hipLaunchKernelGGL(select_hist_kernel<0>, dim3(grid), dim3(kHistThreads), 0, stream, keys, total, b.state, b.hist, bud);
  hipLaunchKernelGGL(select_hist_kernel<1>, dim3(grid), dim3(kHistThreads), 0, stream, keys, total, b.state, b.hist, bud);
  hipLaunchKernelGGL(select_hist_kernel<2>, dim3(grid), dim3(kHistThreads), 0, stream, keys, total, b.state, b.hist, bud);
  const int per_wg = max_block > 1024 ? kOutlierCountItemsMin : kOutlierCountItems;
  const int n_wg = (n_items + per_wg - 1) / per_wg;
  hipLaunchKernelGGL(outlier_count_kernel, dim3((unsigned)n_wg, (unsigned)H), dim3(kSelThreads), 0, stream, eps, N, items,
                     n_items, b.state, b.hist, b.item_cnt, b.wg_cnt, per_wg);
  hipLaunchKernelGGL(outlier_offsets_kernel, dim3((unsigned)H), dim3(kSelThreads), 0, stream, b.item_cnt, b.item_base,
                     n_items, H, b.hist, b.wg_cnt, n_wg, b.counts, b.offsets, b.tiles, tile_rows, b.max_tiles);
  return hipGetLastError();
}

}  // namespace httm
