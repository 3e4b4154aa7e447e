// Stage 3: attention over the reduced per-head sequences (paper Sec. 3.2 Eq. 3-4):
//   O = softmax(Q K^T * scale) V, per head, no mask, ragged (M_q[h], M_k[h]).
//
// Flash-style single pass with bf16 MFMA (v_mfma_f32_32x32x16_bf16) and fp32 softmax state.
// The kernel is bound by the matrix cores (4*M_q*M_k*64 flop per head against a few MB of
// K/V that stay in L2 / Infinity Cache); with d_head = 64 the softmax needs about as many
// vector-ALU cycles as the two matrix products need MFMA cycles, so the design is about
// (a) taking vector instructions out of the inner loop and (b) giving every wave independent
// MFMA and vector work in the same stretch of code so that both pipes run at once.
//
// Work decomposition
//   * workgroup = NW waves = one tile of 32*QT*NW query rows of one head; a wave owns 32*QT rows;
//   * K/V are streamed in tiles of 64 rows through LDS, double buffered, one barrier per tile;
//   * blockIdx -> tile mapping is XCD-aware: workgroups are dispatched round-robin over the 8
//     XCDs, so tile = (bid % 8) * (grid/8) + bid / 8 gives every XCD a contiguous range of
//     tiles, i.e. about two heads, whose K/V then stay in that XCD's L2.
//
// Transposed formulation.  Each wave computes S^T = K Q^T (A = K tile from LDS, B = Q^T from
// registers) so that in the 32x32 accumulator layout a lane owns ONE query column and 16 of the
// 32 key rows: the softmax reductions are sums inside a lane plus one exchange with lane^32 at
// the very end, and every per-row quantity is a per-lane scalar for the O^T = V^T P^T
// accumulators as well.  P^T goes from the accumulator registers straight into the B operand of
// the second MFMA (fp32 -> bf16 in registers, no LDS round trip).  That fixes which 8 keys a lane
// supplies per MFMA step: {16j + 4*half + 0..3, 16j + 8 + 4*half + 0..3}.  The matching A operand
// (V^T: a lane's channel, those 8 keys) comes out of the row-major V tile through two transposing
// LDS reads (ds_read_b64_tr_b16), so V is never transposed in memory or in registers.
//
// Both tiles go from global memory straight into LDS (global_load_lds_dwordx4: no registers, no
// LDS store instructions); every lane fetches the 16-byte chunk that belongs at its position
// under the tile's swizzle, which keeps the operand reads free of bank conflicts.
//
// Software pipeline.  Work is cut into steps of 32 keys.  In step t a wave issues, in one
// basic block, the QK^T MFMAs of step t+1, the PV MFMAs of step t-1 and the softmax of step t:
// the 16 MFMAs do not depend on the ~100 vector instructions next to them, so the matrix core
// and the vector ALU overlap inside a single wave (two waves per SIMD then fill what is left).
// V lags K by one tile in LDS because of the t-1.  In the steady state the order of issue is
// written out (steady_step(): one MFMA, then two exp2 and a pack, behind a scheduling fence), the
// loop runs two tiles per trip so that the LDS buffer indices are constants, and the global->LDS
// requests of an iteration are issued behind the last LDS read of its first step.
//
// Softmax without a running maximum.  softmax is invariant to the per-row shift m, and fp32 /
// bf16 keep their relative precision over the whole exponent range, so m only has to keep
// exp2(s - m) inside that range - it does not have to be the maximum.  Per row, m is the exact
// maximum of the first 32 keys and is then left alone; the vector ALU does one fma (scale and
// shift), exp2, the bf16 conversion and the row sum (a bf16 dot2 against ones) per score, and no
// max, no rescaling of O.  Because the first block's maximum contributes exp2(0) = 1, the row
// sum can never underflow.  Overflow is caught: if a lane's partial row sum of a step is not
// below 2^60 (this also catches inf / NaN), the wave redoes that step's softmax with m raised to
// the step's true maximum and rescales its O and l accumulators - the classic online-softmax
// update, taken only when needed.
//
// Two kernels.  The one described so far (SHIFT = true) takes any keys and any scale.  When stage 2
// has left the merged keys multiplied by scale * log2(e) ("log2 keys": the factor goes into the
// fp32 mean before its one rounding to bf16, so nothing is rounded twice), the raw MFMA scores are
// the base-2 logits, and the fast kernel (SHIFT = false) uses the weights exp2(s) as they are: no
// fma, no shift - a quarter of the vector work per score gone - and takes the row sums from the
// matrix cores as well (row_sum_operand()).  That is safe while a row's sum
// stays well inside the fp32 range; every workgroup checks its final row sums against
// [2^-64, 2^64] and, if a row is outside (or inf / NaN), writes a mark instead of its tile.  The
// SHIFT kernel is launched right behind on the same grid and redoes exactly the marked tiles.
//
// End of a launch.  A CU runs its 256-row tiles two at a time, but one alone nearly twice as fast,
// so the launch time follows the largest number of whole tiles a CU gets.  When the caller has given
// scratch memory, the tiles in excess of a multiple of the CU count are not run whole: their work
// is cut into equal shares over the keys, one or two per CU, that are dispatched behind the whole
// tiles, and attention_split_reduce_kernel adds the pieces of every tile up (attention_split.hpp).
#include <cstring>
#include <mutex>
#include <type_traits>

#include "attention_split.hpp"
#include "dev_common.hpp"
#include "kernels.hpp"

namespace httm {

namespace {

constexpr int kKvTile = 64;
constexpr int kStep = 32;                               // keys per pipeline step
constexpr float kSumLimit = 1.152921504606846976e18f;  // 2^60
constexpr float kShiftLimit = 60.0f;

struct AttnArgs {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  bf16_t* o;
  float scale_log2;  // scale * log2(e); 1 when the keys carry that factor already
  int32_t marked_only;  // the kernel with per-row shifts redoes only the tiles the fast kernel marked
  int32_t H;
  int32_t n_full;                             // tiles with all BQ query rows
  int32_t n_ragged;                           // heads whose last tile is partial
  int32_t full_per_xcd;                       // ceil(n_full / 8)
  int32_t ragged_per_xcd;                     // ceil(n_ragged / 8)
  int32_t tile_start[kAttnMaxHeads + 1];      // first full tile of every head
  int32_t ragged_head[kAttnMaxHeads];         // head of every partial tile
  int64_t q_off[kAttnMaxHeads + 1];
  int64_t k_off[kAttnMaxHeads + 1];
  // When set, a second set of query tiles is described by device memory: rows of head h are
  // [dev_q_off[h], dev_q_off[h+1]) and workgroup t takes tile (head, first row) =
  // (dev_tiles[1+2t], dev_tiles[2+2t]) for t < dev_tiles[0].
  // The workgroups behind the whole tiles and the segments take these tiles; their queries and outputs
  // are q2 / o2.
  const int32_t* dev_q_off;
  const int32_t* dev_tiles;
  const bf16_t* q2;
  bf16_t* o2;
  // Every XCD (workgroup b goes to XCD b % 8) walks a sequence of full_per_xcd + ragged_per_xcd whole
  // tiles and then split_per_xcd shares of the tiles that run in segments over the keys
  // (attention_split.hpp; none in a launch that only redoes marked tiles).  A segment writes
  // un-normalised fp32 results into its slot of the scratch memory and attention_split_reduce_kernel
  // adds them up.  The workgroups behind main_blocks = 8 * (sequence length) take the device-side tile
  // list.  n_ragged / ragged_head and n_full count only the tiles that stay whole.
  int32_t split_per_xcd;
  int32_t main_blocks;
  float* split_o;   // [slots * 256][64] sums of weight * v
  float* split_l;   // [slots * 256]     sums of weights
  float* split_m;   // [slots * 256]     the rows' shifts (kernel with per-row shifts only)
  SplitPlan sp;
};
static_assert(sizeof(AttnArgs) <= 4096, "kernel arguments are limited to 4 KB");

// V tile in LDS: 64 rows of 128 bytes, written by global->LDS loads like the K tile; the 16-byte
// chunk c of row r sits at chunk position c ^ (2 * (r & 3)), so that the four rows a transposing read
// touches (32 bytes each, same channels) fall into four different 32-byte bank groups.
__device__ __forceinline__ int v_swizzle(int row) { return (row & 3) << 1; }

__device__ __forceinline__ f32x16 splat16(float x) {
  f32x16 r;
#pragma unroll
  for (int i = 0; i < 16; ++i) r[i] = x;
  return r;
}

// Per-wave softmax state and accumulators.
template <int QT>
struct WaveState {
  bf16x8 qf[QT][4];      // Q^T fragments
  f32x16 o_acc[2][QT];   // O^T accumulators, [channel tile][query tile]
  f32x16 s_cur[QT];      // raw scores of the current step
  u32x4 p_old[QT][2];    // bf16 P^T of the previous step, packed as MFMA B operands
  float mc[QT];          // shift m in log2 units
  float c;               // factor from raw scores to log2 units (kernel with per-row shifts only)
  float l_run[QT];       // per-lane partial row sums (kernel with per-row shifts)
  f32x4 l_acc[QT];       // row sums of the fast kernel, from the matrix cores: see row_sum_operand()
  bf16x8 ones_a;
};

// Row sums on the matrix cores (fast kernel).  The P^T registers of a lane (query l%32, keys of
// half l/32) read as the B operand of a 16x16x32 MFMA put query l%32 in column l%16 and its
// 8 keys in k-group l/16: column n collects query n from k-groups 0 and 2 and query n+16 from
// k-groups 1 and 3.  An A operand with ones in row 0 over k-groups {0, 2} and in row 1 over {1, 3}
// therefore gives D[0][n] = sum over the 16 keys of query n and D[1][n] = the same for query n+16:
// registers 0 and 1 of lanes 0..15.
__device__ __forceinline__ bf16x8 row_sum_operand(int lane) {
  const int m = lane & 15, kg = lane >> 4;
  const bool one = (m == 0 && (kg & 1) == 0) || (m == 1 && (kg & 1) == 1);
  const uint32_t w = one ? 0x3F803F80u : 0u;
  return __builtin_bit_cast(bf16x8, u32x4{w, w, w, w});
}

// exp2(s*c - m) (SHIFT) or exp2(s), bf16 pack and row sum of one query tile.
template <bool SHIFT>
__device__ __forceinline__ float exp_pack(const f32x16& s, float c, float m, u32x4 (&p)[2]) {
  const bf16x2 ones2 = {(bf16_t)1.0f, (bf16_t)1.0f};
  float ps = 0.f;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float p0 = __builtin_amdgcn_exp2f(SHIFT ? fmaf(s[8 * j + 2 * e], c, -m) : s[8 * j + 2 * e]);
      const float p1 = __builtin_amdgcn_exp2f(SHIFT ? fmaf(s[8 * j + 2 * e + 1], c, -m) : s[8 * j + 2 * e + 1]);
      const uint32_t w = pack_bf16x2(p0, p1);
      p[j][e] = w;
      if (SHIFT) ps = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), ones2, ps, false);
    }
  return ps;
}

// MFMA A operands of one step: 4 K fragments (32 key rows x 64 channels) and 4 V^T fragments
// (64 channels x 32 key positions), 16 bytes per lane each.
struct StepOperands {
  bf16x8 ak[4];
  bf16x8 av[4];
};

// K tile in LDS: 64 rows of 128 bytes, unpadded (it is written by global->LDS loads, 1 KB per
// wave instruction); the 16-byte chunk c of row r sits at chunk position c ^ ((r >> 1) & 7), which
// makes the operand reads of 16 consecutive rows hit 16 distinct bank groups.
__device__ __forceinline__ int k_swizzle(int row) { return (row >> 1) & 7; }

// `sk` points at the first of the 32 rows of this step (row 0 or 32 of the tile).
__device__ __forceinline__ void load_k_operands(StepOperands& op, const bf16_t* sk, int l32, int half) {
  const int sw = k_swizzle(l32);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
    op.ak[ks] = *(const bf16x8*)(sk + l32 * kDHead + ((ks * 2 + half) ^ sw) * 8);
}
// A operands of O^T += V^T P^T from the row-major V tile: ds_read_b64_tr_b16 hands lane 4a+e of a
// 16-lane group element e of the 8 bytes that lane 4r+a of the group addressed, as its r-th value.
// Lane 4r+a addresses key k0+r, channels c0+4a..c0+4a+3, so lane i receives keys k0..k0+3 of channel
// c0+i - four consecutive keys of one V^T row.  Two reads (k0 = 16j + 4*half and 8 keys further)
// give the 8 keys a lane's P^T registers hold; the four groups of a wave are (half, 16 channels).
// `sv` points at the first of the 32 key rows of this step.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
__device__ __forceinline__ void load_v_operands(StepOperands& op, const bf16_t* sv, int l32, int half) {
  const int i = l32 & 15, chalf = l32 >> 4;
  const int krow = 4 * half + (i >> 2);
#pragma unroll
  for (int dt = 0; dt < 2; ++dt) {
    const int chunk = (4 * dt + 2 * chalf + ((i & 3) >> 1)) ^ v_swizzle(krow);
    const bf16_t* base = sv + krow * kDHead + chunk * 8 + 4 * (i & 1);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(base + (16 * j) * kDHead));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(base + (16 * j + 8) * kDHead));
      op.av[dt * 2 + j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  }
}

// One pipeline step of a wave outside the steady state (first tile, last tile, drain); the order of
// issue is the compiler's.
//   DO_QK : scores of the NEXT step from the 32 K rows at `sk`           -> becomes s_cur
//   DO_PV : O^T += V^T P^T of the PREVIOUS step, V rows at `svt`
//   DO_SM : softmax of the CURRENT step (s_cur -> p_old); its first key is `kv_first`
//   MASK  : keys >= Mk get weight 0;  FIRST : this is step 0 and fixes m
template <int QT, bool SHIFT, bool DO_QK, bool DO_PV, bool DO_SM, bool MASK, bool FIRST>
__device__ __forceinline__ void pipeline_step(WaveState<QT>& w, const bf16_t* sk, const bf16_t* svt,
                                              int kv_first, int Mk, int l32, int half) {
  StepOperands op;
  f32x16 s_next[QT];
  if (DO_QK) {
    load_k_operands(op, sk, l32, half);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
        s_next[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            op.ak[ks], w.qf[qt][ks], ks == 0 ? splat16(0.f) : s_next[qt], 0, 0, 0);
  }
  if (DO_PV) {
    load_v_operands(op, svt, l32, half);
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          w.o_acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
              op.av[dt * 2 + j], __builtin_bit_cast(bf16x8, w.p_old[qt][j]), w.o_acc[dt][qt], 0, 0, 0);
    if (!SHIFT) {
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          w.l_acc[qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              w.ones_a, __builtin_bit_cast(bf16x8, w.p_old[qt][j]), w.l_acc[qt], 0, 0, 0);
    }
  }
  if (DO_SM) {
    // s_cur[qt][r]: key kv_first + 8*(r/4) + 4*half + r%4, query column l32 of tile qt
    if (MASK) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int kv = kv_first + 8 * (r >> 2) + 4 * half + (r & 3);
        if (kv >= Mk) {
#pragma unroll
          for (int qt = 0; qt < QT; ++qt) w.s_cur[qt][r] = -INFINITY;
        }
      }
    }
    u32x4 p_new[QT][2];
    float psum[QT];
    if (!SHIFT) {
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) psum[qt] = exp_pack<false>(w.s_cur[qt], 1.f, 0.f, p_new[qt]);
    } else if (FIRST) {
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        float tmax = w.s_cur[qt][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, w.s_cur[qt][r]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        w.mc[qt] = tmax * w.c;
        psum[qt] = exp_pack<true>(w.s_cur[qt], w.c, w.mc[qt], p_new[qt]);
      }
    } else {
      bool redo = false;
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        psum[qt] = exp_pack<true>(w.s_cur[qt], w.c, w.mc[qt], p_new[qt]);
        redo = redo || !(psum[qt] < kSumLimit);
      }
      // rare: raise m to this step's maximum where needed and redo the step's softmax
      if (__any(redo)) {
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
          float tmax = w.s_cur[qt][0];
#pragma unroll
          for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, w.s_cur[qt][r]);
          tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
          const float rel = fmaf(tmax, w.c, -w.mc[qt]);  // log2 units above the current m
          const float delta = rel > kShiftLimit ? rel : 0.f;
          const float sc = __builtin_amdgcn_exp2f(-delta);
          w.l_run[qt] *= sc;
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) w.o_acc[dt][qt][r] *= sc;
          w.mc[qt] += delta;
          psum[qt] = exp_pack<true>(w.s_cur[qt], w.c, w.mc[qt], p_new[qt]);
        }
      }
    }
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      if (SHIFT) w.l_run[qt] += psum[qt];
#pragma unroll
      for (int j = 0; j < 2; ++j) w.p_old[qt][j] = p_new[qt][j];
    }
  }
  if (DO_QK) {
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) w.s_cur[qt] = s_next[qt];
  }
}

// The steady-state step (of both kernels) with the order of issue written out: one MFMA, then its
// share of the softmax of the current step (two exp2, one bf16 pack of the pair before), fenced so
// that the compiler keeps the interleave.  PV of step t-1 first (the V operands retire, their
// successors are requested), then QK^T of step t+1 and the K operands; a row-sum MFMA after every
// fourth product.  `between` runs after the step's last LDS read: the global->LDS requests of the
// iteration go there, because the compiler makes every LDS read wait for all requests issued
// before it in program order.
template <int QT, bool SHIFT, bool PREFETCH, typename Between>
__device__ __forceinline__ void steady_step(WaveState<QT>& w, StepOperands& op, const bf16_t* sk_next,
                                            const bf16_t* sv_next, int l32, int half, Between between) {
  // 8 * QT groups: 4 * QT products of each kind, every group with 2 of the 16 * QT scores of the lane
  constexpr int NG = 8 * QT;
  f32x16 s_next[QT];
  float ex[16 * QT];
  u32x4 p_new[QT][2];
  float psum[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) psum[qt] = 0.f;
  const bf16x2 ones2 = {(bf16_t)1.0f, (bf16_t)1.0f};
  auto soft = [&](int g) {   // values 2g, 2g+1 of the 32 scores of this lane
    // (the empty asm after a result only pins where the instruction is issued)
    const int qt = (2 * g) >> 4;
    const float x0 = w.s_cur[qt][(2 * g) & 15], x1 = w.s_cur[qt][(2 * g + 1) & 15];
    ex[2 * g] = __builtin_amdgcn_exp2f(SHIFT ? fmaf(x0, w.c, -w.mc[qt]) : x0);
    asm volatile("" : "+v"(ex[2 * g]));
    ex[2 * g + 1] = __builtin_amdgcn_exp2f(SHIFT ? fmaf(x1, w.c, -w.mc[qt]) : x1);
    asm volatile("" : "+v"(ex[2 * g + 1]));
  };
  auto pack = [&](int p) {
    uint32_t r = pack_bf16x2(ex[2 * p], ex[2 * p + 1]);
    asm volatile("" : "+v"(r));
    p_new[p >> 3][(p & 7) >> 2][p & 3] = r;
    if (SHIFT) {
      psum[p >> 3] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, r), ones2, psum[p >> 3], false);
      asm volatile("" : "+v"(psum[p >> 3]));
    }
  };
  auto row_sum = [&](int g) {   // a row-sum MFMA after every fourth product: 2 * QT per step, (query tile, j)
    if (!SHIFT && (g & 3) == 3) {
      const int r = g >> 2, rq = r % QT, rj = r / QT;
      w.l_acc[rq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
          w.ones_a, __builtin_bit_cast(bf16x8, w.p_old[rq][rj]), w.l_acc[rq], 0, 0, 0);
    }
  };
  // PV of step t-1 first: the V operands retire and their successors are requested ...
#pragma unroll
  for (int g = 0; g < NG / 2; ++g) {
    const int qt = g % QT, dt = (g / QT) & 1, j = g / (2 * QT);
    w.o_acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
        op.av[dt * 2 + j], __builtin_bit_cast(bf16x8, w.p_old[qt][j]), w.o_acc[dt][qt], 0, 0, 0);
    soft(g);
    if (g > 0) pack(g - 1);
    row_sum(g);
    __builtin_amdgcn_sched_barrier(0);
  }
  if (PREFETCH) {
    load_v_operands(op, sv_next, l32, half);
    __builtin_amdgcn_sched_barrier(0);
  }
  // ... then QK^T of step t+1
#pragma unroll
  for (int g = NG / 2; g < NG; ++g) {
    const int i = g - NG / 2, ks = i / QT, qt = i % QT;
    s_next[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op.ak[ks], w.qf[qt][ks],
                                                         ks == 0 ? splat16(0.f) : s_next[qt], 0, 0, 0);
    soft(g);
    pack(g - 1);
    row_sum(g);
    __builtin_amdgcn_sched_barrier(0);
  }
  pack(NG - 1);
  if (PREFETCH) load_k_operands(op, sk_next, l32, half);
  __builtin_amdgcn_sched_barrier(0);
  between();        // requests that must follow the step's last LDS read in program order
  __builtin_amdgcn_sched_barrier(0);
  if (SHIFT) {
    // rare: raise m to this step's maximum where a row sum left the range, redo the step's weights
    bool redo = false;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) redo = redo || !(psum[qt] < kSumLimit);
    if (__any(redo)) {
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        float tmax = w.s_cur[qt][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, w.s_cur[qt][r]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float rel = fmaf(tmax, w.c, -w.mc[qt]);
        const float delta = rel > kShiftLimit ? rel : 0.f;
        const float sc = __builtin_amdgcn_exp2f(-delta);
        w.l_run[qt] *= sc;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) w.o_acc[dt][qt][r] *= sc;
        w.mc[qt] += delta;
        psum[qt] = exp_pack<true>(w.s_cur[qt], w.c, w.mc[qt], p_new[qt]);
      }
    }
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) w.l_run[qt] += psum[qt];
  }
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    w.s_cur[qt] = s_next[qt];
#pragma unroll
    for (int j = 0; j < 2; ++j) w.p_old[qt][j] = p_new[qt][j];
  }
}

// bf16 bit pattern (a NaN with a payload that arithmetic does not produce) that the fast kernel
// leaves in channel 0 of a tile's first output row when the tile has to be redone.
constexpr uint16_t kRedoMark = 0x7FA5;
// Row sums the fast kernel accepts (inf and NaN fail the test as well): inside, the weights of a
// row's best keys are far from both ends of the fp32 range, and no weight exceeds 2^64, so that the
// unnormalised products with V stay finite for |v| below 1e19.
constexpr float kFastSumMin = 5.421010862427522e-20f;    // 2^-64
constexpr float kFastSumMax = 1.8446744073709552e19f;    // 2^64

// One query tile (or one segment of it) of a workgroup: see attention_kernel.
//   h, q0          : head and first query row of the tile
//   dev_tile       : the tile comes from the device-side list (rows q_base_dev .. + mq_dev of q2 / o2)
//   seg.slot >= 0  : only the key tiles [seg.t0, seg.t1) of the head, results into scratch slot seg.slot
template <int QT, int NW, bool SHIFT>
__device__ __forceinline__ void attention_tile(const AttnArgs& a, bf16_t (*s_k)[kKvTile * kDHead],
                                               bf16_t (*s_v)[kKvTile * kDHead], const int h, const int q0,
                                               const bool dev_tile, const int64_t q_base_dev, const int mq_dev,
                                               const SplitSegment seg) {
  constexpr int NT = 64 * NW;
  constexpr int BQ = 32 * QT * NW;
  constexpr int LDK = 8 / NW;                              // 1 KB global->LDS loads per wave per tile
  const bool piece = seg.slot >= 0;
  const int64_t q_base = dev_tile ? q_base_dev : a.q_off[h];
  int64_t k_base = a.k_off[h];
  const int Mq = dev_tile ? mq_dev : (int)(a.q_off[h + 1] - q_base);
  const bf16_t* __restrict__ q_rows = dev_tile ? a.q2 : a.q;
  bf16_t* __restrict__ o_rows = dev_tile ? a.o2 : a.o;
  int Mk = (int)(a.k_off[h + 1] - k_base);
  uint16_t* mark = (uint16_t*)(o_rows + (q_base + q0) * kDHead);
  if (SHIFT && a.marked_only && (Mk == 0 || *(volatile const uint16_t*)mark != kRedoMark)) return;

  // (the empty asm keeps per-lane values that derive from the thread index from being computed once
  // in front of the loop over a share's segments and held in registers across the whole tile)
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  // a segment sees its key tiles as the whole key sequence
  const int64_t piece_row0 = (int64_t)(piece ? seg.slot : 0) * BQ;
  if (piece) {
    k_base += (int64_t)seg.t0 * kKvTile;
    Mk = (seg.t1 * kKvTile < Mk ? seg.t1 * kKvTile : Mk) - seg.t0 * kKvTile;
  }
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: LDS destinations stay scalar
  const int l32 = lane & 31, half = lane >> 5;
  const int wq0 = q0 + wave * 32 * QT;  // first query row of this wave
  // A wave of a partial tile that owns no valid row only helps to stage K/V and to keep the
  // barriers; it issues no MFMA and no softmax.
  const bool active = __builtin_amdgcn_readfirstlane((int)(wq0 < Mq)) != 0;   // wave-uniform, and known to be

  if (Mk == 0) {
    // softmax over an empty key set: defined as zero output
    for (int e = tid; e < BQ * kRowChunks; e += NT) {
      const int row = q0 + (e >> 3);
      if (row < Mq) ((u32x4*)o_rows)[(q_base + row) * kRowChunks + (e & 7)] = u32x4{0, 0, 0, 0};
    }
    return;
  }

  WaveState<QT> w;
  // ---- Q^T fragments (B operand): lane -> query column, 8 consecutive channels ---------------
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    int row = wq0 + qt * 32 + l32;
    row = row < Mq ? row : Mq - 1;
    const bf16_t* p = q_rows + (q_base + row) * kDHead + half * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) w.qf[qt][ks] = *(const bf16x8*)(p + ks * 16);
    w.mc[qt] = 0.f;
    w.l_run[qt] = 0.f;
    w.l_acc[qt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < 2; ++dt) w.o_acc[dt][qt] = splat16(0.f);
  }

  // ---- K/V tile staging: global -> registers -> LDS ---------------------------------------------
  const char* kg = (const char*)(a.k + k_base * kDHead);   // wave-uniform bases; per-lane offsets
  const char* vg = (const char*)(a.v + k_base * kDHead);   // below fit 32 bits (rows < 2^24 here)
  // K: straight from global memory into LDS, no registers.  Lane l of a wave instruction fills
  // bytes [16 l, 16 l + 16) of a 1 KB block = rows 8*blk .. 8*blk+7; it fetches the chunk that
  // belongs at its position under the swizzle.
  auto load_k = [&](int kv0, int buf, bool inside = false) {   // inside: the whole tile lies below Mk
#pragma unroll
    for (int i = 0; i < LDK; ++i) {
      const int blk = wave * LDK + i;
      const int r = blk * 8 + (lane >> 3);
      const int c = (lane & 7) ^ k_swizzle(r);
      int row = kv0 + r;
      if (!inside) row = row < Mk ? row : Mk - 1;
      const char* src = kg + (uint32_t)(row * kRowBytes + c * 16);
      bf16_t* dst = &s_k[buf][blk * 512];
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    }
  };
  // V the same way, under its own swizzle
  auto load_v = [&](int kv0, int buf, bool inside = false) {
#pragma unroll
    for (int i = 0; i < LDK; ++i) {
      const int blk = wave * LDK + i;
      const int r = blk * 8 + (lane >> 3);
      const int c = (lane & 7) ^ v_swizzle(r);
      int row = kv0 + r;
      if (!inside) row = row < Mk ? row : Mk - 1;
      const char* src = vg + (uint32_t)(row * kRowBytes + c * 16);
      bf16_t* dst = &s_v[buf][blk * 512];
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                       (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
    }
  };

  w.c = a.scale_log2;
  w.ones_a = row_sum_operand(lane);
  const int n_tiles = (Mk + kKvTile - 1) / kKvTile;

  // Steps are numbered t = 0 .. 2*n_tiles-1 (32 keys each).  Outer iteration j runs the pipeline
  // slots t = 2j-1 and t = 2j, which read K tile j (scores of steps 2j, 2j+1) and V tile j-1
  // (products of steps 2j-2, 2j-1), while K tile j+1 and V tile j are on their way into the
  // other LDS buffers.

  // ---- j = 0 ---------------------------------------------------------------------------------------
  load_k(0, 0);
  load_v(0, 0);
  if (n_tiles > 1) load_k(kKvTile, 1);
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the global->LDS loads have landed
  __syncthreads();
  if (active) {
    pipeline_step<QT, SHIFT, true, false, false, false, false>(w, &s_k[0][0], nullptr, 0, Mk, l32, half);
    if (n_tiles > 1)
      pipeline_step<QT, SHIFT, true, false, true, false, true>(w, &s_k[0][kStep * kDHead], nullptr, 0,
                                                        Mk, l32, half);
    else
      pipeline_step<QT, SHIFT, true, false, true, true, true>(w, &s_k[0][kStep * kDHead], nullptr, 0,
                                                       Mk, l32, half);
  }
  __syncthreads();

  // ---- j = 1 .. n_tiles-2: steady state, no masking ------------------------------------------------
  int j = 1;
  StepOperands op;
  // Two tiles per trip with the buffer indices as constants (j is odd at the top): the LDS
  // addresses become instruction offsets instead of a dozen vector adds per tile.
  auto steady_tile = [&](auto parity, int jt) {
    constexpr int P = decltype(parity)::value;        // jt & 1
    const bf16_t* kb = &s_k[P][0];
    const bf16_t* vb = &s_v[P ^ 1][0];
    auto request = [&]() {
      if ((jt + 2) * kKvTile <= Mk)
        load_k((jt + 1) * kKvTile, P ^ 1, true);
      else
        load_k((jt + 1) * kKvTile, P ^ 1);
      load_v(jt * kKvTile, P, true);                     // jt < n_tiles - 1: a full tile
    };
    // (a wave without valid rows runs the loop below instead: no global->LDS request may precede
    // an LDS read on the path of an active wave, the compiler would wait for it before the read)
    load_k_operands(op, kb, l32, half);
    load_v_operands(op, vb, l32, half);
    steady_step<QT, SHIFT, true>(w, op, kb + kStep * kDHead, vb + kStep * kDHead, l32, half, request);
    steady_step<QT, SHIFT, false>(w, op, nullptr, nullptr, l32, half, [] {});
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): K tile jt+1 and V tile jt are in LDS
    __syncthreads();
  };
  if (!active) {
    // a wave of a partial tile without valid rows: it only stages its share of K / V
    for (; j < n_tiles - 1; ++j) {
      load_k((j + 1) * kKvTile, (j + 1) & 1);
      load_v(j * kKvTile, j & 1);
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
    }
  } else {
    for (; j + 1 < n_tiles - 1; j += 2) {
      steady_tile(std::integral_constant<int, 1>{}, j);
      steady_tile(std::integral_constant<int, 0>{}, j + 1);
    }
    if (j < n_tiles - 1) {
      steady_tile(std::integral_constant<int, 1>{}, j);
      ++j;
    }
  }

  // ---- j = n_tiles-1 (if it is not j = 0): the last K tile, its first step may be ragged ---------
  if (j == n_tiles - 1) {
    load_v(j * kKvTile, j & 1);
    const bf16_t* kb = &s_k[j & 1][0];
    const bf16_t* vb = &s_v[(j - 1) & 1][0];
    if (active) {
      pipeline_step<QT, SHIFT, true, true, true, false, false>(w, kb, vb, 0, Mk, l32, half);
      pipeline_step<QT, SHIFT, true, true, true, true, false>(w, kb + kStep * kDHead, vb + kStep * kDHead,
                                                       2 * j * kStep, Mk, l32, half);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the last V tile is in LDS
    __syncthreads();
  }

  // ---- j = n_tiles: drain ---------------------------------------------------------------------------
  if (active) {
    const bf16_t* vb = &s_v[(n_tiles - 1) & 1][0];
    pipeline_step<QT, SHIFT, false, true, true, true, false>(w, nullptr, vb, (2 * n_tiles - 1) * kStep, Mk,
                                                      l32, half);
    pipeline_step<QT, SHIFT, false, true, false, false, false>(w, nullptr, vb + kStep * kDHead, 0, Mk, l32, half);
  }

  float l_tot[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    if (SHIFT) {
      l_tot[qt] = w.l_run[qt] + __shfl_xor(w.l_run[qt], 32);
    } else {
      const float s0 = __shfl(w.l_acc[qt][0], l32 & 15), s1 = __shfl(w.l_acc[qt][1], l32 & 15);
      l_tot[qt] = l32 < 16 ? s0 : s1;
    }
  }
  if (piece) {
    // a segment: unnormalised sums (and the shifts they are relative to) for attention_split_reduce_kernel
    if (active) {
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        const int row = wq0 + qt * 32 + l32;
        if (row < Mq) {
          // slot layout [16 channel groups of 4][BQ rows][4]: group (dt * 4 + g) * 2 + half holds the
          // channels dt * 32 + 8 * g + 4 * half .. + 3, so that the 32 lanes of a half write 512
          // contiguous bytes and the kernel that adds the segments up reads whole lines
          float* po = a.split_o + piece_row0 * kDHead + (row - q0) * 4;
#pragma unroll
          for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int g = 0; g < 4; ++g)
              *(f32x4*)(po + ((dt * 4 + g) * 2 + half) * (BQ * 4)) =
                  f32x4{w.o_acc[dt][qt][4 * g], w.o_acc[dt][qt][4 * g + 1], w.o_acc[dt][qt][4 * g + 2],
                        w.o_acc[dt][qt][4 * g + 3]};
          if (half == 0) {
            a.split_l[piece_row0 + (row - q0)] = l_tot[qt];
            if (SHIFT) a.split_m[piece_row0 + (row - q0)] = w.mc[qt];
          }
        }
      }
    }
    return;
  }
  if (!SHIFT) {
    // Rare: a row of this tile left the range in which unshifted weights are safe.  The whole
    // workgroup (its tiles are staged together) leaves the tile to the kernel with per-row shifts.
    bool bad = false;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) bad = bad || !(l_tot[qt] >= kFastSumMin && l_tot[qt] <= kFastSumMax);
    if (__syncthreads_or(active && bad)) {
      if (tid == 0) *mark = kRedoMark;
      return;
    }
  }

  // ---- normalise and store ---------------------------------------------------------------------
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const float inv = 1.0f / l_tot[qt];
    const int row = wq0 + qt * 32 + l32;
    if (row < Mq) {
      bf16_t* orow = o_rows + (q_base + row) * kDHead;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 ow;
          ow[0] = pack_bf16x2(w.o_acc[dt][qt][4 * g] * inv, w.o_acc[dt][qt][4 * g + 1] * inv);
          ow[1] = pack_bf16x2(w.o_acc[dt][qt][4 * g + 2] * inv, w.o_acc[dt][qt][4 * g + 3] * inv);
          *(u32x2*)(orow + dt * 32 + 8 * g + 4 * half) = ow;
        }
    }
  }
}

// SHIFT = false: the fast kernel (keys carry the logit scale; weights exp2(s)).  SHIFT = true: per-row
// shifts and the overflow guard; with a.marked_only it is launched right after the fast kernel on
// the same grid and a workgroup leaves at once unless the fast kernel marked its tile.
template <int QT, int NW, bool SHIFT>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, QT == 1 ? 3 : 2)))
void attention_kernel(const AttnArgs a) {
  constexpr int NT = 64 * NW;
  constexpr int BQ = 32 * QT * NW;
  constexpr int LD_ITER = kKvTile * kRowChunks / NT;       // 16-byte K chunks per thread per tile
  static_assert(LD_ITER >= 2 && LD_ITER % 2 == 0, "tile staging needs an even chunk count");
  constexpr int kTileElems = kKvTile * kDHead;
  __shared__ __align__(16) bf16_t s_k[2][kTileElems];    // [kv][d], 128-byte rows, chunk-swizzled
  __shared__ __align__(16) bf16_t s_v[2][kTileElems];    // [kv][d], 128-byte rows, chunk-swizzled

  // blockIdx -> work.  Workgroups go round-robin to the 8 XCDs, and in blockIdx order to free
  // slots.  Every XCD walks its whole tiles first - the partial last tiles of the heads (they are
  // short, so they should not be what the grid ends on), then a contiguous range of full tiles -
  // and then its shares of the tiles that run in segments; the device-side tile list comes last.
  const int block = (int)blockIdx.x;
  const int xcd = block & 7;
  int h = 0, q0 = 0, mq_dev = 0;
  int64_t q_base_dev = 0;
  int share = -1, first = 0, count = 1;           // share >= 0: `count` segments, in the tiles first, first + 1, ...
  const bool dev_tile = block >= a.main_blocks;
  const int pos = block >> 3, whole_per_xcd = a.full_per_xcd + a.ragged_per_xcd;
  if (dev_tile) {
    if (!a.dev_tiles) return;
    const int t = block - a.main_blocks;
    if (t >= a.dev_tiles[0]) return;
    h = a.dev_tiles[1 + 2 * t];
    q0 = a.dev_tiles[2 + 2 * t];
    q_base_dev = a.dev_q_off[h];
    mq_dev = a.dev_q_off[h + 1] - a.dev_q_off[h];
  } else if (pos >= whole_per_xcd) {
    const int item = pos - whole_per_xcd;
    share = xcd * a.split_per_xcd + item;
    if (item >= a.split_per_xcd || share >= a.sp.shares) return;
    split_share_tiles(a.sp, share, &first, &count);
  } else if (pos < a.ragged_per_xcd) {
    const int i = pos * 8 + xcd;
    if (i >= a.n_ragged) return;
    h = a.ragged_head[i];
    q0 = (a.tile_start[h + 1] - a.tile_start[h]) * BQ;
  } else {
    const int tile = xcd * a.full_per_xcd + (pos - a.ragged_per_xcd);
    if (tile >= a.n_full) return;
    while (tile >= a.tile_start[h + 1]) ++h;
    q0 = (tile - a.tile_start[h]) * BQ;
  }
  // a whole tile; or a share of the tiles that run in segments: its segments one after the other
  for (int i = 0; i < count; ++i) {
    SplitSegment seg = {0, 0, 0, 0, -1};
    if (share >= 0) {
      seg = split_segment(a.sp, share, first + i);
      h = seg.head;
      q0 = seg.q0;
      if (i) __syncthreads();                       // the tile buffers in LDS are free again
    }
    attention_tile<QT, NW, SHIFT>(a, s_k, s_v, h, q0, dev_tile, q_base_dev, mq_dev, seg);
  }
}

// The split tiles after a kernel ran them in segments: four workgroups per split tile (64 rows each)
// add its segments in ascending key order (run-to-run identical) and store the normalised rows.
// After the fast kernel every workgroup tests the row sums of the whole tile like that kernel does (a
// tile with a row outside the window gets the mark and is redone by the kernel with per-row
// shifts); after the kernel with per-row shifts every segment is first brought to the largest of
// the segments' shifts of its row.
constexpr int kReduceRows = 64;
template <int BQ, bool SHIFT>
__global__ __launch_bounds__(256) void attention_split_reduce_kernel(const AttnArgs a) {
  static_assert(BQ == 256, "one thread per row of the tile in the first phase");
  __shared__ float s_inv[BQ];
  __shared__ float s_max[SHIFT ? BQ : 1];      // the row's largest shift
  __shared__ __align__(16) uint32_t s_out[kReduceRows * 32];   // the normalised bf16 rows, for whole-line stores
  const int e = blockIdx.x >> 2, part = blockIdx.x & 3, tid = threadIdx.x;
  const SplitTile t = split_tile(a.sp, e);
  const int64_t q_base = a.q_off[t.head];
  const int left = (int)(a.q_off[t.head + 1] - q_base) - t.q0;
  const int rows = left < BQ ? left : BQ;
  const int np = t.last_share - t.first_share + 1;
  // consecutive shares of one tile have consecutive slots
  const int64_t row0 = (int64_t)split_slot(t.first_share, e) * BQ;     // segment p: rows from row0 + p * BQ
  // ---- the row sums of the whole tile (every workgroup of the tile, so that all four decide alike)
  bool bad = false;
  if (tid < rows) {
    float l = 0.f;
    if (SHIFT) {
      float m = -1e30f;
#pragma unroll 4
      for (int p = 0; p < np; ++p) m = fmaxf(m, a.split_m[row0 + (int64_t)p * BQ + tid]);
#pragma unroll 4
      for (int p = 0; p < np; ++p) {
        const float wgt = __builtin_amdgcn_exp2f(a.split_m[row0 + (int64_t)p * BQ + tid] - m);
        l = fmaf(a.split_l[row0 + (int64_t)p * BQ + tid], wgt, l);
      }
      s_max[tid] = m;
    } else {
#pragma unroll 4
      for (int p = 0; p < np; ++p) l += a.split_l[row0 + (int64_t)p * BQ + tid];
      bad = !(l >= kFastSumMin && l <= kFastSumMax);
    }
    s_inv[tid] = 1.0f / l;
  }
  if (__syncthreads_or(bad)) {
    if (tid == 0 && part == 0) *(uint16_t*)(a.o + (q_base + t.q0) * kDHead) = kRedoMark;
    return;
  }
  // ---- rows part * 64 .. + 63: thread -> row r = tid % 64 and the 16-byte output chunks c, c + 4
  const int r = part * kReduceRows + (tid & 63), c0 = tid >> 6;
  if (part * kReduceRows >= rows) return;
  const int rr = r < rows ? r : rows - 1;          // a row past the end reads a valid row and stores nothing
  float acc[2][8];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[i][q] = 0.f;
  const float m_row = SHIFT ? s_max[rr] : 0.f;
#pragma unroll 4
  for (int p = 0; p < np; ++p) {
    const float* ps = a.split_o + (row0 + (int64_t)p * BQ) * kDHead + rr * 4;
    f32x4 v[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) v[i][hf] = *(const f32x4*)(ps + ((c0 + 4 * i) * 2 + hf) * (BQ * 4));
    const float wgt = SHIFT ? __builtin_amdgcn_exp2f(a.split_m[row0 + (int64_t)p * BQ + rr] - m_row) : 1.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          acc[i][4 * hf + q] = SHIFT ? fmaf(v[i][hf][q], wgt, acc[i][4 * hf + q]) : acc[i][4 * hf + q] + v[i][hf][q];
  }
  const float inv = s_inv[rr];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    u32x4 o;
#pragma unroll
    for (int q = 0; q < 4; ++q) o[q] = pack_bf16x2(acc[i][2 * q] * inv, acc[i][2 * q + 1] * inv);
    *(u32x4*)&s_out[(tid & 63) * 32 + (c0 + 4 * i) * 4] = o;
  }
  __syncthreads();
  // whole 128-byte rows: 8 threads per row
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int lr = (tid >> 3) + 32 * i, ch = tid & 7;
    if (part * kReduceRows + lr < rows)
      ((u32x4*)a.o)[(q_base + t.q0 + part * kReduceRows + lr) * kRowChunks + ch] = *(const u32x4*)&s_out[lr * 32 + ch * 4];
  }
}

// compute units of the current device (asked once per device)
int64_t compute_units() {
  static int cached[64] = {0};
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cached[dev]) return cached[dev];
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
  cached[dev] = n;
  return n;
}

// 128-row tiles that run at once (three workgroups per CU): a problem with no more of them runs those
constexpr int64_t kSmallTileRound = 768;

// `extra_tiles` workgroups are appended for the device-side tile list (a.dev_tiles), if any.
// `scratch` (fp32 words, or nullptr): room for the tiles that run in segments (attention_split.hpp).
// a.marked_only != 0: the fast kernel, then the kernel with per-row shifts on the marked tiles.
template <int QT, int NW>
hipError_t launch_cfg(AttnArgs& a, const int64_t* q_off_host, const int64_t* k_off_host, int H,
                      hipStream_t stream, int extra_tiles = 0, float* scratch = nullptr, int64_t scratch_words = 0) {
  constexpr int BQ = 32 * QT * NW;
  int64_t full = 0;
  int ragged = 0;
  for (int h = 0; h < H; ++h) {
    const int64_t mq = q_off_host[h + 1] - q_off_host[h];
    a.tile_start[h] = (int32_t)full;
    a.q_off[h] = q_off_host[h];
    a.k_off[h] = k_off_host[h];
    full += mq / BQ;
    if (mq % BQ) a.ragged_head[ragged++] = h;
  }
  for (int h = H; h <= kAttnMaxHeads; ++h) {
    a.tile_start[h] = (int32_t)full;
    a.q_off[h] = q_off_host[H];
    a.k_off[h] = k_off_host[H];
  }
  for (int i = ragged; i < kAttnMaxHeads; ++i) a.ragged_head[i] = 0;
  a.n_full = (int32_t)full;
  a.n_ragged = ragged;
  a.full_per_xcd = (int32_t)((full + 7) / 8);
  a.ragged_per_xcd = (ragged + 7) / 8;
  if (full + ragged + extra_tiles == 0) return hipSuccess;
  a.main_blocks = 8 * (a.full_per_xcd + a.ragged_per_xcd);
  a.split_per_xcd = 0;
  a.split_o = nullptr;
  a.split_l = nullptr;
  a.split_m = nullptr;
  a.sp.n_tiles = 0;
  a.sp.slots = 0;
  const unsigned grid = (unsigned)a.main_blocks + (unsigned)extra_tiles;
  AttnArgs f = a;   // the first launch when tiles are split
  unsigned fgrid = grid;
  bool split = false;
  if (BQ == kAttnTileRows && scratch) {
    int64_t kept_full = full;
    int split_ragged = 0;
    plan_attention_split(q_off_host, k_off_host, H, compute_units(), &f.sp, &kept_full, &split_ragged);
    const int64_t slots = split_slots(f.sp);
    split = f.sp.n_tiles > 0 && slots * kAttnSlotWords <= scratch_words;
    if (split) {
      // the first partial tiles (in head order) and the last full tiles run in segments; the others
      // keep their order: partial tiles in front of the full tiles
      f.n_full = (int32_t)kept_full;
      f.full_per_xcd = (int32_t)((kept_full + 7) / 8);
      f.n_ragged = ragged - split_ragged;
      f.ragged_per_xcd = (f.n_ragged + 7) / 8;
      for (int i = 0; i < f.n_ragged; ++i) f.ragged_head[i] = a.ragged_head[split_ragged + i];
      f.split_per_xcd = (f.sp.shares + 7) / 8;
      f.main_blocks = 8 * (f.full_per_xcd + f.ragged_per_xcd + f.split_per_xcd);
      f.split_o = scratch;
      f.split_l = scratch + slots * kAttnTileRows * kDHead;
      f.split_m = f.split_l + slots * kAttnTileRows;
      fgrid = (unsigned)f.main_blocks + (unsigned)extra_tiles;
    } else {
      f.sp.n_tiles = 0;
      f.sp.slots = 0;
    }
  }
  if (a.marked_only) {
    // the fast kernel (and the sum of its segments), then the kernel with per-row shifts on the marked tiles
    hipLaunchKernelGGL((attention_kernel<QT, NW, false>), dim3(fgrid), dim3(64 * NW), 0, stream, f);
    if (split)
      hipLaunchKernelGGL((attention_split_reduce_kernel<kAttnTileRows, false>), dim3(4u * (unsigned)f.sp.n_tiles), dim3(256), 0, stream, f);
    hipLaunchKernelGGL((attention_kernel<QT, NW, true>), dim3(grid), dim3(64 * NW), 0, stream, a);
  } else {
    hipLaunchKernelGGL((attention_kernel<QT, NW, true>), dim3(fgrid), dim3(64 * NW), 0, stream, f);
    if (split)
      hipLaunchKernelGGL((attention_split_reduce_kernel<kAttnTileRows, true>), dim3(4u * (unsigned)f.sp.n_tiles), dim3(256), 0, stream, f);
  }
  return hipGetLastError();
}

}  // namespace

int64_t attention_scratch_need(const int64_t* q_off_host, const int64_t* k_off_host, int H) {
  SplitPlan sp;
  int64_t kept_full = 0;
  int split_ragged = 0;
  plan_attention_split(q_off_host, k_off_host, H, compute_units(), &sp, &kept_full, &split_ragged);
  return split_slots(sp) * kAttnSlotWords * 4;
}

hipError_t launch_attention_dev_tiles(const void* q, const void* k, const void* v, void* o,
                                      const int32_t* q_off_dev, const int32_t* tiles, int max_tiles,
                                      const int64_t* k_off_host, int H, float scale, bool log2_keys,
                                      hipStream_t stream) {
  static_assert(kAttnDevTileRows == 32 * 2 * 4, "the device tile list is cut for attention_kernel<2, 4>");
  if (max_tiles <= 0) return hipSuccess;
  AttnArgs a;
  std::memset(&a, 0, sizeof(a));
  a.q = (const bf16_t*)q;
  a.k = (const bf16_t*)k;
  a.v = (const bf16_t*)v;
  a.o = (bf16_t*)o;
  a.scale_log2 = log2_keys ? 1.0f : scale * 1.4426950408889634f;
  a.marked_only = log2_keys ? 1 : 0;
  a.H = H;
  for (int h = 0; h <= kAttnMaxHeads; ++h) a.k_off[h] = k_off_host[h < H ? h : H];
  a.dev_q_off = q_off_dev;
  a.dev_tiles = tiles;
  a.q2 = a.q;
  a.o2 = a.o;
  a.main_blocks = 0;        // no whole tiles, no segments: every workgroup takes the device-side list
  if (a.marked_only)
    hipLaunchKernelGGL((attention_kernel<2, 4, false>), dim3((unsigned)max_tiles), dim3(256), 0, stream, a);
  hipLaunchKernelGGL((attention_kernel<2, 4, true>), dim3((unsigned)max_tiles), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_attention_both(const void* q, const void* k, const void* v, void* o,
                                 const int64_t* q_off_host, const int64_t* k_off_host, int H, float scale,
                                 const void* q2, void* o2, const int32_t* q2_off_dev, const int32_t* tiles,
                                 int max_tiles, bool log2_keys, hipStream_t stream, void* scratch,
                                 int64_t scratch_bytes) {
  AttnArgs a;
  std::memset(&a, 0, sizeof(a));
  a.q = (const bf16_t*)q;
  a.k = (const bf16_t*)k;
  a.v = (const bf16_t*)v;
  a.o = (bf16_t*)o;
  a.scale_log2 = log2_keys ? 1.0f : scale * 1.4426950408889634f;
  a.marked_only = log2_keys ? 1 : 0;
  a.H = H;
  a.dev_q_off = q2_off_dev;
  a.dev_tiles = max_tiles > 0 ? tiles : nullptr;
  a.q2 = (const bf16_t*)q2;
  a.o2 = (bf16_t*)o2;
  return launch_cfg<2, 4>(a, q_off_host, k_off_host, H, stream, max_tiles > 0 ? max_tiles : 0, (float*)scratch,
                          scratch_bytes / 4);
}

hipError_t launch_attention(const void* q, const void* k, const void* v, void* o,
                            const int64_t* q_off_host, const int64_t* k_off_host, int H,
                            float scale, bool log2_keys, hipStream_t stream, void* scratch, int64_t scratch_bytes) {
  AttnArgs a;
  std::memset(&a, 0, sizeof(a));
  a.q = (const bf16_t*)q;
  a.k = (const bf16_t*)k;
  a.v = (const bf16_t*)v;
  a.o = (bf16_t*)o;
  a.scale_log2 = log2_keys ? 1.0f : scale * 1.4426950408889634f;
  a.marked_only = log2_keys ? 1 : 0;
  a.H = H;
  // Tiles of 256 query rows (two workgroups per CU) are the efficient shape, and with scratch memory
  // the tiles in excess of a multiple of the CU count run in segments, so that any tile count fills
  // the chip.  Without that split, a short problem that fits into one round of 128-row tiles (three
  // workgroups per CU, 768 at a time) runs those instead: they fill the chip where the big tiles
  // leave a third of it idle (measured: 0.132 against 0.144 ms at 16 x 5516 rows; with 800 small
  // tiles, a second round, 0.19 against 0.17 ms).
  int64_t tiles128 = 0;
  for (int h = 0; h < H; ++h) tiles128 += (q_off_host[h + 1] - q_off_host[h] + 127) / 128;
  if (tiles128 <= kSmallTileRound) {
    const bool splits = scratch && attention_scratch_need(q_off_host, k_off_host, H) > 0 &&
                        attention_scratch_need(q_off_host, k_off_host, H) <= scratch_bytes;
    if (!splits) return launch_cfg<1, 4>(a, q_off_host, k_off_host, H, stream);
  }
  return launch_cfg<2, 4>(a, q_off_host, k_off_host, H, stream, 0, (float*)scratch, scratch_bytes / 4);
}

// ---- scratch that belongs to the library -------------------------------------------------------
// For callers that cannot allocate device memory (code under HIP graph capture, serving loops, test
// harnesses that forbid it): the room for the partial results of the tiles that run in pieces, as a
// device array of fixed size.  Every GPU the library runs on holds its own copy at its own address
// until the process ends; the array's name is only a host-side handle, the address comes from
// hipGetSymbolAddress, once per device, and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char g_static_scratch[kAttnStaticScratchBytes];

hipError_t attention_static_scratch(void** ptr) {
  static std::mutex mu;
  static void* per_device[64] = {nullptr};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!per_device[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    per_device[dev] = p;
  }
  *ptr = per_device[dev];
  return hipSuccess;
}

}  // namespace httm
