// Stage 3: attention over the reduced per-head sequences (paper Sec. 3.2 Eq. 3-4):
//   O = softmax(Q K^T * scale) V, per head, no mask, ragged (M_q[h], M_k[h]).
//
// Flash-style single pass with bf16 MFMA (v_mfma_f32_32x32x16_bf16) and fp32 online softmax.
// The kernel is bound by the matrix cores (4*M_q*M_k*64 flop per head against a few MB of
// K/V that stay in L2 / Infinity Cache).
//
// Work decomposition
//   * workgroup = 4 waves = one tile of BQ = 128*QT query rows of one head; wave w owns 32*QT rows;
//   * K/V are streamed in tiles of 64 rows through LDS, double buffered: the global loads of
//     tile i+1 are issued before the MFMAs of tile i and written to the other buffer after them,
//     one barrier per tile;
//   * blockIdx -> tile mapping is XCD-aware: workgroups are dispatched round-robin over the 8
//     XCDs, so tile = (bid % 8) * (grid/8) + bid / 8 gives every XCD a contiguous range of
//     tiles, i.e. about two heads, whose K/V then stay in that XCD's L2.
//
// Transposed formulation.  Each wave computes S^T = K Q^T (A = K tile from LDS, B = Q^T from
// registers) so that in the 32x32 accumulator layout a lane owns ONE query column and 16 of the
// 32 key rows: the row-max / row-sum of the softmax are reductions inside a lane plus one
// exchange with lane^32, and the rescaling factor of the online softmax is a per-lane scalar
// for the O^T = V^T P^T accumulators as well.  P^T goes from the accumulator registers straight
// into the B operand of the second MFMA (fp32 -> bf16 in registers, no LDS round trip).  That
// fixes which 8 keys a lane supplies per MFMA step: {16j + 4*half + 0..3, 16j + 8 + 4*half + 0..3};
// V is therefore stored transposed in LDS with key positions 2 and 3 bit-swapped, so that the
// matching A operand (V^T rows = channels) is one aligned 16-byte read.
#include "dev_common.hpp"
#include "kernels.hpp"

namespace httm {

namespace {

constexpr int kKvTile = 64;
constexpr int kAttnThreads = 256;

struct AttnArgs {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  bf16_t* o;
  float scale_log2;  // scale * log2(e)
  int32_t H;
  int32_t total_tiles;
  int32_t tile_start[kAttnMaxHeads + 1];
  int64_t q_off[kAttnMaxHeads + 1];
  int64_t k_off[kAttnMaxHeads + 1];
};

// position of key row `kv` (0..63) inside a transposed V row in LDS: bits 2 and 3 swapped
__device__ __forceinline__ int vt_pos(int kv) {
  return (kv & ~0xC) | ((kv & 4) << 1) | ((kv & 8) >> 1);
}

template <int QT>
__global__ __launch_bounds__(kAttnThreads) void attention_kernel(const AttnArgs a) {
  constexpr int BQ = 128 * QT;
  __shared__ __align__(16) bf16_t s_k[2][kKvTile * kLdsRowElems];   // [kv][d], 144-byte rows
  __shared__ __align__(16) bf16_t s_vt[2][kDHead * kLdsRowElems];   // [d][kv position]

  const int per_xcd = gridDim.x >> 3;
  const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (tile >= a.total_tiles) return;
  int h = 0;
  while (tile >= a.tile_start[h + 1]) ++h;
  const int64_t q_base = a.q_off[h], k_base = a.k_off[h];
  const int Mq = (int)(a.q_off[h + 1] - q_base);
  const int Mk = (int)(a.k_off[h + 1] - k_base);
  const int q0 = (tile - a.tile_start[h]) * BQ;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int wq0 = q0 + wave * 32 * QT;  // first query row of this wave

  if (Mk == 0) {
    // softmax over an empty key set: defined as zero output
    for (int e = tid; e < BQ * kRowChunks; e += kAttnThreads) {
      const int row = q0 + (e >> 3);
      if (row < Mq) ((u32x4*)a.o)[(q_base + row) * kRowChunks + (e & 7)] = u32x4{0, 0, 0, 0};
    }
    return;
  }

  // ---- Q^T fragments (B operand): lane -> query column, 8 consecutive channels ---------------
  bf16x8 qf[QT][4];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    int row = wq0 + qt * 32 + l32;
    row = row < Mq ? row : Mq - 1;
    const bf16_t* p = a.q + (q_base + row) * kDHead + half * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[qt][ks] = *(const bf16x8*)(p + ks * 16);
  }

  // ---- accumulators ---------------------------------------------------------------------------
  f32x16 o_acc[2][QT];
  float m_run[QT], l_run[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[dt][qt][r] = 0.f;
  }

  // ---- K/V tile staging -----------------------------------------------------------------------
  const u32x4* kg = (const u32x4*)(a.k + k_base * kDHead);
  const u32x4* vg = (const u32x4*)(a.v + k_base * kDHead);
  const int ld_c = tid & 7, ld_r = tid >> 3;  // chunk, row-in-pass (0..31)
  u32x4 kreg[2], vreg[2];
  auto load_tile = [&](int kv0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int row = kv0 + ld_r + 32 * i;
      row = row < Mk ? row : Mk - 1;
      kreg[i] = kg[(int64_t)row * kRowChunks + ld_c];
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      int row = kv0 + 2 * ld_r + i;
      row = row < Mk ? row : Mk - 1;
      vreg[i] = vg[(int64_t)row * kRowChunks + ld_c];
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
      *(u32x4*)(&s_k[buf][(ld_r + 32 * i) * kLdsRowElems + ld_c * 8]) = kreg[i];
    // V rows 2*ld_r and 2*ld_r+1, channels ld_c*8 .. +7  ->  V^T[channel][pos], two keys per word
    const int pos = vt_pos(2 * ld_r);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t w0 = vreg[0][e], w1 = vreg[1][e];
      const uint32_t lo = (w0 & 0xffffu) | (w1 << 16);          // channel 2e   of both keys
      const uint32_t hi = (w0 >> 16) | (w1 & 0xffff0000u);      // channel 2e+1 of both keys
      *(uint32_t*)(&s_vt[buf][(ld_c * 8 + 2 * e) * kLdsRowElems + pos]) = lo;
      *(uint32_t*)(&s_vt[buf][(ld_c * 8 + 2 * e + 1) * kLdsRowElems + pos]) = hi;
    }
  };

  const int n_tiles = (Mk + kKvTile - 1) / kKvTile;
  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int it = 0; it < n_tiles; ++it) {
    const int buf = it & 1;
    const int kv0 = it * kKvTile;
    if (it + 1 < n_tiles) load_tile(kv0 + kKvTile);

    // ---- S^T = K Q^T --------------------------------------------------------------------------
    f32x16 s_acc[2][QT];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[kt][qt][r] = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 ak =
            *(const bf16x8*)(&s_k[buf][(kt * 32 + l32) * kLdsRowElems + ks * 16 + half * 8]);
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          s_acc[kt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qf[qt][ks], s_acc[kt][qt], 0, 0, 0);
      }

    // ---- mask the ragged tail of the last tile ----------------------------------------------
    if (kv0 + kKvTile > Mk) {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kv0 + kt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
          if (kv >= Mk) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) s_acc[kt][qt][r] = -INFINITY;
          }
        }
    }

    // ---- online softmax (per lane = per query column) ------------------------------------------
    bf16x8 pf[2][2][QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
      float mx = s_acc[0][qt][0];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_acc[kt][qt][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[qt], mx * a.scale_log2);
      const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_new);
      m_run[qt] = m_new;
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          p[r] = __builtin_amdgcn_exp2f(fmaf(s_acc[kt][qt][r], a.scale_log2, -m_new));
          psum += p[r];
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          u32x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(p[8 * j + 2 * e], p[8 * j + 2 * e + 1]);
          pf[kt][j][qt] = __builtin_bit_cast(bf16x8, w);
        }
      }
      l_run[qt] = l_run[qt] * alpha + psum;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[dt][qt][r] *= alpha;
    }

    // ---- O^T += V^T P^T -------------------------------------------------------------------------
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const bf16x8 av = *(const bf16x8*)(
              &s_vt[buf][(dt * 32 + l32) * kLdsRowElems + kt * 32 + j * 16 + half * 8]);
#pragma unroll
          for (int qt = 0; qt < QT; ++qt)
            o_acc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, pf[kt][j][qt], o_acc[dt][qt], 0, 0, 0);
        }

    if (it + 1 < n_tiles) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- normalise and store ---------------------------------------------------------------------
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const float l_tot = l_run[qt] + __shfl_xor(l_run[qt], 32);
    const float inv = 1.0f / l_tot;
    const int row = wq0 + qt * 32 + l32;
    if (row < Mq) {
      bf16_t* orow = a.o + (q_base + row) * kDHead;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w;
          w[0] = pack_bf16x2(o_acc[dt][qt][4 * g] * inv, o_acc[dt][qt][4 * g + 1] * inv);
          w[1] = pack_bf16x2(o_acc[dt][qt][4 * g + 2] * inv, o_acc[dt][qt][4 * g + 3] * inv);
          *(u32x2*)(orow + dt * 32 + 8 * g + 4 * half) = w;
        }
    }
  }
}

}  // namespace

hipError_t launch_attention(const void* q, const void* k, const void* v, void* o,
                            const int64_t* q_off_host, const int64_t* k_off_host, int H,
                            float scale, hipStream_t stream) {
  constexpr int QT = 1;
  constexpr int BQ = 128 * QT;
  AttnArgs a;
  a.q = (const bf16_t*)q;
  a.k = (const bf16_t*)k;
  a.v = (const bf16_t*)v;
  a.o = (bf16_t*)o;
  a.scale_log2 = scale * 1.4426950408889634f;
  a.H = H;
  int64_t tiles = 0;
  for (int h = 0; h < H; ++h) {
    a.tile_start[h] = (int32_t)tiles;
    a.q_off[h] = q_off_host[h];
    a.k_off[h] = k_off_host[h];
    tiles += (q_off_host[h + 1] - q_off_host[h] + BQ - 1) / BQ;
  }
  for (int h = H; h <= kAttnMaxHeads; ++h) {
    a.tile_start[h] = (int32_t)tiles;
    a.q_off[h] = q_off_host[H];
    a.k_off[h] = k_off_host[H];
  }
  a.total_tiles = (int32_t)tiles;
  if (tiles == 0) return hipSuccess;
  const unsigned grid = (unsigned)((tiles + 7) / 8 * 8);
  hipLaunchKernelGGL((attention_kernel<QT>), dim3(grid), dim3(kAttnThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace httm
