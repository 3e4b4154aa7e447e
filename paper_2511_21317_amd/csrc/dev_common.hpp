// Device-side helpers shared by the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace httm {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kDHead = 64;            // channels per head
constexpr int kRowBytes = kDHead * 2; // one bf16 token row
constexpr int kRowChunks = 8;         // 16-byte chunks per row

// A token row in LDS is padded from 128 to 144 bytes: consecutive rows then start 9 sixteen-byte
// granules apart, so the 16-byte MFMA operand reads of 8 (or 16) consecutive rows fall into
// distinct bank groups.
constexpr int kLdsRowBytes = 144;
constexpr int kLdsRowElems = kLdsRowBytes / 2;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
  return __uint_as_float(bits16 << 16);
}
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
  bf16_t r = (bf16_t)x;
  return __builtin_bit_cast(uint16_t, r);
}

// Block-local position of the dst token of cluster m (Sec. 3.2 dst/src partition inside a block of
// n tokens that keeps k clusters): the n0 anchored tokens at the front of the block first (App. C.2),
// the other k - n0 evenly strided over the remaining n - n0 tokens, the first of them included.
// n0 = 0 gives floor(m * n / k).
// (32-bit product: for blocks of at most 32768 tokens, which is every merging block.)
__device__ __forceinline__ int dst_position(int m, int n, int k, int n0) {
  return m < n0 ? m : n0 + ((m - n0) * (n - n0)) / (k - n0);
}
// The same for a "block" of any size below 2^31 tokens (un-blocked matching of a whole sequence):
// (m - n0) * (n - n0) passes 2^31 from n = 46341 on, so the product is taken in 64 bits there.
__device__ __forceinline__ int dst_position_any(int m, int n, int k, int n0) {
  if (n <= 32768) return dst_position(m, n, k, n0);
  return m < n0 ? m : n0 + (int)(((int64_t)(m - n0) * (int64_t)(n - n0)) / (int64_t)(k - n0));
}

// Cluster whose dst token sits at block position p, or -1 if p is a src position (inverse of
// dst_position_any; k = number of dst tokens).
__device__ __forceinline__ int cluster_at(int p, int n, int k, int n0) {
  if (p < n0) return p;
  if (k == n0) return -1;
  // 64-bit: (p - n0) * (k - n0) passes 2^31 for sequences of more than ~46 000 tokens
  const int m = n0 + (int)(((int64_t)(p - n0) * (int64_t)(k - n0) + (n - n0) - 1) / (int64_t)(n - n0));
  return (m < k && dst_position_any(m, n, k, n0) == p) ? m : -1;
}

// The same two maps for a merging block (at most 4096 tokens: every product below stays under 2^25
// and every quotient under 2^13) without an integer division per call.  The quotient comes from a
// float reciprocal (relative error below 2^-21, so it is off by at most one) and is put right with
// the exact integer remainder.
__device__ __forceinline__ int div_block(int num, int den, float rcp_den) {
  int q = (int)((float)num * rcp_den);
  const int r = num - q * den;
  q = r < 0 ? q - 1 : q;
  q = r >= den ? q + 1 : q;
  return q;
}
struct BlockMap {
  int n, k, n0;
  float rcp_k, rcp_n;   // 1 / (k - n0) and 1 / (n - n0); unused (and infinite) where those are 0
  __device__ __forceinline__ BlockMap(int n_, int k_, int n0_)
      : n(n_), k(k_), n0(n0_), rcp_k(__builtin_amdgcn_rcpf((float)(k_ - n0_))),
        rcp_n(__builtin_amdgcn_rcpf((float)(n_ - n0_))) {}
  __device__ __forceinline__ int dst_position(int m) const {
    const int p = n0 + div_block((m - n0) * (n - n0), k - n0, rcp_k);
    return m < n0 || k == n0 ? m : p;
  }
  // dst tokens at positions below p (0 <= p <= n): floor(j * A / B) < x  <=>  j < ceil(x * B / A)
  __device__ __forceinline__ int dst_before(int p) const {
    const int m = n0 + div_block((p - n0) * (k - n0) + (n - n0) - 1, n - n0, rcp_n);
    return p <= n0 ? p : (k == n0 ? n0 : m);
  }
  __device__ __forceinline__ int cluster_at(int p) const {
    if (p < n0) return p;
    if (k == n0) return -1;
    const int m = dst_before(p);
    return (m < k && dst_position(m) == p) ? m : -1;
  }
  // Position of the s-th src token (0 <= s < n - k, ascending position): the smallest p with s + 1
  // src tokens at positions <= p.  The count grows by at most one per position, so that p is a src
  // position; 12 halvings cover 4096 positions.
  __device__ __forceinline__ int src_position(int s) const {
    int lo = 0, hi = n - 1;
#pragma unroll 1
    for (int i = 0; i < 12; ++i) {
      const int mid = (lo + hi) >> 1;
      const bool enough = mid + 1 - dst_before(mid + 1) >= s + 1;
      hi = enough ? mid : hi;
      lo = enough ? lo : mid + 1;
    }
    return lo;
  }
};

// last word of a raw buffer descriptor on gfx9-family targets (32-bit data format, no swizzle, no
// stride), and the cache-policy bit of a buffer load that marks it non-temporal
constexpr int kRawBufferWord3 = 0x00020000;
constexpr int kBufferNonTemporal = 2;

}  // namespace httm
