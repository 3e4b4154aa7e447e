// Measurement helper of bench.py, not part of the HTTM path and not part of libhttm.so: what this
// chip sustains on v_mfma_f32_32x32x16_bf16 alone.  Every wave runs four independent chains of that
// instruction on registers (seeded pseudo-random bf16 operands in [-1, 1], no memory access in the
// loop), one or two workgroups of four waves per compute unit.  The published 2.5 PFLOP/s assumes
// 2.4 GHz; under this loop the clock settles where the power limit puts it, and the rate it reaches
// is the practical ceiling for a kernel built on this instruction (the attention kernel, Sec. 3.2
// Eq. 3-4 of the paper).  bench.py reports it next to the roofline fraction, which stays a fraction
// of the published peak.
#include <hip/hip_runtime.h>
#include <cstdint>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int kChains = 4;

__global__ __launch_bounds__(256) void mfma_probe_kernel(float* __restrict__ out, int rounds) {
  bf16x8 a[kChains], b[kChains];
  uint32_t h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  for (int k = 0; k < kChains; ++k)
    for (int i = 0; i < 8; ++i) {
      h = h * 1664525u + 1013904223u;
      a[k][i] = (__bf16)(((int)((h >> 8) % 2001u) - 1000) * 0.001f);
      h = h * 1664525u + 1013904223u;
      b[k][i] = (__bf16)(((int)((h >> 8) % 2001u) - 1000) * 0.001f);
    }
  f32x16 acc[kChains];
  for (int c = 0; c < kChains; ++c)
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int it = 0; it < rounds; ++it) {   // 16 instructions per round
#pragma unroll
    for (int u = 0; u < kChains; ++u)
#pragma unroll
      for (int c = 0; c < kChains; ++c)
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c], b[(c + u) % kChains], acc[c], 0, 0, 0);
  }
  float s = 0.f;
  for (int c = 0; c < kChains; ++c)
    for (int r = 0; r < 16; ++r) s += acc[c][r];
  if (s == 123.456f) out[0] = s;   // keeps the loop alive; never true in practice
}

}  // namespace

// Launches the loop on `stream`: 256 * wgs_per_cu workgroups, `rounds` rounds of 16 MFMA instructions
// per wave.  `out`: 4 bytes of device memory.  Returns the flop it executes (0 on a bad argument or a
// launch error): grid * 4 waves * rounds * 16 instructions * 32768.
extern "C" __attribute__((visibility("default"))) double httm_probe_mfma_bf16(float* out, int rounds, int wgs_per_cu,
                                                                              void* stream) {
  if (!out || rounds <= 0 || wgs_per_cu <= 0 || wgs_per_cu > 8) return 0.0;
  const int grid = 256 * wgs_per_cu;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, out, rounds);
  if (hipGetLastError() != hipSuccess) return 0.0;
  return (double)grid * 4.0 * rounds * 16.0 * 32768.0;
}
