// Two measurement kernels: what this device reaches on the two roofs the merged operators are priced
// against, measured with the same launch path and timing hook as the operators themselves.
//   probe_mfma_kernel:     the issue rate of the bf16 matrix instruction the contractions use, from registers only
//                          (four independent 32 x 32 accumulators per wavefront, nothing else in the loop);
//   probe_hbm_read_kernel: a read-only stream over a buffer (16 bytes per lane and load, non-temporal, several
//                          loads in flight per lane), the access shape of a weight stream.
#pragma once
#include "nf_common.h"

namespace nf {

constexpr int kProbeWaves = 16;                               // wavefronts per workgroup of the matrix probe (4 per SIMD)
constexpr double kProbeFlopsPerMfma = 2.0 * 32 * 32 * 16;

__global__ __launch_bounds__(kProbeWaves * kWave) void probe_mfma_kernel(float* sink, int iters, int never) {
  typedef __attribute__((ext_vector_type(8))) __bf16 v8bf;
  typedef __attribute__((ext_vector_type(16))) float v16f;
  v8bf a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(1.0f + (float)(threadIdx.x % 7));
    b[e] = (__bf16)(0.5f + (float)e);
  }
  v16f acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (never) sink[0] = s;                                     // the host passes 0: keeps the loop alive, writes nothing
}

constexpr int kProbeReadUnroll = 8;

// chunks = number of 16-byte pieces; workgroup b reads pieces b * 256 * U ... in steps of the whole grid
__global__ __launch_bounds__(256) void probe_hbm_read_kernel(const uint4* __restrict__ src, size_t chunks, uint32_t* sink, int never) {
  constexpr int U = kProbeReadUnroll;
  const size_t per_round = (size_t)gridDim.x * 256 * U;
  uint32_t x = 0;
  for (size_t base = (size_t)blockIdx.x * 256 * U + threadIdx.x; base < chunks; base += per_round) {
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t c = base + (size_t)u * 256;
      v[u] = c < chunks ? ldnt16(src + c) : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) x ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (never) sink[0] = x;                                     // the host passes 0
}

}  // namespace nf
