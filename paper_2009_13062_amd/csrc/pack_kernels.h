// Offline re-layout of the merged matmul's weights (they are static at inference and are almost all of the
// bytes a forward pass moves): W[z][K][Nout] row-major  ->  MFMA operand fragments,
//   Wp[z][j][s][lane][e] = W[z][16 s + 8 (lane / 32) + e][32 j + lane % 32]     j < Nout/32, s < K/16, e < 8,
// so that the 64 lanes of a wavefront fetch the operand of one 32x32x16 multiplication (column block j, 16-k
// slice s) as one contiguous kilobyte, and the fragments a wavefront needs in turn follow one another.
#pragma once
#include "nf_common.h"

namespace nf {

// one thread = one lane's 16 bytes of one fragment; the 32 lanes of a half read 64 contiguous bytes per e
__global__ __launch_bounds__(256) void pack_fragments_kernel(const bf16_t* __restrict__ W, bf16_t* __restrict__ Wp,
                                                             int K, int Nout, size_t chunks) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= chunks) return;
  const int ks = K / 16, nb = Nout / 32;
  size_t r = c;
  const int lane = r % 64; r /= 64;
  const int s = r % ks;    r /= ks;
  const int j = r % nb;
  const size_t z = r / nb;
  const bf16_t* src = W + (z * K + (size_t)16 * s + 8 * (lane / 32)) * Nout + (size_t)32 * j + lane % 32;
  uint32_t o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
    o[e] = (uint32_t)src[(size_t)(2 * e) * Nout] | ((uint32_t)src[(size_t)(2 * e + 1) * Nout] << 16);
  *reinterpret_cast<uint4*>(Wp + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
}

}  // namespace nf
