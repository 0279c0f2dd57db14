// Offline re-layout of the merged matmul's weights (they are static at inference and are almost all of the
// bytes a forward pass moves): W[z][K][Nout] row-major  ->  blocks of [32 k][32 n] elements (2 KB of bf16),
// ordered [z][panel][k-block][block within panel].  A GEMM tile whose width divides the panel width then
// reads, per k-step, ONE contiguous run of BN * 64 bytes instead of 32 row pieces of BN * 2 bytes, and the
// block is already the LDS image the transposing fragment read wants.
#pragma once
#include "nf_common.h"

namespace nf {

// one thread = one 16-byte chunk (8 consecutive n) of the packed tensor
__global__ __launch_bounds__(256) void pack_weight_kernel(const bf16_t* __restrict__ W, bf16_t* __restrict__ Wp,
                                                          int K, int Nout, int panel, size_t chunks) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= chunks) return;
  const int pb = panel / 32, kbs = K / 32;
  size_t r = c;
  const int c8 = r % 4;  r /= 4;          // chunk within the 64-byte row of a block
  const int kr = r % 32; r /= 32;         // k row within the block
  const int j = r % pb;  r /= pb;         // block within the panel
  const int kb = r % kbs; r /= kbs;       // k-block
  const int p = r % (Nout / panel);       // panel
  const size_t z = r / (Nout / panel);
  const size_t src = (z * K + (size_t)kb * 32 + kr) * Nout + (size_t)(p * pb + j) * 32 + c8 * 8;
  *reinterpret_cast<uint4*>(Wp + c * 8) = *reinterpret_cast<const uint4*>(W + src);
}

}  // namespace nf
