// Instantiation of the fragment-packed weight-streaming matmul kernels (gemm_frag.h) and of the packer.
#include <atomic>

#include "gemm_frag.h"
#include "gemm_launch.h"
#include "pack_kernels.h"

#ifndef NF_FRAG_NS
#define NF_FRAG_NS 4
#endif

namespace nf {

template <class Cfg>
__global__ __launch_bounds__(Cfg::kThreads) void gemm_frag_kernel(GemmArgs a) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  lds_u8_t* smem = (lds_u8_t*)smem_raw;
  unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  // consecutive ids: row tiles of one column tile, then the next column tile, then the next problem
  const int tm = id % a.tiles_m;  id /= a.tiles_m;
  const int tn = id % a.tiles_n;  id /= a.tiles_n;
  const int z0 = id % a.nz0;
  const int z1 = id / a.nz0;
  const int row0 = tm * Cfg::kBM, col0 = tn * Cfg::kBN;
  const long coff = z0 * a.sC0 + z1 * a.sC1 + (long)row0 * a.ldc + col0;
  const bf16_t* A = a.A + z0 * a.sA0 + z1 * a.sA1 + (long)row0 * a.lda;
  const float* bias = a.ep.col_bias ? a.ep.col_bias + z0 * a.ep.col_vec_stride0 + z1 * a.ep.col_vec_stride1 + col0 : nullptr;
  const bf16_t* Bw = a.B + z0 * a.sB0 + z1 * a.sB1 + (long)(col0 / 32) * a.K * 32;   // column block col0/32: K/16 fragments of 512 elements
  gemm_frag_tile<Cfg>(A, a.lda, Bw, a.K, smem, a.C + coff, a.R ? a.R + coff : nullptr, a.ldc, bias, a.ep.act, tn,
                      a.touch_a ? a.tiles_n : 0);
}

template <class Cfg>
static nf_status launch_frag(GemmLaunch& L, hipStream_t s) {
  GemmArgs& a = L.a;
  if (a.rows % Cfg::kBM || a.cols % Cfg::kBN || a.K % (Cfg::kBK * Cfg::kNS) || a.K / Cfg::kBK < Cfg::kNS) return NF_EUNSUPPORTED;
  a.tiles_m = a.rows / Cfg::kBM;
  a.tiles_n = a.cols / Cfg::kBN;
  // 16-byte moves everywhere: A rows, packed fragments, output, residual, column constants
  if (a.lda % 8 || a.ldc % 8 || ((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15) || ((uintptr_t)a.C & 15) ||
      ((uintptr_t)a.R & 15) || ((uintptr_t)a.ep.col_bias & 15) || a.ep.col_vec_stride0 % 4 || a.ep.col_vec_stride1 % 4 ||
      a.sA0 % 8 || a.sA1 % 8 || a.sB0 % 8 || a.sB1 % 8 || a.sC0 % 8 || a.sC1 % 8)
    return NF_EUNSUPPORTED;
  if (!a.ep.act_before_residual && a.ep.act != NF_ACT_NONE && a.R) return NF_EUNSUPPORTED;
  if (a.ep.row_bias || a.ep.row_scale) return NF_EUNSUPPORTED;
  const long long total = (long long)a.tiles_m * a.tiles_n * a.nz0 * L.nz1;
  if (total <= 0 || total > 0x7fffffffLL) return NF_EUNSUPPORTED;
  a.touch_a = touch_a_pays(total, (long long)a.rows * a.K, (long long)a.nz0 * L.nz1);
  auto kern = gemm_frag_kernel<Cfg>;
  constexpr int kLds = Cfg::kLdsBytes;
  if (kLds > 64 * 1024) {
    static std::atomic<bool> opted_in{false};
    if (!opted_in.load(std::memory_order_acquire)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLds) !=
          hipSuccess)
        return NF_ELAUNCH;
      opted_in.store(true, std::memory_order_release);
    }
  }
  nf_launch(kern, dim3((unsigned)total), dim3(Cfg::kThreads), kLds, s, a);
  return hipGetLastError() == hipSuccess ? NF_OK : NF_ELAUNCH;
}

nf_status launch_gemm_frag(int cfg, GemmLaunch& L, hipStream_t s) {
  switch (cfg) {
    case F96: return launch_frag<FragCfg<3, 4, 1, NF_FRAG_NS>>(L, s);
    case F288: return launch_frag<FragCfg<9, 1, 2, NF_FRAG_NS>>(L, s);
    case F384: return launch_frag<FragCfg<12, 1, 2, NF_FRAG_NS>>(L, s);
    case F128: return launch_frag<FragCfg<4, 1, 2, NF_FRAG_NS>>(L, s);
    case F256: return launch_frag<FragCfg<8, 1, 2, NF_FRAG_NS>>(L, s);
    case F96h: return launch_frag<FragCfg<3, 2, 2, NF_FRAG_NS, 2>>(L, s);
    case F288h: return launch_frag<FragCfg<9, 1, 2, NF_FRAG_NS, 2>>(L, s);
    case F384h: return launch_frag<FragCfg<12, 1, 2, NF_FRAG_NS, 2>>(L, s);
  }
  return NF_EUNSUPPORTED;
}

nf_status launch_pack_fragments(const bf16_t* W, bf16_t* Wp, long long problems, int K, int Nout, hipStream_t s) {
  const long long chunks = problems * K * Nout / 8, blocks = (chunks + 255) / 256;
  if (blocks > 0x7fffffffLL) return NF_EUNSUPPORTED;
  nf_launch(pack_fragments_kernel, dim3((unsigned)blocks), dim3(256), 0, s, W, Wp, K, Nout, (size_t)chunks);
  return hipGetLastError() == hipSuccess ? NF_OK : NF_ELAUNCH;
}

}  // namespace nf
