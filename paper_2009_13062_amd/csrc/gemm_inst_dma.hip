// Instantiation of the direct-to-LDS pipelined bf16 MFMA contraction kernels (whole-tile problems).
#include <atomic>

#include "gemm_dma.h"
#include "gemm_launch.h"

#ifndef NF_NS_288
#define NF_NS_288 4
#endif
#ifndef NF_NS_96
#define NF_NS_96 4
#endif
#ifndef NF_NS_384
#define NF_NS_384 4
#endif

namespace nf {

template <class Cfg>
__global__ __launch_bounds__(Cfg::kThreads) void gemm_dma_kernel(GemmArgs a) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  lds_u8_t* smem = (lds_u8_t*)smem_raw;
  unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  // consecutive ids: row tiles of one column panel, then the next panel, then the next problem
  const int tm = id % a.tiles_m;  id /= a.tiles_m;
  const int tn = id % a.tiles_n;  id /= a.tiles_n;
  const int z0 = id % a.nz0;
  const int z1 = id / a.nz0;
  const int row0 = tm * Cfg::kBM, col0 = tn * Cfg::kBN;
  const long coff = z0 * a.sC0 + z1 * a.sC1 + (long)row0 * a.ldc + col0;
  const bf16_t* A = a.A + z0 * a.sA0 + z1 * a.sA1 + (long)row0 * a.lda;
  const bf16_t* B = a.B + z0 * a.sB0 + z1 * a.sB1 + col0;
  const long rvo = z0 * a.ep.row_vec_stride0 + z1 * a.ep.row_vec_stride1 + row0;
  const long cvo = z0 * a.ep.col_vec_stride0 + z1 * a.ep.col_vec_stride1 + col0;
  gemm_dma_tile<Cfg>(A, a.lda, B, a.ldb, a.K, smem, a.C + coff, a.R ? a.R + coff : nullptr, a.ldc, a.ep, rvo, cvo,
                     tn, a.touch_a ? a.tiles_n : 0);
}

template <class Cfg>
nf_status launch_dma(GemmLaunch& L, hipStream_t s) {
  GemmArgs& a = L.a;
  if (a.rows % Cfg::kBM || a.cols % Cfg::kBN || a.K % Cfg::kBK) return NF_EUNSUPPORTED;
  a.tiles_m = a.rows / Cfg::kBM;
  a.tiles_n = a.cols / Cfg::kBN;
  const long long total = (long long)a.tiles_m * a.tiles_n * a.nz0 * L.nz1;
  if (total <= 0 || total > 0x7fffffffLL) return NF_EUNSUPPORTED;
  a.touch_a = touch_a_pays(total, (long long)a.rows * a.K, (long long)a.nz0 * L.nz1);
  auto kern = gemm_dma_kernel<Cfg>;
  if (Cfg::kLdsBytes > 64 * 1024) {
    static std::atomic<bool> opted_in{false};
    if (!opted_in.load(std::memory_order_acquire)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              Cfg::kLdsBytes) != hipSuccess)
        return NF_ELAUNCH;
      opted_in.store(true, std::memory_order_release);
    }
  }
  nf_launch(kern, dim3((unsigned)total), dim3(Cfg::kThreads), Cfg::kLdsBytes, s, a);
  return hipGetLastError() == hipSuccess ? NF_OK : NF_ELAUNCH;
}

nf_status launch_gemm_dma(int cfg, GemmLaunch& L, hipStream_t s) {
  switch (cfg) {
    case D256x256k32s4: return launch_dma<DmaCfg<256, 256, 32, 2, 4, 4>>(L, s);
    case D128x128k32s4: return launch_dma<DmaCfg<128, 128, 32, 2, 4, 4>>(L, s);
    case D128x128k64s3w8: return launch_dma<DmaCfg<128, 128, 64, 2, 4, 3>>(L, s);
    case D128x384k32s4w12: return launch_dma<DmaCfg<128, 384, 32, 2, 6, NF_NS_384>>(L, s);
    case D128x288k32s4w12: return launch_dma<DmaCfg<128, 288, 32, 4, 3, NF_NS_288>>(L, s);
    case D128x96k64s4w12: return launch_dma<DmaCfg<128, 96, 64, 4, 3, NF_NS_96>>(L, s);
  }
  return NF_EUNSUPPORTED;
}

}  // namespace nf
