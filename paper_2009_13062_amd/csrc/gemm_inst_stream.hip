// Instantiation of the streaming (several column tiles per workgroup, register epilogue) bf16 MFMA matmul kernels.
#include <atomic>

#include "gemm_launch.h"
#include "gemm_stream.h"

#ifndef NF_NS_S384
#define NF_NS_S384 4
#endif

namespace nf {

template <class Cfg, bool PB>
__global__ __launch_bounds__(Cfg::kThreads) void gemm_stream_kernel(GemmArgs a, int nsub) {
  extern __shared__ __align__(1024) unsigned char smem_raw[];
  lds_u8_t* smem = (lds_u8_t*)smem_raw;
  unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  // consecutive ids: row tiles of one group of column tiles, then the next group, then the next problem
  const int groups_n = a.tiles_n / nsub;
  const int tm = id % a.tiles_m;  id /= a.tiles_m;
  const int tg = id % groups_n;   id /= groups_n;
  const int z0 = id % a.nz0;
  const int z1 = id / a.nz0;
  const int row0 = tm * Cfg::kBM, col0 = tg * nsub * Cfg::kBN;
  const long coff = z0 * a.sC0 + z1 * a.sC1 + (long)row0 * a.ldc + col0;
  const bf16_t* A = a.A + z0 * a.sA0 + z1 * a.sA1 + (long)row0 * a.lda;
  const float* bias = a.ep.col_bias ? a.ep.col_bias + z0 * a.ep.col_vec_stride0 + z1 * a.ep.col_vec_stride1 + col0 : nullptr;
  // row-major weights: column col0 of row 0; fragment-packed: column block col0 / 32 (K/16 fragments of 512 elements each)
  const bf16_t* B = a.B + z0 * a.sB0 + z1 * a.sB1 + (PB ? (long)(col0 / 32) * a.K * 32 : (long)col0);
  gemm_stream_tiles<Cfg, PB>(A, a.lda, B, a.ldb, PB ? (long)Cfg::kBN * a.K : (long)Cfg::kBN, a.K, nsub, smem, a.C + coff,
                             a.R ? a.R + coff : nullptr, a.ldc, bias, a.ep.act, tg, a.touch_a ? groups_n : 0);
}

template <class Cfg, bool PB = false>
static nf_status launch_stream(GemmLaunch& L, int nsub, hipStream_t s) {
  GemmArgs& a = L.a;
  if (a.rows % Cfg::kBM || a.cols % Cfg::kBN || a.K % Cfg::kBK || nsub < 1) return NF_EUNSUPPORTED;
  a.tiles_m = a.rows / Cfg::kBM;
  a.tiles_n = a.cols / Cfg::kBN;
  if (a.tiles_n % nsub) return NF_EUNSUPPORTED;
  // the register epilogue moves 16 bytes per lane (output, residual, column constants)
  if (a.ldc % 8 || ((uintptr_t)a.C & 15) || ((uintptr_t)a.R & 15) || ((uintptr_t)a.ep.col_bias & 15) ||
      a.ep.col_vec_stride0 % 4 || a.ep.col_vec_stride1 % 4 || a.sC0 % 8 || a.sC1 % 8)
    return NF_EUNSUPPORTED;
  if (!a.ep.act_before_residual && a.ep.act != NF_ACT_NONE && a.R) return NF_EUNSUPPORTED;
  if (a.ep.row_bias || a.ep.row_scale) return NF_EUNSUPPORTED;
  const long long total = (long long)a.tiles_m * (a.tiles_n / nsub) * a.nz0 * L.nz1;
  if (total <= 0 || total > 0x7fffffffLL) return NF_EUNSUPPORTED;
  a.touch_a = touch_a_pays(total, (long long)a.rows * a.K, (long long)a.nz0 * L.nz1);
  if (PB && (a.K % 16 || ((uintptr_t)a.B & 15) || a.sB0 % 8 || a.sB1 % 8 || a.lda % 8 || ((uintptr_t)a.A & 15) || a.sA0 % 8 || a.sA1 % 8))
    return NF_EUNSUPPORTED;
  auto kern = gemm_stream_kernel<Cfg, PB>;
  constexpr int kLds = Cfg::kLdsPipe;
  if (kLds > 64 * 1024) {
    static std::atomic<bool> opted_in{false};
    if (!opted_in.load(std::memory_order_acquire)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kLds) !=
          hipSuccess)
        return NF_ELAUNCH;
      opted_in.store(true, std::memory_order_release);
    }
  }
  nf_launch(kern, dim3((unsigned)total), dim3(Cfg::kThreads), kLds, s, a, nsub);
  return hipGetLastError() == hipSuccess ? NF_OK : NF_ELAUNCH;
}

nf_status launch_gemm_stream(int cfg, int nsub, GemmLaunch& L, hipStream_t s) {
  switch (cfg) {
    case S128x96k64: return launch_stream<DmaCfg<128, 96, 64, 4, 3, 5>>(L, nsub, s);
    case S128x128k32: return launch_stream<DmaCfg<128, 128, 32, 2, 4, 8>>(L, nsub, s);
    case S128x288k32: return launch_stream<DmaCfg<128, 288, 32, 4, 3, 5>>(L, nsub, s);
    case S128x384k32: return launch_stream<DmaCfg<128, 384, 32, 2, 6, NF_NS_S384>>(L, nsub, s);
    case S256x256k32: return launch_stream<DmaCfg<256, 256, 32, 2, 4, 4>>(L, nsub, s);
    case S256x128k32: return launch_stream<DmaCfg<256, 128, 32, 4, 2, 6>>(L, nsub, s);
  }
  return NF_EUNSUPPORTED;
}

nf_status launch_gemm_stream_packed(int nsub, GemmLaunch& L, hipStream_t s) {
  return launch_stream<DmaCfg<256, 256, 32, 2, 4, 4>, true>(L, nsub, s);
}

}  // namespace nf
