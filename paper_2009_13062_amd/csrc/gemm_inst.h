// Kernel template + launcher of the bf16 MFMA contraction; included by the gemm_inst_*.hip
// translation units, each of which instantiates launch_gemm_bkind for one B-loader kind.
#pragma once
#include <atomic>
#include <type_traits>

#include "gemm_launch.h"

namespace nf {

// B_NT: B is the weight matrix of a matmul, read once per forward pass: loaded non-temporal (ldnt16).
// Convolution weights (the A operand) are re-read by every position tile of a group and by design come from
// L2 after the first one, so they keep the default policy (non-temporal loads of them measured 2x slower on
// the 3x3 layers of ResNet-50).
template <class Cfg, int ALIGN_A, int BKIND, bool B_NT>
// 8-wave tiles are budgeted for two workgroups per CU: 4 wavefronts per SIMD, 128 registers per lane
// (the dense B kinds only: the gathering loaders would spill under that budget)
__global__ __launch_bounds__(Cfg::kThreads, (Cfg::kThreads == 512 && (BKIND == 8 || BKIND == 1)) ? 4 : 1)
void gemm_mfma_kernel(GemmArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  lds_bf16_t* smem = (lds_bf16_t*)smem_raw;
  unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  // consecutive ids: row tiles of one column panel, then the next panel, then the next problem,
  // so the tiles sharing a B panel (weights of the matmul) are in flight together on one XCD.
  const int tm = id % a.tiles_m;  id /= a.tiles_m;
  const int tn = id % a.tiles_n;  id /= a.tiles_n;
  const int z0 = id % a.nz0;
  const int z1 = id / a.nz0;
  const int row0 = tm * Cfg::kBM, col0 = tn * Cfg::kBN;
  const int rows_left = a.rows - row0, cols_left = a.cols - col0;

  const long coff = z0 * a.sC0 + z1 * a.sC1 + (long)row0 * a.ldc + col0;
  bf16_t* C = a.C + coff;
  const bf16_t* R = a.R ? a.R + coff : nullptr;
  const long rvo = z0 * a.ep.row_vec_stride0 + z1 * a.ep.row_vec_stride1 + row0;
  const long cvo = z0 * a.ep.col_vec_stride0 + z1 * a.ep.col_vec_stride1 + col0;
  const bf16_t* Abase = a.A + z0 * a.sA0 + z1 * a.sA1 + (long)row0 * a.lda;
  const bf16_t* Bbase = a.B + z0 * a.sB0 + z1 * a.sB1;
  if constexpr (BKIND == 0 || BKIND == 2 || BKIND == 21 || BKIND == 22 || BKIND == 24 || BKIND == 27) {
    if constexpr (BKIND == 27 && Cfg::kDepth > 1 && ALIGN_A == 16) {
      if (a.K % (kBK * Cfg::kDepth) == 0) {
        ADeepLoader<Cfg::kBM, Cfg::kThreads> la;
        la.init(Abase, a.lda, rows_left, threadIdx.x);
        BRow7DeepLoader<Cfg::kBN, Cfg::kThreads> lb;
        lb.init(Bbase, a.geom, a.cols / 7, threadIdx.x);
        gemm_tile<Cfg, true>(la, lb, a.K, smem, C, R, a.ldc, rows_left, cols_left, a.ep, rvo, cvo);
        return;
      }
    }
    if constexpr ((BKIND == 21 || BKIND == 22 || BKIND == 24) && Cfg::kDepth > 1 && ALIGN_A == 16) {
      // whole k-step multiples stream through the deep pipeline
      if (a.K % (kBK * Cfg::kDepth) == 0) {
        ADeepLoader<Cfg::kBM, Cfg::kThreads> la;
        la.init(Abase, a.lda, rows_left, threadIdx.x);
        BPairDeepLoader<Cfg::kBN, BKIND == 24 ? 4 : (BKIND == 22 ? 2 : 1), Cfg::kThreads> lb;
        lb.init(Bbase, a.geom, col0, cols_left, threadIdx.x);
        gemm_tile<Cfg, true>(la, lb, a.K, smem, C, R, a.ldc, rows_left, cols_left, a.ep, rvo, cvo);
        return;
      }
    }
    ATileLoader<Cfg::kBM, ALIGN_A, false, Cfg::kThreads> la;
    la.base = Abase; la.lda = a.lda; la.rows_left = rows_left; la.K = a.K;
    using Pairs = BStride2PairLoader<Cfg::kBN, BKIND == 24 ? 4 : 2, Cfg::kThreads>;
    using Strided = typename std::conditional<BKIND == 2 || BKIND == 21 || BKIND == 27, BStridedPointwiseLoader<Cfg::kBN, Cfg::kThreads>, Pairs>::type;
    typename std::conditional<BKIND == 0, BIm2colLoader<Cfg::kBN, Cfg::kThreads>, Strided>::type lb;
    lb.xg = Bbase; lb.g = a.geom; lb.cols_left = cols_left; lb.K = a.K; lb.col0 = col0;
    gemm_tile<Cfg>(la, lb, a.K, smem, C, R, a.ldc, rows_left, cols_left, a.ep, rvo, cvo);
  } else {
    if constexpr (Cfg::kDepth > 1 && ALIGN_A == 16) {
      // whole k-step multiples stream through the deep pipeline
      if (a.K % (kBK * Cfg::kDepth) == 0 && a.ldb >= 8) {
        ADeepLoader<Cfg::kBM, Cfg::kThreads> la;
        la.init(Abase, a.lda, rows_left, threadIdx.x);
        BDeepLoader<Cfg::kBN, BKIND == 8, Cfg::kThreads, B_NT> lb;
        lb.init(Bbase + col0, a.ldb, cols_left, a.K, a.B_end, threadIdx.x);
        gemm_tile<Cfg, true>(la, lb, a.K, smem, C, R, a.ldc, rows_left, cols_left, a.ep, rvo, cvo);
        return;
      }
    }
    auto general = [&]() {
      ATileLoader<Cfg::kBM, ALIGN_A, false, Cfg::kThreads> la;
      la.base = Abase; la.lda = a.lda; la.rows_left = rows_left; la.K = a.K;
      BDenseLoader<Cfg::kBN, BKIND == 0 ? 1 : BKIND, false, Cfg::kThreads, B_NT> lb;
      lb.base = Bbase + col0; lb.end = a.B_end; lb.ldb = a.ldb; lb.cols_left = cols_left; lb.K = a.K;
      gemm_tile<Cfg>(la, lb, a.K, smem, C, R, a.ldc, rows_left, cols_left, a.ep, rvo, cvo);
    };
    if constexpr (ALIGN_A == 16 && BKIND == 8) {
      // interior tiles of fully aligned problems run without any predicate in the k loop
      if (rows_left >= Cfg::kBM && cols_left >= Cfg::kBN && a.K % kBK == 0) {
        ATileLoader<Cfg::kBM, 16, true, Cfg::kThreads> la;
        la.base = Abase; la.lda = a.lda; la.rows_left = rows_left; la.K = a.K;
        BDenseLoader<Cfg::kBN, 8, true, Cfg::kThreads, B_NT> lb;
        lb.base = Bbase + col0; lb.end = a.B_end; lb.ldb = a.ldb; lb.cols_left = cols_left; lb.K = a.K;
        gemm_tile<Cfg>(la, lb, a.K, smem, C, R, a.ldc, rows_left, cols_left, a.ep, rvo, cvo);
      } else {
        general();
      }
    } else {
      general();
    }
  }
}

template <class Cfg, int ALIGN_A, int BKIND, bool B_NT>
nf_status launch_gemm_w(GemmLaunch& L, hipStream_t s) {
  GemmArgs& a = L.a;
  a.tiles_m = (a.rows + Cfg::kBM - 1) / Cfg::kBM;
  a.tiles_n = (a.cols + Cfg::kBN - 1) / Cfg::kBN;
  const long long total = (long long)a.tiles_m * a.tiles_n * a.nz0 * L.nz1;   // each factor < 2^31 / checked by caller
  if (total <= 0 || total > 0x7fffffffLL) return NF_EUNSUPPORTED;
  auto kern = gemm_mfma_kernel<Cfg, ALIGN_A, BKIND, B_NT>;
  if (Cfg::kLdsBytes > 64 * 1024) {
    // tiles above the default 64 KB of dynamic LDS opt in once per kernel (idempotent; a benign race)
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

// the dense B kinds serve the matmul (B = weights, non-temporal) and the pointwise convolution (B = activations)
template <class Cfg, int ALIGN_A, int BKIND>
nf_status launch_gemm(GemmLaunch& L, hipStream_t s) {
  if constexpr (BKIND == 8 || BKIND == 1) {
    if (!L.weights_are_a) return launch_gemm_w<Cfg, ALIGN_A, BKIND, true>(L, s);
  }
  return launch_gemm_w<Cfg, ALIGN_A, BKIND, false>(L, s);
}

template <int ALIGN_A, int BKIND>
nf_status launch_gemm_tile(int tile, GemmLaunch& L, hipStream_t s) {
  // depth of the load pipeline for the B kinds with branch-free loaders (the others keep one step in flight)
  constexpr bool kDense = BKIND == 8 || BKIND == 1 || BKIND == 21 || BKIND == 22 || BKIND == 24 || BKIND == 27;
  constexpr int D2 = kDense ? 2 : 1, D4 = kDense ? 4 : 1;
  switch (tile) {
    case T64x64: return launch_gemm<TileCfg<64, 64, 2, 2, D4>, ALIGN_A, BKIND>(L, s);
    case T32x128: return launch_gemm<TileCfg<32, 128, 1, 4, D2>, ALIGN_A, BKIND>(L, s);
    case T128x128w8: return launch_gemm<TileCfg<128, 128, 2, 4, D2>, ALIGN_A, BKIND>(L, s);
  }
  return NF_EUNSUPPORTED;
}

// A rows that are 8- or 4-byte aligned are read with the 2-byte loader's wider siblings only
// where a workload needs them; everything else falls to the element-wise loader.
template <int BKIND>
nf_status launch_gemm_bkind(int align_a, int tile, GemmLaunch& L, hipStream_t s) {
  if (align_a >= 16) return launch_gemm_tile<16, BKIND>(tile, L, s);
  if (align_a >= 8) return launch_gemm_tile<8, BKIND>(tile, L, s);
  return launch_gemm_tile<2, BKIND>(tile, L, s);
}

}  // namespace nf
