// bf16 MFMA contraction core shared by the merged matmul and the merged convolution.
//
//   C[z][i][j] = sum_k A[z][i][k] * B[z][k][j]     fp32 accumulation, one fused epilogue
//
// z runs over the independent input-weight pairs (models, or models x groups x images): the
// model index is a grid coordinate, never a loop inside a tile, so no tile ever mixes two models.
//
// A is row-major with k contiguous (activation rows of the matmul; weight rows of a convolution).
// B is "k-major": element (k, j) has j contiguous in memory (the matmul's W[K][Nout]; a
// convolution's input planes, where j runs over output positions).  The MFMA wants 8 consecutive
// k per lane for BOTH operands, so the B loader transposes 8x8 blocks in registers on the way from
// HBM to LDS.  Both LDS tiles are then [row][k] with a padded pitch and are read with 16-byte
// ds_reads that hit distinct banks.
//
// Workgroup = 256 threads = 4 wavefronts.  Wave (wm, wn) owns a (BM/WGM) x (BN/WGN) block of the
// tile, as FM x FN MFMA 32x32x16 accumulators.  K advances in steps of 64 with the next step's
// global loads in flight (registers) while the current one is multiplied out of LDS; LDS is
// double buffered so one barrier per step suffices.
#pragma once
#include "nf_common.h"

namespace nf {

constexpr int kBK = 64;            // k extent of one LDS stage
constexpr int kPitch = kBK + 8;    // LDS row pitch in elements: 144 B -> 16-B slots rotate by one per row

struct Epilogue {
  const float* row_bias;    // [z][i] or null      (convolution bias per output channel)
  const float* row_scale;   // [z][i] or null      (folded batch norm), with row_shift
  const float* row_shift;
  const float* col_bias;    // [z][j] or null      (matmul bias per output feature)
  const bf16_t* residual;   // addressed like C, or null (C may alias it)
  long row_vec_stride0, row_vec_stride1;   // z = z1 * nz0 + z0 -> offset z0*stride0 + z1*stride1
  long col_vec_stride0, col_vec_stride1;
  int act;
  int act_before_residual;  // matmul: act(.) + residual;  convolution: act(. + residual)
};

struct GemmShape {
  int rows, cols, K;        // per-problem extents of C and of the contraction
  int nz0, nz1;             // batch = nz1 x nz0 problems
  int tiles_m, tiles_n;
};

// ------------------------------------------------------------------------------------------
// global -> register loads of 8 consecutive k (one LDS "chunk"), for a given byte alignment
// ------------------------------------------------------------------------------------------
// ALIGN = guaranteed alignment in bytes of (row start + any multiple of ALIGN/2 elements).
// Elements at k >= klim read as zero; klim - k is a multiple of ALIGN/2 by the dispatch rules.
template <int ALIGN>
__device__ __forceinline__ uint4 load_k8(const bf16_t* p, int k, int klim, bool row_ok) {
  uint4 r = make_uint4(0, 0, 0, 0);
  if (!row_ok) return r;
  if constexpr (ALIGN == 16) {
    if (k < klim) r = *reinterpret_cast<const uint4*>(p);
  } else if constexpr (ALIGN == 8) {
    uint2 a = make_uint2(0, 0), b = make_uint2(0, 0);
    if (k < klim) a = *reinterpret_cast<const uint2*>(p);
    if (k + 4 < klim) b = *reinterpret_cast<const uint2*>(p + 4);
    r = make_uint4(a.x, a.y, b.x, b.y);
  } else if constexpr (ALIGN == 4) {
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = (k + 2 * e < klim) ? *reinterpret_cast<const uint32_t*>(p + 2 * e) : 0u;
    r = make_uint4(w[0], w[1], w[2], w[3]);
  } else {
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = (k + e < klim) ? (uint32_t)p[e] : 0u;
    r = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
  }
  return r;
}

// Loader of the A tile [BM][64]: chunk c -> row c/8, k-chunk c%8, so 8 neighbouring lanes read and
// write 128 contiguous bytes.
template <int BM, int ALIGN>
struct ATileLoader {
  static constexpr int kChunks = BM * (kBK / 8);
  static constexpr int kPer = (kChunks + 255) / 256;
  const bf16_t* base;   // A + problem offset + row0*lda
  long lda;
  int rows_left;        // rows of the problem from row0 on
  int K;
  uint4 regs[kPer];

  __device__ __forceinline__ void fetch(int k0, int tid) {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int c = tid + t * 256;
      const int r = c / 8, kc = (c % 8) * 8;
      const bool ok = (kChunks % 256 == 0 || c < kChunks) && r < rows_left;
      regs[t] = load_k8<ALIGN>(base + (long)r * lda + k0 + kc, k0 + kc, K, ok);
    }
  }
  __device__ __forceinline__ void commit(bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int c = tid + t * 256;
      if (kChunks % 256 == 0 || c < kChunks) {
        const int r = c / 8, kc = (c % 8) * 8;
        *reinterpret_cast<uint4*>(lds + r * kPitch + kc) = regs[t];
      }
    }
  }
};

// 8 (k) x VEC (j) block held as 8 rows of VEC/2 dwords -> VEC vectors of 8 consecutive k.
template <int VEC>
__device__ __forceinline__ void transpose_k8(const uint32_t (&in)[8][(VEC + 1) / 2], uint4 (&out)[VEC]) {
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    uint32_t w[4];
#pragma unroll
    for (int kp = 0; kp < 4; ++kp) {
      const uint32_t lo = in[2 * kp][e / 2], hi = in[2 * kp + 1][e / 2];
      w[kp] = (e & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
    }
    out[e] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// Loader of the B tile from a dense k-major matrix B[k][j] (j contiguous, row pitch ldb):
// task t -> k-block t%8 (8 consecutive k) and j-chunk t/8 (VEC consecutive j).  8 neighbouring
// lanes read the same j-chunk of 8 row groups and, after the register transpose, write 128
// contiguous bytes of one LDS row.  VEC = 8 / 4 / 1 needs 16 / 8 / 2-byte aligned rows.
template <int BN, int VEC>
struct BDenseLoader {
  static constexpr int kTasks = (kBK / 8) * (BN / VEC);
  static constexpr int kPer = (kTasks + 255) / 256;
  static constexpr int kDw = (VEC + 1) / 2;
  const bf16_t* base;   // B + problem offset + col0
  long ldb;
  int cols_left, K;
  uint32_t regs[kPer][8][kDw];

  __device__ __forceinline__ void fetch(int k0, int tid) {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * 256;
      const int kb = (task % 8) * 8, j = (task / 8) * VEC;
      const bool ok = (kTasks % 256 == 0 || task < kTasks) && j < cols_left;
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int k = k0 + kb + r;
        const bf16_t* p = base + (long)k * ldb + j;
        const bool live = ok && k < K;
        if constexpr (VEC == 8) {
          const uint4 v = live ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
          regs[t][r][0] = v.x; regs[t][r][1] = v.y; regs[t][r][2] = v.z; regs[t][r][3] = v.w;
        } else if constexpr (VEC == 4) {
          const uint2 v = live ? *reinterpret_cast<const uint2*>(p) : make_uint2(0, 0);
          regs[t][r][0] = v.x; regs[t][r][1] = v.y;
        } else {
          regs[t][r][0] = live ? (uint32_t)*p : 0u;
        }
      }
    }
  }
  __device__ __forceinline__ void commit(bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * 256;
      if (kTasks % 256 == 0 || task < kTasks) {
        const int kb = (task % 8) * 8, j = (task / 8) * VEC;
        uint4 out[VEC];
        transpose_k8<VEC>(regs[t], out);
#pragma unroll
        for (int e = 0; e < VEC; ++e) *reinterpret_cast<uint4*>(lds + (j + e) * kPitch + kb) = out[e];
      }
    }
  }
};

// Geometry of the implicit B matrix of a convolution: row k = (ci, ky, kx) of one group, column
// j = output position (oy, ox); element = x[channel0 + ci][oy*stride + ky*dil - pad][ox*stride + kx*dil - pad]
// or zero outside the image (Appendix A Eq. 1, cross-correlation on the zero-padded input).
struct Im2colGeom {
  int H, W, KH, KW, Wo, stride, pad, dil;
};

// Loader of the B tile gathered from the input planes: same task shape as the dense loader with
// VEC = 1 (one output position, 8 consecutive k), element-wise loads with bounds checks.
template <int BN>
struct BIm2colLoader {
  static constexpr int kTasks = (kBK / 8) * BN;
  static constexpr int kPer = kTasks / 256;
  static_assert(kTasks % 256 == 0, "tile too small");
  const bf16_t* xg;     // first input plane of this group and image
  Im2colGeom g;
  int cols_left, K, col0;
  uint4 regs[kPer];

  __device__ __forceinline__ void fetch(int k0, int tid) {
    const int khw = g.KH * g.KW;
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * 256;
      const int kb = (task % 8) * 8, j = task / 8;
      uint32_t h[8];
      if (j < cols_left) {
        const int p = col0 + j;
        const int oy = p / g.Wo, ox = p - oy * g.Wo;
        const int iy0 = oy * g.stride - g.pad, ix0 = ox * g.stride - g.pad;
        int k = k0 + kb;
        int ci = k / khw, rem = k - ci * khw;
        int ky = rem / g.KW, kx = rem - ky * g.KW;
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const int iy = iy0 + ky * g.dil, ix = ix0 + kx * g.dil;
          const bool live = (k + r) < K && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W;
          h[r] = live ? (uint32_t)xg[((long)ci * g.H + iy) * g.W + ix] : 0u;
          if (++kx == g.KW) { kx = 0; if (++ky == g.KH) { ky = 0; ++ci; } }
        }
      } else {
#pragma unroll
        for (int r = 0; r < 8; ++r) h[r] = 0u;
      }
      regs[t] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
  }
  __device__ __forceinline__ void commit(bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * 256;
      const int kb = (task % 8) * 8, j = task / 8;
      *reinterpret_cast<uint4*>(lds + j * kPitch + kb) = regs[t];
    }
  }
};

// ------------------------------------------------------------------------------------------
// The tile main loop and epilogue
// ------------------------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN>
struct TileCfg {
  static_assert(WGM * WGN == 4, "4 wavefronts per workgroup");
  static constexpr int kBM = BM, kBN = BN, kWGM = WGM, kWGN = WGN;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int FM = WM / 32, FN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
  static constexpr int kLdsA = BM * kPitch, kLdsB = BN * kPitch;          // elements per stage
  static constexpr int kLdsBytes = 2 * (kLdsA + kLdsB) * (int)sizeof(bf16_t);
};

template <class Cfg, class ALoader, class BLoader>
__device__ __forceinline__ void gemm_tile(ALoader& la, BLoader& lb, int K, bf16_t* smem,
                                          bf16_t* C, const bf16_t* R, long ldc, int rows_left,
                                          int cols_left, const Epilogue& ep, long row_vec_off,
                                          long col_vec_off) {
  constexpr int FM = Cfg::FM, FN = Cfg::FN;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / Cfg::kWGN, wn = wave % Cfg::kWGN;   // this wave's block of the tile
  bf16_t* As[2] = {smem, smem + Cfg::kLdsA};
  bf16_t* Bs[2] = {smem + 2 * Cfg::kLdsA, smem + 2 * Cfg::kLdsA + Cfg::kLdsB};

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (K + kBK - 1) / kBK;
  la.fetch(0, tid);
  lb.fetch(0, tid);
  la.commit(As[0], tid);
  lb.commit(Bs[0], tid);
  __syncthreads();

  // lane -> MFMA operand slice: row (lane % 32) of the 32-row block, k offset 8 * (lane / 32)
  const int frag_row = lane % 32, frag_k = (lane / 32) * 8;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      la.fetch((kt + 1) * kBK, tid);
      lb.fetch((kt + 1) * kBK, tid);
    }
    const bf16_t* a_lds = As[cur] + (wm * Cfg::WM + frag_row) * kPitch + frag_k;
    const bf16_t* b_lds = Bs[cur] + (wn * Cfg::WN + frag_row) * kPitch + frag_k;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8_t af[FM], bfr[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = *reinterpret_cast<const bf16x8_t*>(a_lds + i * 32 * kPitch + kk * 16);
#pragma unroll
      for (int j = 0; j < FN; ++j) bfr[j] = *reinterpret_cast<const bf16x8_t*>(b_lds + j * 32 * kPitch + kk * 16);
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      la.commit(As[cur ^ 1], tid);
      lb.commit(Bs[cur ^ 1], tid);
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator register r of a 32x32 block holds row 8*(r/4) + 4*(lane/32) + r%4,
  // column lane%32.
  const int col_in = lane % 32, row_in = (lane / 32) * 4;
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int col = wn * Cfg::WN + j * 32 + col_in;
      if (col >= cols_left) continue;
      const float cb = ep.col_bias ? ep.col_bias[col_vec_off + col] : 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = wm * Cfg::WM + i * 32 + 8 * (r / 4) + row_in + (r % 4);
        if (row >= rows_left) continue;
        float v = acc[i][j][r] + cb;
        if (ep.row_bias) v += ep.row_bias[row_vec_off + row];
        if (ep.row_scale) v = fmaf(v, ep.row_scale[row_vec_off + row], ep.row_shift[row_vec_off + row]);
        const long o = (long)row * ldc + col;
        if (ep.act_before_residual) {
          v = apply_act(v, ep.act);
          if (R) v += bf16_to_f32(R[o]);
        } else {
          if (R) v += bf16_to_f32(R[o]);
          v = apply_act(v, ep.act);
        }
        C[o] = f32_to_bf16(v);
      }
    }
  }
}

}  // namespace nf
