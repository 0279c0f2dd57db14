// General-shape kernels for the merged matmul and the merged convolution: plain fp32 FMA, any
// size, any alignment, float or bf16 storage.  They serve the fp32 storage type and every bf16
// shape the MFMA kernels do not take.
#pragma once
#include "nf_common.h"

namespace nf {

// Ragged merged matmul: per-model output widths (the per-task classification heads, Section 5.1).
// One workgroup = (model, 8 rows, 64 columns); its 4 wavefronts split K, each lane owns one column and 8
// rows, so a wavefront reads 64 consecutive weights of a k row (coalesced, any alignment) and the
// activations as wave-uniform broadcasts; the four partial sums meet in LDS.  The model of a workgroup is
// found from the prefix sums of the per-model tile counts, which travel in the kernel arguments.
constexpr int kRaggedMaxModels = 256;
struct RaggedTable {
  int tile_start[kRaggedMaxModels + 1];   // first workgroup of model m (prefix sum of rows tiles x column tiles)
  int col_start[kRaggedMaxModels + 1];    // first output column of model m in the concatenation (prefix sum of nout)
};

template <typename T>
__global__ __launch_bounds__(256) void linear_ragged_kernel(const T* __restrict__ X, const T* __restrict__ W,
                                                           const float* __restrict__ bias, T* __restrict__ Y, int M,
                                                           int N, int K, int act, RaggedTable tab) {
  __shared__ float part[4][8][64];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  // binary search: the last model whose first tile is <= blockIdx.x
  int lo = 0, hi = M - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) / 2;
    if (tab.tile_start[mid] <= (int)blockIdx.x) lo = mid; else hi = mid - 1;
  }
  const int m = lo;
  const int nout = tab.col_start[m + 1] - tab.col_start[m];
  const int tiles_n = (nout + 63) / 64;
  const int t = blockIdx.x - tab.tile_start[m];
  const int row0 = (t / tiles_n) * 8, col = (t % tiles_n) * 64 + lane;
  const T* Xm = X + ((size_t)m * N + row0) * K;
  const T* Wm = W + (size_t)tab.col_start[m] * K;          // model m's [K][nout] block of the concatenation
  const int rows = min(8, N - row0);
  float acc[8] = {};
  const int kper = (K + 3) / 4, k0 = wave * kper, k1 = min(K, k0 + kper);
  if (col < nout) {
    for (int k = k0; k < k1; ++k) {
      const float w = load_f32(Wm + (size_t)k * nout + col);
#pragma unroll
      for (int r = 0; r < 8; ++r)
        if (r < rows) acc[r] = fmaf(load_f32(Xm + (size_t)r * K + k), w, acc[r]);
    }
  }
#pragma unroll
  for (int r = 0; r < 8; ++r) part[wave][r][lane] = acc[r];
  __syncthreads();
  // 512 outputs, 256 threads: two each; the k slices are added in order
  for (int o = threadIdx.x; o < 8 * 64; o += 256) {
    const int r = o / 64, c = (t % tiles_n) * 64 + o % 64;
    if (r >= rows || c >= nout) continue;
    float v = ((part[0][r][o % 64] + part[1][r][o % 64]) + part[2][r][o % 64]) + part[3][r][o % 64];
    if (bias) v += bias[tab.col_start[m] + c];
    v = apply_act(v, act);
    store_f32(Y + (size_t)tab.col_start[m] * N + (size_t)(row0 + r) * nout + c, v);
  }
}

// Merged matmul (Section 3.1): one 64x64 output tile of one model per workgroup; the model
// index is folded into the grid.  256 threads, 4x4 outputs each, K in steps of 16 through LDS.
template <typename T>
__global__ __launch_bounds__(256) void linear_generic_kernel(
    const T* __restrict__ X, const T* __restrict__ W, const float* __restrict__ bias,
    const T* residual, T* Y, int N, int K, int Nout, int act, int tiles_m, int tiles_n) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tid = threadIdx.x;
  unsigned id = blockIdx.x;
  const int tn = id % tiles_n;  id /= tiles_n;
  const int tm = id % tiles_m;  id /= tiles_m;
  const int m = id;
  const int row0 = tm * 64, col0 = tn * 64;
  const T* Xm = X + (size_t)m * N * K;
  const T* Wm = W + (size_t)m * K * Nout;
  const int tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int idx = tid + t * 256;
      const int r = idx / 16, k = idx % 16;
      const int gr = row0 + r, gk = k0 + k;
      As[k][r] = (gr < N && gk < K) ? load_f32(Xm + (size_t)gr * K + gk) : 0.f;
      const int kb = idx / 64, c = idx % 64;
      const int gc = col0 + c, gkb = k0 + kb;
      Bs[kb][c] = (gc < Nout && gkb < K) ? load_f32(Wm + (size_t)gkb * Nout + gc) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gr = row0 + ty * 4 + i;
    if (gr >= N) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gc = col0 + tx * 4 + j;
      if (gc >= Nout) continue;
      float v = acc[i][j];
      if (bias) v += bias[(size_t)m * Nout + gc];
      v = apply_act(v, act);
      const size_t o = ((size_t)m * N + gr) * Nout + gc;
      if (residual) v += load_f32(residual + o);
      store_f32(Y + o, v);
    }
  }
}

struct ConvGeom {
  int B, Ctot_in, Ctot_out, cig, cog;   // merged channel counts; per-group channel counts
  int H, W, KH, KW, Ho, Wo, stride, pad, dil;
};

// Merged convolution (Appendix A Eq. 2 with M*g groups): one thread per output element; the
// group of merged output channel c is c / cog and its first input channel is (c / cog) * cig.
template <typename T>
__global__ __launch_bounds__(256) void conv2d_generic_kernel(
    const T* __restrict__ x, const T* __restrict__ w, const float* __restrict__ bias,
    const float* __restrict__ scale, const float* __restrict__ shift, const T* residual, T* y,
    ConvGeom g, int act, size_t total) {
  for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256) {
    const int ox = (int)(o % g.Wo);
    size_t t = o / g.Wo;
    const int oy = (int)(t % g.Ho);  t /= g.Ho;
    const int c = (int)(t % g.Ctot_out);
    const int b = (int)(t / g.Ctot_out);
    const int cbase = (c / g.cog) * g.cig;
    const T* wc = w + (size_t)c * g.cig * g.KH * g.KW;
    float acc = 0.f;
    for (int ci = 0; ci < g.cig; ++ci) {
      const T* xc = x + ((size_t)b * g.Ctot_in + cbase + ci) * g.H * g.W;
      for (int ky = 0; ky < g.KH; ++ky) {
        const int iy = oy * g.stride + ky * g.dil - g.pad;
        if (iy < 0 || iy >= g.H) continue;
        for (int kx = 0; kx < g.KW; ++kx) {
          const int ix = ox * g.stride + kx * g.dil - g.pad;
          if (ix < 0 || ix >= g.W) continue;
          acc = fmaf(load_f32(wc + (ci * g.KH + ky) * g.KW + kx), load_f32(xc + (size_t)iy * g.W + ix), acc);
        }
      }
    }
    if (bias) acc += bias[c];
    if (scale) acc = fmaf(acc, scale[c], shift[c]);
    if (residual) acc += load_f32(residual + o);
    store_f32(y + o, apply_act(acc, act));
  }
}

}  // namespace nf
