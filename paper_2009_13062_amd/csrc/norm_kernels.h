// HBM-bound kernels: merged layer norm (one wavefront per row of one model), merged inference
// batch norm, its folding into scale/shift, pools and the merge-dimension transpose.
#pragma once
#include "nf_common.h"

namespace nf {

template <typename T, int VEC> struct VecIO;
template <> struct VecIO<float, 4> {
  static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct VecIO<bf16_t, 4> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[4]) {
    const uint2 t = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[4]) {
    uint2 t;
    t.x = pack_bf16x2(v[0], v[1]);
    t.y = pack_bf16x2(v[2], v[3]);
    *reinterpret_cast<uint2*>(p) = t;
  }
};
template <typename T> struct VecIO<T, 1> {
  static __device__ __forceinline__ void load(const T* p, float (&v)[1]) { v[0] = load_f32(p); }
  static __device__ __forceinline__ void store(T* p, const float (&v)[1]) { store_f32(p, v[0]); }
};

// Merged layer norm = group norm with M groups (Section 3.1).  One 64-lane wavefront owns one
// (model, row): statistics are reduced across the lanes, never across models.  A row of up to
// 64*VEC*MAXIT features stays in registers between the passes (x and residual are read once);
// longer rows are re-read from L2.  mean, then mean of squared deviations (biased), in fp32.
template <typename T, int VEC, int MAXIT>
__global__ __launch_bounds__(256) void layernorm_kernel(
    const T* x, const T* residual, const float* __restrict__ gamma, const float* __restrict__ beta,
    T* y, int M, int rows, int H, float eps, int channel_layout) {
  const int lane = threadIdx.x % kWave;
  const long wrow = (long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;   // m*rows + r
  if (wrow >= (long)M * rows) return;
  const int m = (int)(wrow / rows), r = (int)(wrow % rows);
  const size_t base = channel_layout ? ((size_t)r * M + m) * H : ((size_t)m * rows + r) * H;
  const T* xr = x + base;
  const T* rr = residual ? residual + base : nullptr;
  const float* gm = gamma + (size_t)m * H;
  const float* bt = beta + (size_t)m * H;
  const bool cached = H <= kWave * VEC * MAXIT;
  float v[MAXIT][VEC];
  float sum = 0.f;
  if (cached) {
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
      const int i = (it * kWave + lane) * VEC;
      if (i < H) {
        VecIO<T, VEC>::load(xr + i, v[it]);
        if (rr) {
          float t[VEC];
          VecIO<T, VEC>::load(rr + i, t);
#pragma unroll
          for (int e = 0; e < VEC; ++e) v[it][e] += t[e];
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) sum += v[it][e];
      }
    }
  } else {
    for (int i = lane * VEC; i < H; i += kWave * VEC) {
      float a[VEC];
      VecIO<T, VEC>::load(xr + i, a);
      if (rr) {
        float t[VEC];
        VecIO<T, VEC>::load(rr + i, t);
#pragma unroll
        for (int e = 0; e < VEC; ++e) a[e] += t[e];
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) sum += a[e];
    }
  }
  const float mean = wave_sum(sum) / (float)H;
  float sq = 0.f;
  if (cached) {
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
      const int i = (it * kWave + lane) * VEC;
      if (i < H) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { const float dlt = v[it][e] - mean; sq = fmaf(dlt, dlt, sq); }
      }
    }
  } else {
    for (int i = lane * VEC; i < H; i += kWave * VEC) {
      float a[VEC];
      VecIO<T, VEC>::load(xr + i, a);
      if (rr) {
        float t[VEC];
        VecIO<T, VEC>::load(rr + i, t);
#pragma unroll
        for (int e = 0; e < VEC; ++e) a[e] += t[e];
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) { const float dlt = a[e] - mean; sq = fmaf(dlt, dlt, sq); }
    }
  }
  const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)H + eps);
  T* yr = y + base;
  if (cached) {
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
      const int i = (it * kWave + lane) * VEC;
      if (i < H) {
        float o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = fmaf((v[it][e] - mean) * rstd, gm[i + e], bt[i + e]);
        VecIO<T, VEC>::store(yr + i, o);
      }
    }
  } else {
    for (int i = lane * VEC; i < H; i += kWave * VEC) {
      float a[VEC], o[VEC];
      VecIO<T, VEC>::load(xr + i, a);
      if (rr) {
        float t[VEC];
        VecIO<T, VEC>::load(rr + i, t);
#pragma unroll
        for (int e = 0; e < VEC; ++e) a[e] += t[e];
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) o[e] = fmaf((a[e] - mean) * rstd, gm[i + e], bt[i + e]);
      VecIO<T, VEC>::store(yr + i, o);
    }
  }
}

// The same for rows that fit in registers, ROWS consecutive rows of one model per wavefront (rows % ROWS
// == 0): gamma and beta, 8 bytes per feature against 2 or 4 of the row itself, are fetched once per ROWS
// rows instead of once per row, and the loads of all ROWS rows are in flight together.
template <typename T, int VEC, int MAXIT, int ROWS>
__global__ __launch_bounds__(256) void layernorm_rows_kernel(
    const T* x, const T* residual, const float* __restrict__ gamma, const float* __restrict__ beta,
    T* y, int M, int rows, int H, float eps, int channel_layout) {
  const int lane = threadIdx.x % kWave;
  const long wrow = ((long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave) * ROWS;   // m*rows + r of the first row
  if (wrow >= (long)M * rows) return;
  const int m = (int)(wrow / rows), r0 = (int)(wrow % rows);
  const float* gm = gamma + (size_t)m * H;
  const float* bt = beta + (size_t)m * H;
  size_t base[ROWS];
#pragma unroll
  for (int q = 0; q < ROWS; ++q)
    base[q] = channel_layout ? ((size_t)(r0 + q) * M + m) * H : ((size_t)m * rows + r0 + q) * H;
  float v[ROWS][MAXIT][VEC];
  float sum[ROWS];
#pragma unroll
  for (int q = 0; q < ROWS; ++q) {
    sum[q] = 0.f;
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
      const int i = (it * kWave + lane) * VEC;
      if (i < H) {
        VecIO<T, VEC>::load(x + base[q] + i, v[q][it]);
        if (residual) {
          float t[VEC];
          VecIO<T, VEC>::load(residual + base[q] + i, t);
#pragma unroll
          for (int e = 0; e < VEC; ++e) v[q][it][e] += t[e];
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) sum[q] += v[q][it][e];
      }
    }
  }
  float mean[ROWS], rstd[ROWS];
#pragma unroll
  for (int q = 0; q < ROWS; ++q) mean[q] = wave_sum(sum[q]) / (float)H;
#pragma unroll
  for (int q = 0; q < ROWS; ++q) {
    float sq = 0.f;
#pragma unroll
    for (int it = 0; it < MAXIT; ++it) {
      const int i = (it * kWave + lane) * VEC;
      if (i < H) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { const float dlt = v[q][it][e] - mean[q]; sq = fmaf(dlt, dlt, sq); }
      }
    }
    rstd[q] = 1.0f / sqrtf(wave_sum(sq) / (float)H + eps);
  }
#pragma unroll
  for (int it = 0; it < MAXIT; ++it) {
    const int i = (it * kWave + lane) * VEC;
    if (i < H) {
      float g[VEC], b[VEC];
#pragma unroll
      for (int e = 0; e < VEC; ++e) { g[e] = gm[i + e]; b[e] = bt[i + e]; }
#pragma unroll
      for (int q = 0; q < ROWS; ++q) {
        float o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = fmaf((v[q][it][e] - mean[q]) * rstd[q], g[e], b[e]);
        VecIO<T, VEC>::store(y + base[q] + i, o);
      }
    }
  }
}

// Merged inference batch norm (Section 3.1): per merged channel c of x[B][Ctot][HW].
// One workgroup row per (b, c); gridDim.y splits long HW.
template <typename T>
__global__ __launch_bounds__(256) void batchnorm_kernel(
    const T* x, const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ var, const T* residual, T* y,
    int Ctot, int HW, float eps, int act) {
  const size_t bc = blockIdx.x;
  const int c = (int)(bc % Ctot);
  const float s = gamma[c] / sqrtf(var[c] + eps);
  const float mu = mean[c], bta = beta[c];
  const size_t base = bc * (size_t)HW;
  for (int p = blockIdx.y * 256 + threadIdx.x; p < HW; p += gridDim.y * 256) {
    float v = fmaf(load_f32(x + base + p) - mu, s, bta);
    if (residual) v += load_f32(residual + base + p);
    store_f32(y + base + p, apply_act(v, act));
  }
}

// The same operator over the flat tensor, 16 bytes per thread (8 bf16 or 4 float): a chunk starts in channel
// (f / HW) % Ctot and walks on to the next channel where a plane ends inside it (planes of 49 or 196
// elements), so every plane size moves whole, aligned 16-byte accesses and small planes leave no lanes
// idle.  Needs 16-byte aligned tensors and an element count that is a multiple of the chunk.
template <typename T>
__global__ __launch_bounds__(256) void batchnorm_flat_kernel(
    const T* x, const float* __restrict__ gamma, const float* __restrict__ beta,
    const float* __restrict__ mean, const float* __restrict__ var, const T* residual, T* y,
    int Ctot, int HW, float eps, int act, size_t chunks) {
  constexpr int V = 16 / (int)sizeof(T);
  const size_t ch = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (ch >= chunks) return;
  const size_t f0 = ch * V;
  int c = (int)((f0 / HW) % Ctot), p = (int)(f0 % HW);
  float s = gamma[c] / sqrtf(var[c] + eps), mu = mean[c], bta = beta[c];
  float v[V], r[V];
  if constexpr (sizeof(T) == 2) {
    const uint4 xv = *reinterpret_cast<const uint4*>(x + f0);
    const uint32_t w[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[2 * e] = __uint_as_float(w[e] << 16); v[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u); }
    uint4 rv = make_uint4(0, 0, 0, 0);
    if (residual) rv = *reinterpret_cast<const uint4*>(residual + f0);
    const uint32_t q[4] = {rv.x, rv.y, rv.z, rv.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) { r[2 * e] = __uint_as_float(q[e] << 16); r[2 * e + 1] = __uint_as_float(q[e] & 0xffff0000u); }
  } else {
    const float4 xv = *reinterpret_cast<const float4*>(x + f0);
    v[0] = xv.x; v[1] = xv.y; v[2] = xv.z; v[3] = xv.w;
    float4 rv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (residual) rv = *reinterpret_cast<const float4*>(residual + f0);
    r[0] = rv.x; r[1] = rv.y; r[2] = rv.z; r[3] = rv.w;
  }
#pragma unroll
  for (int e = 0; e < V; ++e) {
    float o = fmaf(v[e] - mu, s, bta);
    if (residual) o += r[e];
    v[e] = apply_act(o, act);
    if (++p == HW && e + 1 < V) {              // the plane ends inside the chunk: next channel (next image after the last)
      p = 0;
      c = c + 1 == Ctot ? 0 : c + 1;
      s = gamma[c] / sqrtf(var[c] + eps); mu = mean[c]; bta = beta[c];
    }
  }
  if constexpr (sizeof(T) == 2) {
    *reinterpret_cast<uint4*>(y + f0) = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                                                   pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
  } else {
    *reinterpret_cast<float4*>(y + f0) = make_float4(v[0], v[1], v[2], v[3]);
  }
}

__global__ __launch_bounds__(256) void bn_fold_kernel(
    const float* __restrict__ gamma, const float* __restrict__ beta, const float* __restrict__ mean,
    const float* __restrict__ var, float* scale, float* shift, int n, float eps) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= n) return;
  const float s = gamma[c] / sqrtf(var[c] + eps);
  scale[c] = s;
  shift[c] = beta[c] - mean[c] * s;
}

// Max pooling per channel of the channel-merged tensor (Section 3.1, non-trainable operators).
template <typename T>
__global__ __launch_bounds__(256) void maxpool2d_kernel(const T* __restrict__ x, T* y, int H, int W,
                                                        int Ho, int Wo, int k, int stride, int pad,
                                                        size_t total) {
  for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256) {
    const int ox = (int)(o % Wo);
    size_t t = o / Wo;
    const int oy = (int)(t % Ho);
    const size_t bc = t / Ho;
    const T* xc = x + bc * (size_t)H * W;
    float best = -INFINITY;
    for (int ky = 0; ky < k; ++ky) {
      const int iy = oy * stride + ky - pad;
      if (iy < 0 || iy >= H) continue;
      for (int kx = 0; kx < k; ++kx) {
        const int ix = ox * stride + kx - pad;
        if (ix < 0 || ix >= W) continue;
        const float v = load_f32(xc + (size_t)iy * W + ix);
        best = v > best ? v : best;
      }
    }
    store_f32(y + o, best);
  }
}

// The ResNet stem pool: 3x3 window, stride 2, pad 1 on bf16 rows whose width is a multiple of 8.  One
// thread produces 4 consecutive outputs of a row from one 16-byte load (8 pixels) plus the pixel to their
// left per input row; same comparison as the general kernel (v > best, so NaN inputs are ignored).
__global__ __launch_bounds__(256) void maxpool3x3s2_bf16_kernel(const bf16_t* __restrict__ x, bf16_t* y, int H, int W,
                                                                int Ho, int Wo, size_t total4) {
  const int q = Wo / 4;
  for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total4; o += (size_t)gridDim.x * 256) {
    const int ox0 = (int)(o % q) * 4;
    size_t t = o / q;
    const int oy = (int)(t % Ho);
    const size_t bc = t / Ho;
    const bf16_t* xc = x + bc * (size_t)H * W;
    float m[9];                                   // column maxima over the 3 input rows: cols 2 ox0 - 1 .. 2 ox0 + 7
#pragma unroll
    for (int c = 0; c < 9; ++c) m[c] = -INFINITY;
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
      const int iy = oy * 2 + ky - 1;
      if (iy < 0 || iy >= H) continue;
      const bf16_t* row = xc + (size_t)iy * W + ox0 * 2;
      const uint4 v = *reinterpret_cast<const uint4*>(row);
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      if (ox0 > 0) { const float l = bf16_to_f32(row[-1]); m[0] = l > m[0] ? l : m[0]; }
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const float f = __uint_as_float(c % 2 ? (w[c / 2] & 0xffff0000u) : (w[c / 2] << 16));
        m[c + 1] = f > m[c + 1] ? f : m[c + 1];
      }
    }
    uint32_t out[2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float best = m[2 * j];
      best = m[2 * j + 1] > best ? m[2 * j + 1] : best;
      best = m[2 * j + 2] > best ? m[2 * j + 2] : best;
      const uint32_t h = (uint32_t)f32_to_bf16(best);
      if (j % 2) out[j / 2] |= h << 16; else out[j / 2] = h;
    }
    *reinterpret_cast<uint2*>(y + (bc * Ho + oy) * (size_t)Wo + ox0) = make_uint2(out[0], out[1]);
  }
}

// Global average pooling: one wavefront per (b, channel).
template <typename T>
__global__ __launch_bounds__(256) void avgpool_global_kernel(const T* __restrict__ x, T* y, size_t nchan,
                                                             int HW) {
  const int lane = threadIdx.x % kWave;
  const size_t ch = (size_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
  if (ch >= nchan) return;
  const T* xc = x + ch * (size_t)HW;
  float s = 0.f;
  for (int p = lane; p < HW; p += kWave) s += load_f32(xc + p);
  s = wave_sum(s);
  if (lane == 0) store_f32(y + ch, s / (float)HW);
}

// The same for planes of at most 64 positions (the 7 x 7 output of a ResNet): 16 lanes per channel, 4
// channels per wavefront, so a wavefront reads 4 * HW contiguous elements instead of HW.
template <typename T>
__global__ __launch_bounds__(256) void avgpool_global_small_kernel(const T* __restrict__ x, T* y, size_t nchan,
                                                                   int HW) {
  const int sub = threadIdx.x % 16;
  const size_t ch = ((size_t)blockIdx.x * 256 + threadIdx.x) / 16;
  float s = 0.f;
  if (ch < nchan) {
    const T* xc = x + ch * (size_t)HW;
    for (int p = sub; p < HW; p += 16) s += load_f32(xc + p);
  }
#pragma unroll
  for (int d = 8; d >= 1; d /= 2) s += __shfl_xor(s, d, 16);
  if (sub == 0 && ch < nchan) store_f32(y + ch, s / (float)HW);
}

// Batch-merged [M][rows][H] <-> channel-merged [rows][M*H] (Section 3.2, Algorithm 1's reshape).
// Index o runs over the destination, so writes are fully coalesced; reads are H-contiguous runs.
template <typename T>
__global__ __launch_bounds__(256) void merge_transpose_kernel(const T* __restrict__ src, T* dst, int M,
                                                              int rows, int H, int to_channel,
                                                              size_t total) {
  for (size_t o = (size_t)blockIdx.x * 256 + threadIdx.x; o < total; o += (size_t)gridDim.x * 256) {
    const int i = (int)(o % H);
    size_t t = o / H;
    size_t s;
    if (to_channel) {            // dst[r][m][i] <- src[m][r][i]
      const int m = (int)(t % M);
      const size_t r = t / M;
      s = ((size_t)m * rows + r) * H + i;
    } else {                     // dst[m][r][i] <- src[r][m][i]
      const int r = (int)(t % rows);
      const size_t m = t / rows;
      s = ((size_t)r * M + m) * H + i;
    }
    dst[o] = src[s];
  }
}

}  // namespace nf
