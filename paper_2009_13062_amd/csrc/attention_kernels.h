// Merged attention: one independent softmax(Q K^T) V problem per (model, sequence, head).  The
// model index only multiplies the number of problems (Section 3.1, operators that already have
// local computations), so it is folded into the grid with the head index.
#pragma once
#include "gemm_mfma.h"
#include "nf_common.h"

namespace nf {

struct AttnArgs {
  const void* Q; const void* K; const void* V; const float* mask; void* O;
  int M, B, S, heads, d;
  long stride_m, stride_row;
  float scale;
};

// ------------------------------------------------------------------------------------------
// General kernel (float or bf16 storage, any d <= 64*DPL): one wavefront per query row.
// Keys are visited 64 at a time (one per lane) with a running maximum and sum (online softmax);
// the output row is spread over the lanes (feature t = lane + 64 e).
// ------------------------------------------------------------------------------------------
template <typename T, int DPL>
__global__ __launch_bounds__(256) void attention_generic_kernel(AttnArgs a) {
  __shared__ float qs[4][64 * DPL];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const long wid = (long)blockIdx.x * 4 + wave;
  const long total = (long)a.M * a.B * a.heads * a.S;
  if (wid >= total) return;                       // uniform per wavefront
  const int i = (int)(wid % a.S);
  long t = wid / a.S;
  const int h = (int)(t % a.heads);  t /= a.heads;
  const int b = (int)(t % a.B);
  const int m = (int)(t / a.B);
  const T* Qp = (const T*)a.Q + (long)m * a.stride_m + ((long)b * a.S + i) * a.stride_row + (long)h * a.d;
  const T* Kp = (const T*)a.K + (long)m * a.stride_m + ((long)b * a.S) * a.stride_row + (long)h * a.d;
  const T* Vp = (const T*)a.V + (long)m * a.stride_m + ((long)b * a.S) * a.stride_row + (long)h * a.d;
  const float* mk = a.mask ? a.mask + ((long)m * a.B + b) * a.S : nullptr;
#pragma unroll
  for (int e = 0; e < DPL; ++e) {
    const int tt = lane + 64 * e;
    qs[wave][tt] = tt < a.d ? load_f32(Qp + tt) : 0.f;
  }
  __builtin_amdgcn_wave_barrier();
  float mrun = -3.0e38f, lrun = 0.f, acc[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) acc[e] = 0.f;
  for (int j0 = 0; j0 < a.S; j0 += 64) {
    const int j = j0 + lane;
    float s = -3.0e38f;
    if (j < a.S) {
      const T* kr = Kp + (long)j * a.stride_row;
      float dot = 0.f;
      for (int tt = 0; tt < a.d; ++tt) dot = fmaf(qs[wave][tt], load_f32(kr + tt), dot);
      s = dot * a.scale + (mk ? mk[j] : 0.f);
    }
    const float mnew = fmaxf(mrun, wave_max(s));
    const float p = j < a.S ? expf(s - mnew) : 0.f;
    const float corr = expf(mrun - mnew);
    lrun = lrun * corr + wave_sum(p);
#pragma unroll
    for (int e = 0; e < DPL; ++e) acc[e] *= corr;
    const int nj = min(64, a.S - j0);
    for (int jj = 0; jj < nj; ++jj) {
      const float pj = __shfl(p, jj, kWave);
      const T* vr = Vp + (long)(j0 + jj) * a.stride_row;
#pragma unroll
      for (int e = 0; e < DPL; ++e) {
        const int tt = lane + 64 * e;
        if (tt < a.d) acc[e] = fmaf(pj, load_f32(vr + tt), acc[e]);
      }
    }
    mrun = mnew;
  }
  T* Op = (T*)a.O + (((long)m * a.B + b) * a.S + i) * ((long)a.heads * a.d) + (long)h * a.d;
#pragma unroll
  for (int e = 0; e < DPL; ++e) {
    const int tt = lane + 64 * e;
    if (tt < a.d) store_f32(Op + tt, acc[e] / lrun);
  }
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel for head dimension 64.
//
// Workgroup = 4 wavefronts = 128 query rows of one (model, sequence, head); wave w owns 32 of them.
// Keys are streamed through LDS 64 at a time.  Scores are computed TRANSPOSED, S^T = K Q^T, so the
// 32x32 accumulator of a lane holds 16 keys of ONE query (lane % 32): the softmax statistics are
// per-lane scalars (the two lane halves hold the same query and are merged with one cross-half
// shuffle), and the exponentiated scores are already in the register order the second MFMA wants
// for its B operand (O^T = V^T P^T), with the key order inside a 16-key step permuted identically
// on the V^T side.  V is transposed 8x8 in registers on its way into LDS.
// ------------------------------------------------------------------------------------------
// 8 (key) x 8 (feature) block held as 8 rows of 4 dwords -> 8 vectors of 8 consecutive keys.
__device__ __forceinline__ void transpose_8x8_b16(const uint32_t (&in)[8][4], uint4 (&out)[8]) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    uint32_t w[4];
#pragma unroll
    for (int kp = 0; kp < 4; ++kp) {
      const uint32_t lo = in[2 * kp][e / 2], hi = in[2 * kp + 1][e / 2];
      w[kp] = (e & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
    }
    out[e] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

constexpr int kAttnD = 64;
constexpr int kAttnKB = 64;                 // keys per LDS stage
constexpr int kAttnKPitch = kAttnD + 8;     // K tile  [key][t]
constexpr int kAttnVPitch = kAttnKB + 4;    // V^T tile [t][key]; 136 B pitch, read in 8-byte pieces

__global__ __launch_bounds__(256) void attention_mfma_d64_kernel(AttnArgs a, int qblocks) {
  __shared__ __align__(16) bf16_t Ks[kAttnKB * kAttnKPitch];
  __shared__ __align__(16) bf16_t Vt[kAttnD * kAttnVPitch];
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int half = lane / 32, lq = lane % 32;
  unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  const int qb = id % qblocks;  id /= qblocks;
  const int h = id % a.heads;   id /= a.heads;
  const int b = id % a.B;
  const int m = id / a.B;
  const long head_off = (long)m * a.stride_m + ((long)b * a.S) * a.stride_row + (long)h * kAttnD;
  const bf16_t* Qp = (const bf16_t*)a.Q + head_off;
  const bf16_t* Kp = (const bf16_t*)a.K + head_off;
  const bf16_t* Vp = (const bf16_t*)a.V + head_off;
  const float* mk = a.mask ? a.mask + ((long)m * a.B + b) * a.S : nullptr;
  const float kLog2e = 1.4426950408889634f;
  const float sc = a.scale * kLog2e;          // scores are kept in log2 units: exp(x) = exp2(x log2 e)

  // This lane's query row as the B operand of S^T = K Q^T: 8 consecutive features per 16-step.
  const int q = qb * 128 + wave * 32 + lq;
  bf16x8_t qf[kAttnD / 16];
#pragma unroll
  for (int kk = 0; kk < kAttnD / 16; ++kk) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (q < a.S) v = *reinterpret_cast<const uint4*>(Qp + (long)q * a.stride_row + kk * 16 + half * 8);
    qf[kk] = __builtin_bit_cast(bf16x8_t, v);
  }

  f32x16_t o_acc[kAttnD / 32];
#pragma unroll
  for (int tb = 0; tb < kAttnD / 32; ++tb)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[tb][r] = 0.f;
  float mrun = -3.0e38f, lrun = 0.f;          // lrun: this half's partial sum

  for (int j0 = 0; j0 < a.S; j0 += kAttnKB) {
    // ---- stage K[j0 .. j0+64) and V^T into LDS
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int c = tid + t * 256;            // 64 keys x 8 chunks
      const int key = c / 8, kc = (c % 8) * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (j0 + key < a.S) v = *reinterpret_cast<const uint4*>(Kp + (long)(j0 + key) * a.stride_row + kc);
      *reinterpret_cast<uint4*>(Ks + key * kAttnKPitch + kc) = v;
    }
    if (tid < 64) {
      const int kb = (tid % 8) * 8, tc = (tid / 8) * 8;   // 8 keys x 8 features per task
      uint32_t in[8][4];
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (j0 + kb + r < a.S) v = *reinterpret_cast<const uint4*>(Vp + (long)(j0 + kb + r) * a.stride_row + tc);
        in[r][0] = v.x; in[r][1] = v.y; in[r][2] = v.z; in[r][3] = v.w;
      }
      uint4 out[8];
      transpose_8x8_b16(in, out);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        uint2* dst = reinterpret_cast<uint2*>(Vt + (tc + e) * kAttnVPitch + kb);
        dst[0] = make_uint2(out[e].x, out[e].y);
        dst[1] = make_uint2(out[e].z, out[e].w);
      }
    }
    __syncthreads();

    // ---- scores of this wave's 32 queries against the 64 staged keys, transposed
    f32x16_t s_acc[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s_acc[sb][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < kAttnD / 16; ++kk) {
        const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(Ks + (sb * 32 + lq) * kAttnKPitch + kk * 16 + half * 8);
        s_acc[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s_acc[sb], 0, 0, 0);
      }
    }
    // register r of block sb is key j0 + 32 sb + 8 (r/4) + 4 half + r%4, query lane%32
    float mloc = -3.0e38f;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = j0 + sb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
        float s = s_acc[sb][r] * sc;
        if (mk && key < a.S) s += mk[key] * kLog2e;
        s = key < a.S ? s : -3.0e38f;
        s_acc[sb][r] = s;
        mloc = fmaxf(mloc, s);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, kWave));
    const float mnew = fmaxf(mrun, mloc);
    const float corr = __builtin_amdgcn_exp2f(mrun - mnew);
    mrun = mnew;
    float psum = 0.f;
    bf16x8_t pf[2][2];                         // [sb][16-key step]
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(s_acc[sb][8 * st + 2 * e] - mnew);
          const float p1 = __builtin_amdgcn_exp2f(s_acc[sb][8 * st + 2 * e + 1] - mnew);
          const bf16_t h0 = f32_to_bf16(p0), h1 = f32_to_bf16(p1);
          psum += bf16_to_f32(h0) + bf16_to_f32(h1);      // sum what is actually multiplied
          w[e] = (uint32_t)h0 | ((uint32_t)h1 << 16);
        }
        uint4 v = make_uint4(w[0], w[1], w[2], w[3]);
        pf[sb][st] = __builtin_bit_cast(bf16x8_t, v);
      }
    lrun = lrun * corr + psum;
#pragma unroll
    for (int tb = 0; tb < kAttnD / 32; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[tb][r] *= corr;

    // ---- O^T += V^T P^T: step (sb, st) covers keys 32 sb + 16 st + {4 half + 0..3, 8 + 4 half + 0..3}
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int tb = 0; tb < kAttnD / 32; ++tb) {
          const bf16_t* vp = Vt + (tb * 32 + lq) * kAttnVPitch + sb * 32 + st * 16 + 4 * half;
          const uint2 lo = *reinterpret_cast<const uint2*>(vp);
          const uint2 hi = *reinterpret_cast<const uint2*>(vp + 8);
          uint4 v = make_uint4(lo.x, lo.y, hi.x, hi.y);
          o_acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, v), pf[sb][st],
                                                              o_acc[tb], 0, 0, 0);
        }
    __syncthreads();
  }

  const float ltot = lrun + __shfl_xor(lrun, 32, kWave);
  if (q < a.S) {
    const float inv = 1.0f / ltot;
    bf16_t* Op = (bf16_t*)a.O + (((long)m * a.B + b) * a.S + q) * ((long)a.heads * kAttnD) + (long)h * kAttnD;
#pragma unroll
    for (int tb = 0; tb < kAttnD / 32; ++tb)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        uint2 v;
        v.x = (uint32_t)f32_to_bf16(o_acc[tb][4 * rg] * inv) | ((uint32_t)f32_to_bf16(o_acc[tb][4 * rg + 1] * inv) << 16);
        v.y = (uint32_t)f32_to_bf16(o_acc[tb][4 * rg + 2] * inv) | ((uint32_t)f32_to_bf16(o_acc[tb][4 * rg + 3] * inv) << 16);
        *reinterpret_cast<uint2*>(Op + tb * 32 + 8 * rg + 4 * half) = v;
      }
  }
}

}  // namespace nf
