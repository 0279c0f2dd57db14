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
// Relative-position attention (Transformer-XL / XLNet form), general kernel: as above, with the score
//   s_ij = scale * ( (q_i + bias_w) . k_j  +  (q_i + bias_r) . kr[S - i + j] ) + mask_j
// where kr[p] is the model's projected encoding of relative distance S - p (row p of Kr[M][2S][heads*d]).
// The two biased copies of the query row sit in LDS; lane j walks its key row and its position row.
// ------------------------------------------------------------------------------------------
struct AttnRelArgs {
  AttnArgs a;
  const void* Kr;          // [M][2S][heads*d], storage type of Q
  const float* bias_w;     // [M][heads*d] or null
  const float* bias_r;     // [M][heads*d] or null
};

template <typename T, int DPL>
__global__ __launch_bounds__(256) void attention_relpos_kernel(AttnRelArgs ra) {
  const AttnArgs& a = ra.a;
  __shared__ float qw[4][64 * DPL];
  __shared__ float qr[4][64 * DPL];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const long wid = (long)blockIdx.x * 4 + wave;
  const long total = (long)a.M * a.B * a.heads * a.S;
  if (wid >= total) return;                       // uniform per wavefront
  const int i = (int)(wid % a.S);
  long t = wid / a.S;
  const int h = (int)(t % a.heads);  t /= a.heads;
  const int b = (int)(t % a.B);
  const int m = (int)(t / a.B);
  const long hd = (long)a.heads * a.d;
  const T* Qp = (const T*)a.Q + (long)m * a.stride_m + ((long)b * a.S + i) * a.stride_row + (long)h * a.d;
  const T* Kp = (const T*)a.K + (long)m * a.stride_m + ((long)b * a.S) * a.stride_row + (long)h * a.d;
  const T* Vp = (const T*)a.V + (long)m * a.stride_m + ((long)b * a.S) * a.stride_row + (long)h * a.d;
  const T* Rp = (const T*)ra.Kr + ((long)m * 2 * a.S + (a.S - i)) * hd + (long)h * a.d;     // row S - i + j at + j*hd
  const float* mk = a.mask ? a.mask + ((long)m * a.B + b) * a.S : nullptr;
#pragma unroll
  for (int e = 0; e < DPL; ++e) {
    const int tt = lane + 64 * e;
    const float q = tt < a.d ? load_f32(Qp + tt) : 0.f;
    qw[wave][tt] = tt < a.d ? q + (ra.bias_w ? ra.bias_w[m * hd + h * a.d + tt] : 0.f) : 0.f;
    qr[wave][tt] = tt < a.d ? q + (ra.bias_r ? ra.bias_r[m * hd + h * a.d + tt] : 0.f) : 0.f;
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
      const T* pr = Rp + (long)j * hd;
      float ac = 0.f, bd = 0.f;
      for (int tt = 0; tt < a.d; ++tt) {
        ac = fmaf(qw[wave][tt], load_f32(kr + tt), ac);
        bd = fmaf(qr[wave][tt], load_f32(pr + tt), bd);
      }
      s = (ac + bd) * a.scale + (mk ? mk[j] : 0.f);
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
  T* Op = (T*)a.O + (((long)m * a.B + b) * a.S + i) * hd + (long)h * a.d;
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
// Keys and values are streamed through LDS 64 at a time, double buffered, with the next block's
// global loads in flight in registers while the current one is used.  Scores are computed
// TRANSPOSED, S^T = K Q^T, so the 32x32 accumulator of a lane holds 16 keys of ONE query
// (lane % 32): the softmax statistics are per-lane scalars (the two lane halves hold the same query
// and are merged with one cross-half shuffle), and the exponentiated scores are already in the
// register order the second MFMA wants for its B operand (O^T = V^T P^T), with the key order inside
// a 16-key step permuted identically on the V^T side.  V stays [key][feature] in LDS as in memory;
// the V^T fragments come from the transposing LDS read (ds_read_b64_tr_b16).
// ------------------------------------------------------------------------------------------
constexpr int kAttnD = 64;
constexpr int kAttnKB = 64;                 // keys per LDS stage
constexpr int kAttnKPitch = kAttnD + 8;     // K tile [key][t]: 144 B rows, 16-byte fragment reads
constexpr int kAttnVPitch = kAttnD + 32;    // V tile [key][t]: 192 B rows, so the 4 keys x 64 B that 32 lanes of a
                                            // transposing read touch tile the 256 bytes of the 64 LDS banks

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3))) void attention_mfma_d64_kernel(AttnArgs a, int qblocks) {
  __shared__ __align__(16) bf16_t Ks_raw[2 * kAttnKB * kAttnKPitch];
  __shared__ __align__(16) bf16_t Vs_raw[2 * kAttnKB * kAttnVPitch];
  lds_bf16_t* const Ks = (lds_bf16_t*)Ks_raw;
  lds_bf16_t* const Vs = (lds_bf16_t*)Vs_raw;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int half = lane / 32, lq = lane % 32, l16 = lane % 16;
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

  // K and V blocks: 64 keys x 8 chunks of 16 bytes each = 2 chunks per thread per tensor
  uint4 kreg[2], vreg[2];
  auto fetch = [&](int j0) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int c = tid + t * 256, key = c / 8, kc = (c % 8) * 8;
      kreg[t] = vreg[t] = make_uint4(0, 0, 0, 0);
      if (j0 + key < a.S) {
        kreg[t] = *reinterpret_cast<const uint4*>(Kp + (long)(j0 + key) * a.stride_row + kc);
        vreg[t] = *reinterpret_cast<const uint4*>(Vp + (long)(j0 + key) * a.stride_row + kc);
      }
    }
  };
  auto commit = [&](int stage) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int c = tid + t * 256, key = c / 8, kc = (c % 8) * 8;
      lds_store16(Ks + stage * kAttnKB * kAttnKPitch + key * kAttnKPitch + kc, kreg[t]);
      lds_store16(Vs + stage * kAttnKB * kAttnVPitch + key * kAttnVPitch + kc, vreg[t]);
    }
  };
  fetch(0);
  commit(0);
  __syncthreads();

  const int nblk = (a.S + kAttnKB - 1) / kAttnKB;
  for (int blk = 0; blk < nblk; ++blk) {
    const int j0 = blk * kAttnKB, cur = blk & 1;
    if (blk + 1 < nblk) fetch(j0 + kAttnKB);
    const lds_bf16_t* Kc = Ks + cur * kAttnKB * kAttnKPitch;
    const lds_bf16_t* Vc = Vs + cur * kAttnKB * kAttnVPitch;

    // ---- scores of this wave's 32 queries against the 64 staged keys, transposed; the two 32-key
    // accumulators are independent and alternate in the matrix pipe
    f32x16_t s_acc[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_acc[sb][r] = 0.f;
    {
      bf16x8_t kf[kAttnD / 16][2];
#pragma unroll
      for (int kk = 0; kk < kAttnD / 16; ++kk)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
          kf[kk][sb] = *(const lds_bf16x8_t*)(Kc + (sb * 32 + lq) * kAttnKPitch + kk * 16 + half * 8);
#pragma unroll
      for (int kk = 0; kk < kAttnD / 16; ++kk)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
          s_acc[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk][sb], qf[kk], s_acc[sb], 0, 0, 0);
    }
    // register r of block sb is key j0 + 32 sb + 8 (r/4) + 4 half + r%4, query lane%32
    // Without a mask and with a positive scale (uniform over the launch) the scores stay unscaled: the running
    // maximum is taken on them and scaled once, and scale and maximum enter the exponent in one fma.
    const bool raw = mk == nullptr && sc > 0.f;
    if (mk != nullptr) {                       // uniform branch: additive key mask (in log2 units)
      float mv[2][16];
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + sb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
          mv[sb][r] = key < a.S ? mk[key] : 0.f;
        }
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[sb][r] = fmaf(s_acc[sb][r], sc, mv[sb][r] * kLog2e);
    } else if (!raw) {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[sb][r] *= sc;
    }
    if (j0 + kAttnKB > a.S) {                  // uniform: only the last block has keys past the end
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + sb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
          s_acc[sb][r] = key < a.S ? s_acc[sb][r] : -3.0e38f;      // stays the minimum under a positive scale
        }
    }
    float mloc = -3.0e38f;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s_acc[sb][r]);
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, kWave));
    if (raw) mloc = fmaxf(mloc * sc, -3.0e38f);
    const float mnew = fmaxf(mrun, mloc);
    const float corr = __builtin_amdgcn_exp2f(mrun - mnew);
    mrun = mnew;
    float psum = 0.f;
    bf16x8_t pf[2][2];                         // [sb][16-key step]
    const float esc = raw ? sc : 1.0f;         // exponent = s * esc - mnew
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s_acc[sb][8 * st + 2 * e], esc, -mnew));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s_acc[sb][8 * st + 2 * e + 1], esc, -mnew));
          w[e] = pack_bf16x2(p0, p1);
          psum += p0 + p1;                     // fp32 sum of the unrounded weights
        }
        uint4 v = make_uint4(w[0], w[1], w[2], w[3]);
        pf[sb][st] = __builtin_bit_cast(bf16x8_t, v);
      }
    lrun = lrun * corr + psum;
#pragma unroll
    for (int tb = 0; tb < kAttnD / 32; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[tb][r] *= corr;

    // ---- O^T += V^T P^T.  Step (sb, st): k-slots 0-3 are keys 32 sb + 16 st + 4 half + 0..3, slots 4-7 the
    // same + 8.  In a 16-lane group, lane i points at key row (i / 4), features 4 (i % 4) .. + 3 of the
    // 4 x 16 block and receives the 4 keys of feature i.
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int tb = 0; tb < kAttnD / 32; ++tb) {
          const lds_bf16_t* vp = Vc + (sb * 32 + st * 16 + 4 * half + l16 / 4) * kAttnVPitch + tb * 32 +
                                 ((lane / 16) % 2) * 16 + (l16 % 4) * 4;
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)vp);
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(vp + 8 * kAttnVPitch));
          const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o_acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, both), pf[sb][st],
                                                              o_acc[tb], 0, 0, 0);
        }
    if (blk + 1 < nblk) commit(cur ^ 1);
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
        v.x = pack_bf16x2(o_acc[tb][4 * rg] * inv, o_acc[tb][4 * rg + 1] * inv);
        v.y = pack_bf16x2(o_acc[tb][4 * rg + 2] * inv, o_acc[tb][4 * rg + 3] * inv);
        *reinterpret_cast<uint2*>(Op + tb * 32 + 8 * rg + 4 * half) = v;
      }
  }
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel of the relative-position attention for head dimension 64: attention_mfma_d64_kernel with
// the position term.  For a wave's 32 queries i0.. and a 32-key sub-block j0.. the positions S - i + j span
// 63 consecutive rows of Kr starting at S - i0 + j0 - 31, so the term is computed as a dense 32 x 64 "band"
// product RAW[o][i] = q_i . kr[base + o] on the matrix pipe (two more accumulators per sub-block) and the
// diagonal bd[i][j] = RAW[(j - j0) - (i - i0) + 31][i] is picked out through a wave-private LDS tile (row =
// query, pitch 66 floats: both the writes by position and the skewed reads by key are spread over the banks).
// The query biases enter exactly, as two fp32 vectors per key block: c_j = bias_w . k_j per key and
// e_p = bias_r . kr[p] per position, ((q + b) . k = q . k + b . k), one dot product per thread.
// Workgroup = 128 queries of one (model, sequence, head); per key block of 64 keys it stages the 64 K and V
// rows and the 192 Kr rows its four waves' bands cover (rows outside [0, 2S) are zero: they only meet
// query/key pairs past the end).  One workgroup per CU (130 KB of LDS).
// ------------------------------------------------------------------------------------------
constexpr int kRelBand = 192;                              // Kr rows per (query block, key block)
constexpr int kRelXPitch = 66;
constexpr int kRelOffK = 0;
constexpr int kRelOffV = kRelOffK + 2 * kAttnKB * kAttnKPitch * 2;
constexpr int kRelOffR = kRelOffV + 2 * kAttnKB * kAttnVPitch * 2;
constexpr int kRelOffX = kRelOffR + 2 * kRelBand * kAttnKPitch * 2;
constexpr int kRelOffC = kRelOffX + 4 * 32 * kRelXPitch * 4;
constexpr int kRelOffE = kRelOffC + kAttnKB * 4;
constexpr int kRelLdsBytes = kRelOffE + kRelBand * 4;

__global__ __launch_bounds__(256) void attention_relpos_mfma_d64_kernel(AttnRelArgs ra, int qblocks) {
  const AttnArgs& a = ra.a;
  extern __shared__ __align__(16) unsigned char rel_smem[];
  lds_bf16_t* const Ks = (lds_bf16_t*)(rel_smem + kRelOffK);
  lds_bf16_t* const Vs = (lds_bf16_t*)(rel_smem + kRelOffV);
  lds_bf16_t* const Rs = (lds_bf16_t*)(rel_smem + kRelOffR);
  lds_f32_t* const Xs = (lds_f32_t*)(rel_smem + kRelOffX);
  lds_f32_t* const Cs = (lds_f32_t*)(rel_smem + kRelOffC);
  lds_f32_t* const Es = (lds_f32_t*)(rel_smem + kRelOffE);
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int half = lane / 32, lq = lane % 32, l16 = lane % 16;
  unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  const int qb = id % qblocks;  id /= qblocks;
  const int h = id % a.heads;   id /= a.heads;
  const int b = id % a.B;
  const int m = id / a.B;
  const long hd = (long)a.heads * kAttnD;
  const long head_off = (long)m * a.stride_m + ((long)b * a.S) * a.stride_row + (long)h * kAttnD;
  const bf16_t* Qp = (const bf16_t*)a.Q + head_off;
  const bf16_t* Kp = (const bf16_t*)a.K + head_off;
  const bf16_t* Vp = (const bf16_t*)a.V + head_off;
  const bf16_t* Rp = (const bf16_t*)ra.Kr + (long)m * 2 * a.S * hd + (long)h * kAttnD;     // row p at + p * hd
  const float* bw = ra.bias_w ? ra.bias_w + m * hd + h * kAttnD : nullptr;
  const float* br = ra.bias_r ? ra.bias_r + m * hd + h * kAttnD : nullptr;
  const float* mk = a.mask ? a.mask + ((long)m * a.B + b) * a.S : nullptr;
  const float kLog2e = 1.4426950408889634f;
  const float sc = a.scale * kLog2e;

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
  float mrun = -3.0e38f, lrun = 0.f;

  // staging: 64 K rows, 64 V rows (2 chunks of 16 bytes per thread each) and 192 Kr rows (6 chunks per thread)
  uint4 kreg[2], vreg[2], rreg[6];
  auto fetch = [&](int j0) {
    const int p0 = a.S - qb * 128 - 127 + j0;             // Kr row of band row 0
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int c = tid + t * 256, key = c / 8, kc = (c % 8) * 8;
      kreg[t] = vreg[t] = make_uint4(0, 0, 0, 0);
      if (j0 + key < a.S) {
        kreg[t] = *reinterpret_cast<const uint4*>(Kp + (long)(j0 + key) * a.stride_row + kc);
        vreg[t] = *reinterpret_cast<const uint4*>(Vp + (long)(j0 + key) * a.stride_row + kc);
      }
    }
#pragma unroll
    for (int t = 0; t < 6; ++t) {
      const int c = tid + t * 256, row = c / 8, kc = (c % 8) * 8;
      const int p = p0 + row;
      rreg[t] = make_uint4(0, 0, 0, 0);
      if (p >= 0 && p < 2 * a.S) rreg[t] = *reinterpret_cast<const uint4*>(Rp + (long)p * hd + kc);
    }
  };
  auto commit = [&](int stage) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int c = tid + t * 256, key = c / 8, kc = (c % 8) * 8;
      lds_store16(Ks + stage * kAttnKB * kAttnKPitch + key * kAttnKPitch + kc, kreg[t]);
      lds_store16(Vs + stage * kAttnKB * kAttnVPitch + key * kAttnVPitch + kc, vreg[t]);
    }
#pragma unroll
    for (int t = 0; t < 6; ++t) {
      const int c = tid + t * 256, row = c / 8, kc = (c % 8) * 8;
      lds_store16(Rs + stage * kRelBand * kAttnKPitch + row * kAttnKPitch + kc, rreg[t]);
    }
  };
  fetch(0);
  commit(0);
  __syncthreads();

  lds_f32_t* const Xw = Xs + wave * 32 * kRelXPitch;       // this wave's exchange tile [query][position offset]
  const int nblk = (a.S + kAttnKB - 1) / kAttnKB;
  for (int blk = 0; blk < nblk; ++blk) {
    const int j0 = blk * kAttnKB, cur = blk & 1;
    if (blk + 1 < nblk) fetch(j0 + kAttnKB);
    const lds_bf16_t* Kc = Ks + cur * kAttnKB * kAttnKPitch;
    const lds_bf16_t* Vc = Vs + cur * kAttnKB * kAttnVPitch;
    const lds_bf16_t* Rc = Rs + cur * kRelBand * kAttnKPitch;

    // ---- the bias terms of this block: thread t < 64: c_t = bias_w . k_t; thread 64 + r: e_r = bias_r . kr[band row r]
    {
      const bool is_key = tid < kAttnKB;
      const lds_bf16_t* row = is_key ? Kc + tid * kAttnKPitch : Rc + (tid - kAttnKB) * kAttnKPitch;
      const float* bias = is_key ? bw : br;
      float dot = 0.f;
      if (bias != nullptr) {
#pragma unroll
        for (int c8 = 0; c8 < kAttnD / 8; ++c8) {
          const u32x4_t v = *(const lds_u32x4_t*)(row + c8 * 8);
          const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            dot = fmaf(bias[c8 * 8 + 2 * e], __uint_as_float(w[e] << 16), dot);
            dot = fmaf(bias[c8 * 8 + 2 * e + 1], __uint_as_float(w[e] & 0xffff0000u), dot);
          }
        }
      }
      if (is_key) Cs[tid] = dot; else Es[tid - kAttnKB] = dot;
    }
    __syncthreads();

    // ---- content scores, transposed (as attention_mfma_d64_kernel)
    f32x16_t s_acc[2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s_acc[sb][r] = 0.f;
    {
      bf16x8_t kf[kAttnD / 16][2];
#pragma unroll
      for (int kk = 0; kk < kAttnD / 16; ++kk)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
          kf[kk][sb] = *(const lds_bf16x8_t*)(Kc + (sb * 32 + lq) * kAttnKPitch + kk * 16 + half * 8);
#pragma unroll
      for (int kk = 0; kk < kAttnD / 16; ++kk)
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
          s_acc[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk][sb], qf[kk], s_acc[sb], 0, 0, 0);
    }
    // ---- position term: band product, bias e, skew through the wave's LDS tile
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      const int start = 96 - 32 * wave + 32 * sb;           // band row of position offset 0 for this wave and sub-block
      f32x16_t rb[2];
#pragma unroll
      for (int ob = 0; ob < 2; ++ob)
#pragma unroll
        for (int r = 0; r < 16; ++r) rb[ob][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < kAttnD / 16; ++kk)
#pragma unroll
        for (int ob = 0; ob < 2; ++ob) {
          const bf16x8_t rf = *(const lds_bf16x8_t*)(Rc + (start + ob * 32 + lq) * kAttnKPitch + kk * 16 + half * 8);
          rb[ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rf, qf[kk], rb[ob], 0, 0, 0);
        }
      // register r of block ob: position offset o = 32 ob + 8 (r/4) + 4 half + r%4, query lq
#pragma unroll
      for (int ob = 0; ob < 2; ++ob)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int o = 32 * ob + 8 * (r / 4) + 4 * half + (r % 4);
          Xw[lq * kRelXPitch + o] = rb[ob][r] + Es[start + o];
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int jj = 8 * (r / 4) + 4 * half + (r % 4);    // key within the sub-block
        s_acc[sb][r] += Xw[lq * kRelXPitch + jj - lq + 31] + Cs[sb * 32 + jj];
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();                      // the tile is rewritten for the next sub-block
    }

    if (mk != nullptr) {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + sb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
          s_acc[sb][r] = fmaf(s_acc[sb][r], sc, (key < a.S ? mk[key] : 0.f) * kLog2e);
        }
    } else {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[sb][r] *= sc;
    }
    if (j0 + kAttnKB > a.S) {
#pragma unroll
      for (int sb = 0; sb < 2; ++sb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = j0 + sb * 32 + 8 * (r / 4) + 4 * half + (r % 4);
          s_acc[sb][r] = key < a.S ? s_acc[sb][r] : -3.0e38f;
        }
    }
    float mloc = -3.0e38f;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s_acc[sb][r]);
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, kWave));
    const float mnew = fmaxf(mrun, mloc);
    const float corr = __builtin_amdgcn_exp2f(mrun - mnew);
    mrun = mnew;
    float psum = 0.f;
    bf16x8_t pf[2][2];
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(s_acc[sb][8 * st + 2 * e] - mnew);
          const float p1 = __builtin_amdgcn_exp2f(s_acc[sb][8 * st + 2 * e + 1] - mnew);
          w[e] = pack_bf16x2(p0, p1);
          psum += p0 + p1;
        }
        uint4 v = make_uint4(w[0], w[1], w[2], w[3]);
        pf[sb][st] = __builtin_bit_cast(bf16x8_t, v);
      }
    lrun = lrun * corr + psum;
#pragma unroll
    for (int tb = 0; tb < kAttnD / 32; ++tb)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[tb][r] *= corr;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int tb = 0; tb < kAttnD / 32; ++tb) {
          const lds_bf16_t* vp = Vc + (sb * 32 + st * 16 + 4 * half + l16 / 4) * kAttnVPitch + tb * 32 +
                                 ((lane / 16) % 2) * 16 + (l16 % 4) * 4;
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)vp);
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(vp + 8 * kAttnVPitch));
          const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o_acc[tb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, both), pf[sb][st],
                                                              o_acc[tb], 0, 0, 0);
        }
    if (blk + 1 < nblk) commit(cur ^ 1);
    __syncthreads();
  }

  const float ltot = lrun + __shfl_xor(lrun, 32, kWave);
  if (q < a.S) {
    const float inv = 1.0f / ltot;
    bf16_t* Op = (bf16_t*)a.O + (((long)m * a.B + b) * a.S + q) * hd + (long)h * kAttnD;
#pragma unroll
    for (int tb = 0; tb < kAttnD / 32; ++tb)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        uint2 v;
        v.x = pack_bf16x2(o_acc[tb][4 * rg] * inv, o_acc[tb][4 * rg + 1] * inv);
        v.y = pack_bf16x2(o_acc[tb][4 * rg + 2] * inv, o_acc[tb][4 * rg + 3] * inv);
        *reinterpret_cast<uint2*>(Op + tb * 32 + 8 * rg + 4 * half) = v;
      }
  }
}

}  // namespace nf
