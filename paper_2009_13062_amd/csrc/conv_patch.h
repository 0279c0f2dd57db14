// Merged k x k convolution (grouped, groups = M*g: Appendix A Eq. 2) as an implicit GEMM whose B
// operand is never materialised: for CB input channels at a time the zero-padded input patch that a
// tile of 128 consecutive output positions needs is copied into LDS once, and every MFMA B fragment
// is gathered from it.
//
//   C[co][p] = sum_{ci,ky,kx} w[co][ci][ky][kx] * xpad[ci][oy*s + ky][ox*s + kx],   p = oy*Wo + ox
//
// A = the group's weight rows, natural (ci, ky, kx) order, copied 16 bytes at a time.  The 16 k of one
// MFMA step are split by lane half: half h takes channels [h*CB/2, (h+1)*CB/2) of the stage, so a
// lane's 8 k-slots in step kk are t = 8 kk .. 8 kk + 7 of its half's (ci, ky, kx) sequence.  On the A
// side that is one aligned 16-byte LDS read; on the B side slot t of a lane at output position
// (oy, ox) is patch[(t / KHW) + h*CB/2][oy*s + (t % KHW) / KW][ox*s + (t % KHW) % KW]: a per-lane base
// plus an offset that is uniform over the wavefront, read with 2-byte LDS loads.  The patch carries
// its zero padding, so the gather needs no bounds checks: it is zeroed once, and every channel block
// then overwrites only the in-image pixels.  Image column ix lives at patch column ix + kLPad (8), so a
// row is copied as W / VW aligned chunks of VW pixels on both the global and the LDS side.
//
// Narrow groups (ResNeXt: 4, 8 or 16 channels per group): S = 32 / cig consecutive groups are fused
// into one 32-channel block whose weight tile is block diagonal (row r of the tile carries the cig*KHW
// weights of its own group at column offset (r / cog)*cig*KHW, zeros elsewhere).  The MFMA then
// multiplies S times more zeros than data, which is free next to the HBM traffic of such layers.  For
// finite inputs the zero blocks contribute exactly 0; a NaN or infinity in one group's input would
// still reach its S - 1 neighbours through 0 * NaN, so the caller fuses groups of ONE model only
// (g % S == 0): isolation BETWEEN MODELS is exact for any input values.
//
// One workgroup = one (image, group, 128-position tile, BM output channels).  Accumulators and the
// fused epilogue (folded batch norm scale/shift, residual, ReLU) are those of gemm_mfma.h.
#pragma once
#include <type_traits>

#include "gemm_mfma.h"

namespace nf {

constexpr int kLPad = 8;     // patch column of image column 0
constexpr int kHalfShiftMax = 64; // see ConvPatchCfg::half_shift

struct ConvPatchArgs {
  const bf16_t* x; const bf16_t* w; const bf16_t* R; bf16_t* y;
  int cig, cog, nG, H, W, Ho, Wo, HoWo, stride, pad;
  int PW, PS;                 // patch row pitch and plane pitch (elements); PS covers the tallest patch
  int VW, cpr;                // patch rows are copied in chunks of VW pixels (VW | W, power of two <= 8); cpr = W / VW
  int S;                      // groups fused per workgroup (see below); 1 = one group per workgroup
  int cig_real, cog_real;     // S > 1: channels of ONE group; cig = S*cig_real, cog = S*cog_real then describe the fused group
  int tiles_m, tiles_n;
  long x_group, x_image, y_group, y_image;   // element strides
  Epilogue ep;
};

// MINW: wavefronts per SIMD the register allocation must allow (workgroups per CU, at 4 waves each)
template <int BM, int KH, int KW, int CB, int WGM, int WGN, int MINW = 1>
struct ConvPatchCfg {
  static_assert(WGM * WGN == 4, "4 wavefronts");
  static constexpr int kBM = BM, kBN = 128, kWGM = WGM, kWGN = WGN, kThreads = 256;
  static constexpr int WM = BM / WGM, WN = kBN / WGN, FM = WM / 32, FN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
  static constexpr int kKHW = KH * KW, kCB = CB, kKH = KH, kKW = KW;
  static constexpr bool kRowConsts = true;
  static constexpr int kStageK = CB * kKHW;            // k extent of one stage
  static constexpr int kHalfK = kStageK / 2;           // per lane half
  static_assert(kHalfK % 8 == 0, "each half must be a whole number of 8-k slots");
  static constexpr int kSteps = kHalfK / 8;            // MFMA steps per stage
  static constexpr int kAPitch = kStageK + 8;          // elements; (pitch/8) odd -> 16-byte slots rotate
  static_assert((kAPitch / 8) % 2 == 1, "A pitch must rotate bank groups");
  static constexpr int kABytes = BM * kAPitch * 2;
  static constexpr int kEpiPitch = kBN + 4;
  static constexpr int kLdsEpi = WGM * 32 * kEpiPitch * (int)sizeof(float);
  static constexpr int kPatchTasksMax = 12 * 256;
  static constexpr int kMinWaves = MINW;
  // Extra elements before the upper half of a block's planes, chosen so that the two lane halves of a
  // gather read addresses 128 bytes apart modulo the 256 bytes of the 64 LDS banks (plane pitches are
  // multiples of 8 elements, so CB/2 planes are a multiple of 128 bytes).
  __host__ __device__ static constexpr int half_shift(int PS) { return ((CB / 2) * PS) % 128 == 0 ? 64 : 0; }
  static_assert(CB % 16 == 0, "half_shift assumes CB/2 planes of 8-element granularity span whole 128-byte units");
  static constexpr int lds_bytes(int PS) {
    const int pipe = kABytes + (CB * PS + kHalfShiftMax) * 2;
    return pipe > kLdsEpi ? pipe : kLdsEpi;
  }
};

// VW: pixels per patch chunk (= a.VW), a compile-time constant so that the copy has no branches and stages a
// chunk in 16, 8 or 4 bytes of registers.
// FUSED: S > 1 narrow groups share the block (block-diagonal weight tile filled once, single channel block).
template <class Cfg, int VW, bool FUSED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(Cfg::kMinWaves))) void conv_patch_kernel(ConvPatchArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  lds_bf16_t* As = (lds_bf16_t*)smem_raw;
  lds_bf16_t* Ps = As + Cfg::kBM * Cfg::kAPitch;
  constexpr int FM = Cfg::FM, FN = Cfg::FN, KHW = Cfg::kKHW, CB = Cfg::kCB;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / Cfg::kWGN, wn = wave % Cfg::kWGN;
  const int half = lane / 32, l32 = lane % 32;

  unsigned id = xcd_remap(blockIdx.x, gridDim.x);
  const int tm = id % a.tiles_m;  id /= a.tiles_m;
  const int tn = id % a.tiles_n;  id /= a.tiles_n;
  const int G = id % a.nG;
  const int b = id / a.nG;
  const int row0 = tm * Cfg::kBM, p0 = tn * Cfg::kBN;
  const int rows_left = a.cog - row0, cols_left = a.HoWo - p0;

  // ---- geometry of this tile's patch
  const int oy_first = p0 / a.Wo;
  const int p_last = min(p0 + Cfg::kBN, a.HoWo) - 1;
  const int PH = (p_last / a.Wo - oy_first) * a.stride + Cfg::kKH;   // rows actually needed (<= PS / PW)
  const int iy0 = oy_first * a.stride - a.pad;
  const bf16_t* xg = a.x + (long)b * a.x_image + (long)G * a.x_group;
  const bf16_t* wg = a.w + ((long)G * a.cog + row0) * a.cig * KHW;        // S == 1: dense rows of cig*KHW weights

  // ---- per-lane gather bases: patch offset of this lane's output position, per column block
  const int hshift = Cfg::half_shift(a.PS);
  int pix[FN];
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int p = min(p0 + wn * Cfg::WN + j * 32 + l32, p_last);     // clamp: columns past the end are discarded
    const int oy = p / a.Wo, ox = p - oy * a.Wo;
    pix[j] = ((oy - oy_first) * a.stride) * a.PW + ox * a.stride + (kLPad - a.pad) + half * ((CB / 2) * a.PS + hshift);
  }
  const int a_off = (wm * Cfg::WM + l32) * Cfg::kAPitch + half * Cfg::kHalfK;

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- this thread's share of a channel block: weight chunks, and patch chunks (one task = VW pixels of
  // one (channel, patch row)); the task geometry does not change from block to block
  constexpr int kCpr = Cfg::kStageK / 8;
  constexpr int kAChunks = Cfg::kBM * kCpr, kAPer = (kAChunks + 255) / 256;
  constexpr int kNT = Cfg::kPatchTasksMax / 256;            // patch tasks per thread (the host checks the bound)
  int g_off[kNT], l_off[kNT];                              // element offsets; g_off < 0: nothing to copy
  {
    const int ntasks = CB * PH * a.cpr;
#pragma unroll
    for (int u = 0; u < kNT; ++u) {
      const int task = tid + u * 256;
      const int row = task / a.cpr, ch = task - row * a.cpr;
      const int ci = row / PH, py = row - ci * PH;
      const int iy = iy0 + py;
      const bool live = task < ntasks && iy >= 0 && iy < a.H;
      g_off[u] = live ? (ci * a.H + iy) * a.W + ch * VW : -1;
      l_off[u] = ci * a.PS + (ci >= CB / 2 ? hshift : 0) + py * a.PW + kLPad + ch * VW;
    }
  }
  // zero the whole patch once: padding and out-of-image rows are never written again
  for (int c = tid; c < (CB * a.PS + kHalfShiftMax) / 8; c += 256) lds_store16(Ps + c * 8, make_uint4(0, 0, 0, 0));

  // ---- software pipeline over channel blocks: the global loads of block s+1 are in flight in
  // registers while block s is multiplied out of LDS
  uint4 va[kAPer];
  typedef typename std::conditional<VW == 8, uint4, typename std::conditional<VW == 4, uint2, uint32_t>::type>::type patch_regs_t;
  patch_regs_t pv[kNT];
  auto prefetch = [&](int ci0) {
#pragma unroll
    for (int t = 0; t < kAPer; ++t) {
      const int c = tid + t * 256, r = c / kCpr, ch = c - r * kCpr;
      va[t] = make_uint4(0, 0, 0, 0);
      if (!FUSED && (kAChunks % 256 == 0 || c < kAChunks) && r < rows_left)
        va[t] = *reinterpret_cast<const uint4*>(wg + ((long)r * a.cig + ci0) * KHW + ch * 8);
    }
    const bf16_t* xc = xg + (long)ci0 * a.H * a.W;
#pragma unroll
    for (int u = 0; u < kNT; ++u) {
      pv[u] = patch_regs_t{};
      if (g_off[u] >= 0) {
        const bf16_t* p = xc + g_off[u];
        if constexpr (VW == 8) pv[u] = *reinterpret_cast<const uint4*>(p);
        else if constexpr (VW == 4) pv[u] = *reinterpret_cast<const uint2*>(p);
        else if constexpr (VW == 2) pv[u] = *reinterpret_cast<const uint32_t*>(p);
        else pv[u] = *p;
      }
    }
  };
  prefetch(0);
  if constexpr (FUSED) {
    // block-diagonal weight tile of S fused groups (single channel block): zero it, then drop each
    // row's cig_real*KHW weights (8-byte chunks) at its group's column offset
    for (int c = tid; c < Cfg::kBM * Cfg::kAPitch / 8; c += 256) lds_store16(As + c * 8, make_uint4(0, 0, 0, 0));
    __syncthreads();
    const int klen = a.cig_real * KHW, cpw = klen / 4;       // weights per row, 4-element chunks per row
    const bf16_t* ws = a.w + (long)G * a.cog * klen;         // fused group G: rows G*cog .. of the weight tensor
    for (int c = tid; c < a.cog * cpw; c += 256) {
      const int r = c / cpw, ch = c - r * cpw;
      const uint2 v = *reinterpret_cast<const uint2*>(ws + (long)r * klen + ch * 4);
      lds_store8(As + r * Cfg::kAPitch + (r / a.cog_real) * klen + ch * 4, v.x, v.y);
    }
  }
  __syncthreads();                                         // the zero fills are complete

  for (int ci0 = 0; ci0 < a.cig; ci0 += CB) {
    // ---- commit the prefetched block to LDS
    if constexpr (!FUSED) {
#pragma unroll
      for (int t = 0; t < kAPer; ++t) {
        const int c = tid + t * 256, r = c / kCpr, ch = c - r * kCpr;
        if (kAChunks % 256 == 0 || c < kAChunks) lds_store16(As + r * Cfg::kAPitch + ch * 8, va[t]);
      }
    }
#pragma unroll
    for (int u = 0; u < kNT; ++u) {
      if (g_off[u] >= 0) {
        lds_bf16_t* d = Ps + l_off[u];
        if constexpr (VW == 8) lds_store16(d, pv[u]);
        else if constexpr (VW == 4) lds_store8(d, pv[u].x, pv[u].y);
        else if constexpr (VW == 2) *(__attribute__((address_space(3))) uint32_t*)d = pv[u];
        else *d = (bf16_t)pv[u];
      }
    }
    __syncthreads();
    if (ci0 + CB < a.cig) prefetch(ci0 + CB);

    // ---- multiply: kSteps MFMA steps of 16 k (8 per lane half)
#pragma unroll
    for (int kk = 0; kk < Cfg::kSteps; ++kk) {
      bf16x8_t af[FM], bfr[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = *(const lds_bf16x8_t*)(As + a_off + i * 32 * Cfg::kAPitch + kk * 8);
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int t = kk * 8 + e;                          // compile-time after unrolling
          const int off = (t / KHW) * a.PS + ((t % KHW) / Cfg::kKW) * a.PW + (t % KHW) % Cfg::kKW;   // wave-uniform
          h[e] = (uint32_t)Ps[pix[j] + off];
        }
        const uint4 v = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        bfr[j] = __builtin_bit_cast(bf16x8_t, v);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  const long coff = (long)b * a.y_image + (long)G * a.y_group + (long)row0 * a.HoWo + p0;
  const long rvo = (long)G * a.cog + row0;
  gemm_epilogue<Cfg>(acc, (lds_f32_t*)smem_raw, a.y + coff, a.R ? a.R + coff : nullptr, a.HoWo, rows_left, cols_left,
                     a.ep, rvo, 0);
}

}  // namespace nf
