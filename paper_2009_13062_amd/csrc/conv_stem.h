// Merged 7x7 / stride 2 / pad 3 convolution over a few input channels (the ResNet / ResNeXt stem;
// Section 3.1 "Convolution": M models = M groups of CIN input channels each), bf16, as an implicit
// GEMM with the input patch in LDS.
//
//   C[co][p] = sum_{ci,ky,kx} w[co][ci][ky][kx] * xpad[ci][2 oy + ky][2 ox + kx],   p = oy*Wo + ox
//
// With so few channels the k dimension is ordered for the B (activation) side: the 8 k-slots that one
// lane feeds into an MFMA step are ONE patch row segment, slot j = tap kx = j - 1 of row (ci, ky) (slot 0
// carries a zero weight).  Image column ix lives at patch column ix + 8, so the segment of output
// column ox starts at patch column 2 ox + 4: 16 contiguous bytes at a 4-byte aligned LDS address, read
// as dwords instead of eight 2-byte gathers.  The two lane halves take rows 2 s and 2 s + 1 of the
// CIN * 7 (ci, ky) rows in step s.  The weights are scattered into that order when they are copied
// to LDS (a few thousand elements per workgroup), which costs nothing next to the gathers saved.
//
// One workgroup = one (image, model, 128 consecutive output positions) and up to 64 output channels;
// the whole k extent is staged at once.  Accumulators and the fused epilogue (folded batch norm
// scale/shift, residual, ReLU) are those of gemm_mfma.h.
#pragma once
#include "gemm_mfma.h"

namespace nf {

struct ConvStemArgs {
  const bf16_t* x; const bf16_t* w; const bf16_t* R; bf16_t* y;
  int cog, nG, H, W, Ho, Wo, HoWo;
  int PW, PS;                 // patch row pitch and plane pitch (elements, multiples of 8)
  int cpr;                    // 8-pixel chunks per image row (W / 8)
  int tiles_m, tiles_n;
  long x_group, x_image, y_group, y_image;   // element strides
  Epilogue ep;
};

template <int CIN>
struct ConvStemCfg {
  static constexpr int kKH = 7, kKW = 7, kStride = 2, kPad = 3, kColPad = 8;
  static constexpr int kBM = 64, kBN = 128, kWGM = 1, kWGN = 4, kThreads = 256;
  static constexpr int WM = 64, WN = 32, FM = 2, FN = 1;
  static constexpr bool kRowConsts = true;
  static constexpr int kRows = CIN * kKH;                 // (ci, ky) rows of the k dimension
  static constexpr int kSteps = (kRows + 1) / 2;          // MFMA steps of 16 k: two rows each
  static constexpr int kK = kSteps * 16;                  // padded k extent in LDS
  static constexpr int kAPitch = kK + 8;                  // elements; (pitch / 8) odd -> 16-byte slots rotate
  static_assert((kAPitch / 8) % 2 == 1, "A pitch must rotate bank groups");
  static constexpr int kABytes = kBM * kAPitch * 2;
  static constexpr int kEpiPitch = kBN + 4;
  static constexpr int kLdsEpi = kWGM * 32 * kEpiPitch * (int)sizeof(float);
  static constexpr int lds_bytes(int PS) {
    const int pipe = kABytes + CIN * PS * 2;
    return pipe > kLdsEpi ? pipe : kLdsEpi;
  }
};

template <class Cfg, int CIN>
__global__ __launch_bounds__(256) void conv_stem_kernel(ConvStemArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  lds_bf16_t* As = (lds_bf16_t*)smem_raw;
  lds_bf16_t* Ps = As + Cfg::kBM * Cfg::kAPitch;
  constexpr int FM = Cfg::FM, KHW = Cfg::kKH * Cfg::kKW, KW = Cfg::kKW;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
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
  const int PH = (p_last / a.Wo - oy_first) * Cfg::kStride + Cfg::kKH;      // patch rows needed (<= PS / PW)
  const int iy0 = oy_first * Cfg::kStride - Cfg::kPad;
  const bf16_t* xg = a.x + (long)b * a.x_image + (long)G * a.x_group;
  const bf16_t* wg = a.w + ((long)G * a.cog + row0) * (CIN * KHW);

  // ---- zero the weight tile and the patch (padding, slot 0 and the rows past the image stay zero)
  constexpr int kLdsEls = Cfg::kBM * Cfg::kAPitch;
  for (int c = tid; c < (kLdsEls + CIN * a.PS) / 8; c += 256) lds_store16(As + c * 8, make_uint4(0, 0, 0, 0));
  __syncthreads();

  // ---- weights: natural (co, ci, ky, kx) order in memory -> LDS column (ci*7 + ky)*8 + 1 + kx of row co.
  // Task = the 7 taps of one (co, ci, ky): contiguous in memory at element 7 * task (any 2-byte alignment),
  // contiguous in LDS behind the zero slot; one division per task.
  {
    const int ntask = min(rows_left, Cfg::kBM) * Cfg::kRows;
    for (int task = tid; task < ntask; task += 256) {
      const int co = task / Cfg::kRows, r = task - co * Cfg::kRows;      // r = ci*7 + ky
      const bf16_t* src = wg + task * KW;
      lds_bf16_t* dst = As + co * Cfg::kAPitch + r * 8 + 1;
      bf16_t v[KW];
#pragma unroll
      for (int kx = 0; kx < KW; ++kx) v[kx] = src[kx];
#pragma unroll
      for (int kx = 0; kx < KW; ++kx) dst[kx] = v[kx];
    }
  }
  // ---- patch: 8-pixel chunks, aligned on both sides.  32 lanes run along a patch row (chunk index), the 8
  // lane groups of the workgroup take 8 rows at a time: no division anywhere (row -> (channel, patch row) by
  // comparison, CIN being tiny).
  {
    const int nrows = CIN * PH;
    for (int row = tid / 32; row < nrows; row += 8) {
      int ci = 0;
#pragma unroll
      for (int c = 1; c < CIN; ++c) ci += row >= c * PH;
      const int py = row - ci * PH, iy = iy0 + py;
      if (iy < 0 || iy >= a.H) continue;
      const bf16_t* src = xg + ((long)ci * a.H + iy) * a.W;
      lds_bf16_t* dst = Ps + ci * a.PS + py * a.PW + Cfg::kColPad;
      for (int ch = tid % 32; ch < a.cpr; ch += 32) lds_store16(dst + ch * 8, *reinterpret_cast<const uint4*>(src + ch * 8));
    }
  }
  __syncthreads();

  // ---- per-lane gather base: patch offset of this lane's output position (clamped: columns past the
  // end are discarded by the epilogue)
  const int p = min(p0 + wave * Cfg::WN + l32, p_last);
  const int oy = p / a.Wo, ox = p - oy * a.Wo;
  const int pix = ((oy - oy_first) * Cfg::kStride) * a.PW + ox * Cfg::kStride + (Cfg::kColPad - Cfg::kPad - 1);
  const int a_off = l32 * Cfg::kAPitch + half * 8;

  f32x16_t acc[FM][1];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][0][r] = 0.f;

  typedef __attribute__((address_space(3))) const uint32_t lds_cu32_t;
#pragma unroll
  for (int s = 0; s < Cfg::kSteps; ++s) {
    // rows 2s (lower lane half) and 2s+1 (upper half); offsets are wave uniform, the choice is per lane
    constexpr int kRows = Cfg::kRows;
    const int r0 = 2 * s, r1 = 2 * s + 1 < kRows ? 2 * s + 1 : 2 * s;     // a missing last row re-reads row r0 (zero weights)
    const int off0 = (r0 / Cfg::kKH) * a.PS + (r0 % Cfg::kKH) * a.PW;
    const int off1 = (r1 / Cfg::kKH) * a.PS + (r1 % Cfg::kKH) * a.PW;
    lds_cu32_t* src = (lds_cu32_t*)(Ps + pix + (half ? off1 : off0));       // even element index: 4-byte aligned
    uint32_t w0 = src[0], w1 = src[1], w2 = src[2], w3 = src[3];
    w0 &= 0xffff0000u;                                                     // slot 0 multiplies a zero weight: keep it finite
    if (2 * s + 1 >= kRows && half) { w0 = 0; w1 = 0; w2 = 0; w3 = 0; }
    const uint4 v = make_uint4(w0, w1, w2, w3);
    const bf16x8_t bfr = __builtin_bit_cast(bf16x8_t, v);
    bf16x8_t af[FM];
#pragma unroll
    for (int i = 0; i < FM; ++i) af[i] = *(const lds_bf16x8_t*)(As + a_off + i * 32 * Cfg::kAPitch + s * 16);
#pragma unroll
    for (int i = 0; i < FM; ++i)
      acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af[i], acc[i][0], 0, 0, 0);
  }
  __syncthreads();     // every wave is done with the operands before the epilogue reuses LDS

  const long coff = (long)b * a.y_image + (long)G * a.y_group + (long)row0 * a.HoWo + p0;
  const long rvo = (long)G * a.cog + row0;
  gemm_epilogue<Cfg>(acc, (lds_f32_t*)smem_raw, a.y + coff, a.R ? a.R + coff : nullptr, a.HoWo, rows_left, cols_left,
                     a.ep, rvo, 0);
}

}  // namespace nf
