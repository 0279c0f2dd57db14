// Merged 3 x 3 convolution (grouped, groups = M*g: Appendix A Eq. 2) over groups of 32 k input channels,
// bf16, as an implicit GEMM that reads BOTH MFMA operands with one aligned 16-byte LDS read per fragment.
//
//   C[co][p] = sum_{ci,ky,kx} w[co][ci][ky][kx] * xpad[ci][oy*s + ky][ox*s + kx],   p = oy*Wo + ox
//
// The k dimension of a block of 32 input channels is ordered tap-major: MFMA step (tap, g) covers channels
// 16 g .. 16 g + 15 of the block at tap (ky, kx), lane half h taking channels 16 g + 8 h .. + 7.  Both LDS
// tiles are laid out for that order while they are filled:
//   * the input patch of the tile's 128 output positions is kept channel-innermost, pixel (py, px) at
//     (py*PW + px) * 80 bytes holding its 32 channels (the 16 bytes of padding make consecutive pixels
//     rotate over the 64 LDS banks), so the 8 channels a lane needs at a tap are 16 contiguous bytes at
//     pixel(position) + tap offset, the offset being uniform over the wavefront;
//   * the weight tile holds row co as [tap][channel], so the A fragment of step (tap, g) is 16 contiguous
//     bytes as well.
// The reordering happens in registers between the global loads and the LDS writes: a weight task takes the
// 72 contiguous elements w[co][8 o .. 8 o + 7][0..8] (nine 16-byte loads) and writes nine 16-byte vectors,
// one per tap; a patch task takes VW pixels of 8 channel planes (eight loads) and writes VW 16-byte
// vectors, one per pixel.  Byte permutes with compile-time selectors do the shuffling.
// (conv_patch.h keeps the planes apart in LDS and gathers each tap of each channel with a 2-byte read:
// eight LDS reads per fragment, which bounds its 3x3 layers on small images.)
//
// The patch carries its zero padding: it is zeroed once, and every channel block overwrites only the
// in-image pixels.  Image column ix lives at patch column ix + kLPad.  One workgroup = one (image, group,
// 128-position tile, BM output channels); accumulators and the fused epilogue are those of gemm_mfma.h.
#pragma once
#include "conv_patch.h"

namespace nf {

constexpr int kTapCB = 32;          // input channels per block
constexpr int kTapPixPitch = 40;    // elements per patch pixel (32 channels + 8)

template <int BM, int WGM, int WGN, int MINW = 1>
struct ConvTapCfg {
  static_assert(WGM * WGN == 4, "4 wavefronts");
  static constexpr int kBM = BM, kBN = 128, kWGM = WGM, kWGN = WGN, kThreads = 256;
  static constexpr int WM = BM / WGM, WN = kBN / WGN, FM = WM / 32, FN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
  static constexpr int kTaps = 9;
  static constexpr bool kRowConsts = true;
  static constexpr int kAPitch = kTaps * kTapCB + 8;     // elements; (pitch / 8) odd -> 16-byte slots rotate
  static_assert((kAPitch / 8) % 2 == 1, "A pitch must rotate bank groups");
  static constexpr int kABytes = BM * kAPitch * 2;
  static constexpr int kEpiPitch = kBN + 4;
  static constexpr int kLdsEpi = WGM * 32 * kEpiPitch * (int)sizeof(float);
  static constexpr int kWTasks = BM * (kTapCB / 8);      // weight tasks per block: (row, channel octet)
  static constexpr int kWPer = (kWTasks + 255) / 256;
  static constexpr int kMinWaves = MINW;
  static constexpr int lds_bytes(int PS) {
    const int pipe = kABytes + PS * kTapPixPitch * 2;
    return pipe > kLdsEpi ? pipe : kLdsEpi;
  }
};

// VW: pixels per patch chunk (= a.VW; VW | W).  NT: patch tasks per thread (the host checks the bound).
// FUSED: S > 1 narrow groups (4, 8 or 16 channels each) share the single 32-channel block: the weight tile
// is block diagonal (row r carries its own group's channels at channel offset (r / cog_real) * cig_real,
// zeros elsewhere), filled once; see conv_patch.h for why no product crosses a group.
template <class Cfg, int VW, int NT, bool FUSED = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(Cfg::kMinWaves))) void conv_tap_kernel(ConvPatchArgs a) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  lds_bf16_t* As = (lds_bf16_t*)smem_raw;
  lds_bf16_t* Ps = As + Cfg::kBM * Cfg::kAPitch;
  constexpr int FM = Cfg::FM, FN = Cfg::FN, CB = kTapCB, PP = kTapPixPitch;
  constexpr int kDw = VW >= 2 ? VW / 2 : 1;            // dwords per loaded chunk
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
  const int PH = (p_last / a.Wo - oy_first) * a.stride + 3;          // rows actually needed (<= PS / PW)
  const int iy0 = oy_first * a.stride - a.pad;
  const bf16_t* xg = a.x + (long)b * a.x_image + (long)G * a.x_group;
  const bf16_t* wg = a.w + ((long)G * a.cog + row0) * a.cig * 9;

  // ---- this thread's share of a channel block.  Weight task = (row, channel octet); patch task = (channel
  // octet, patch row, chunk of VW pixels).  The geometry does not change from block to block.
  int w_off[Cfg::kWPer], w_dst[Cfg::kWPer];                 // w_dst < 0: no such task
#pragma unroll
  for (int t = 0; t < Cfg::kWPer; ++t) {
    const int task = tid + t * 256, r = task / (CB / 8), o = task % (CB / 8);
    const bool live = Cfg::kWTasks % 256 == 0 || task < Cfg::kWTasks;
    w_off[t] = (min(r, rows_left - 1) * a.cig + 8 * o) * 9;  // rows past the end re-read the last one; never stored
    w_dst[t] = live ? r * Cfg::kAPitch + 8 * o : -1;
  }
  // ---- software pipeline over channel blocks: the global loads of block s+1 are in flight in registers
  // while block s is multiplied out of LDS
  uint32_t wv[Cfg::kWPer][36];
  uint32_t pv[NT][8][kDw];
  const long plane = (long)a.H * a.W;
  auto prefetch_w = [&](int ci0) {
#pragma unroll
    for (int t = 0; t < Cfg::kWPer; ++t) {
      if (FUSED || w_dst[t] < 0) continue;
      const bf16_t* p = wg + w_off[t] + (long)ci0 * 9;
#pragma unroll
      for (int q = 0; q < 9; ++q) {
        const uint4 v = *reinterpret_cast<const uint4*>(p + q * 8);
        wv[t][4 * q] = v.x; wv[t][4 * q + 1] = v.y; wv[t][4 * q + 2] = v.z; wv[t][4 * q + 3] = v.w;
      }
    }
  };
  // The first block's weights are requested before anything else: the index arithmetic below (a handful of
  // integer divisions per lane) and the zero fill of the patch then run under their trip from HBM instead of in
  // front of it (measured: 2.8 us from the start of a workgroup to its first load otherwise).
  prefetch_w(0);


  // ---- fragment addresses (elements): per-lane base + wave-uniform (tap, channel group) offset
  int b_off[FN];
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int p = min(p0 + wn * Cfg::WN + j * 32 + l32, p_last);     // clamp: columns past the end are discarded
    const int oy = p / a.Wo, ox = p - oy * a.Wo;
    b_off[j] = (((oy - oy_first) * a.stride) * a.PW + ox * a.stride + (kLPad - a.pad)) * PP + half * 8;
  }
  const int a_off = (wm * Cfg::WM + l32) * Cfg::kAPitch + half * 8;

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  int g_off[NT], l_off[NT];                                 // g_off < 0: nothing to copy
  {
    const int ntasks = (CB / 8) * PH * a.cpr;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      const int task = tid + u * 256;
      const int rest = task / a.cpr, ch = task - rest * a.cpr;
      const int o = rest / PH, py = rest - o * PH;
      const int iy = iy0 + py;
      const bool live = task < ntasks && iy >= 0 && iy < a.H;
      g_off[u] = live ? (8 * o * a.H + iy) * a.W + ch * VW : -1;
      l_off[u] = (py * a.PW + kLPad + ch * VW) * PP + 8 * o;
    }
  }
  // zero the whole patch once: padding and out-of-image rows are never written again
  for (int c = tid; c < a.PS * PP / 8; c += 256) lds_store16(Ps + c * 8, make_uint4(0, 0, 0, 0));

  auto prefetch_x = [&](int ci0) {
    const bf16_t* xc = xg + (long)ci0 * plane;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      if (g_off[u] < 0) continue;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        const bf16_t* p = xc + g_off[u] + c * plane;
        if constexpr (VW == 8) {
          const uint4 v = *reinterpret_cast<const uint4*>(p);
          pv[u][c][0] = v.x; pv[u][c][1] = v.y; pv[u][c][2] = v.z; pv[u][c][3] = v.w;
        } else if constexpr (VW == 4) {
          const uint2 v = *reinterpret_cast<const uint2*>(p);
          pv[u][c][0] = v.x; pv[u][c][1] = v.y;
        } else if constexpr (VW == 2) {
          pv[u][c][0] = *reinterpret_cast<const uint32_t*>(p);
        } else {
          pv[u][c][0] = *p;
        }
      }
    }
  };
  auto prefetch = [&](int ci0) {
    prefetch_w(ci0);
    prefetch_x(ci0);
  };
  // selectors of perm(hi, lo, sel): 16 bits of `lo` (its low or high half) below 16 bits of `hi`
  auto pick = [](int lo_half, int hi_half) -> uint32_t {
    return (lo_half ? 0x0302u : 0x0100u) | ((hi_half ? 0x0706u : 0x0504u) << 16);
  };
  auto commit = [&]() {
#pragma unroll
    for (int t = 0; t < Cfg::kWPer; ++t) {
      if (FUSED || w_dst[t] < 0) continue;
#pragma unroll
      for (int tap = 0; tap < 9; ++tap) {
        uint32_t o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int e0 = 9 * (2 * q) + tap, e1 = 9 * (2 * q + 1) + tap;     // elements (channel 2q, tap), (channel 2q+1, tap)
          o[q] = __builtin_amdgcn_perm(wv[t][e1 / 2], wv[t][e0 / 2], pick(e0 % 2, e1 % 2));
        }
        lds_store16(As + w_dst[t] + tap * CB, make_uint4(o[0], o[1], o[2], o[3]));
      }
    }
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      if (g_off[u] < 0) continue;
#pragma unroll
      for (int i = 0; i < VW; ++i) {
        uint32_t o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
          o[q] = __builtin_amdgcn_perm(pv[u][2 * q + 1][i / 2], pv[u][2 * q][i / 2], pick(i % 2, i % 2));
        lds_store16(Ps + l_off[u] + i * PP, make_uint4(o[0], o[1], o[2], o[3]));
      }
    }
  };

  prefetch_x(0);
  if constexpr (FUSED) {
    for (int c = tid; c < Cfg::kBM * Cfg::kAPitch / 8; c += 256) lds_store16(As + c * 8, make_uint4(0, 0, 0, 0));
    __syncthreads();
    // task = (row, run of cw = 8 or 4 channels of the row's group): 9*cw contiguous weights, written as one
    // vector of cw channels per tap
    const int cw = a.cig_real >= 8 ? 8 : 4, subs = a.cig_real / cw;
    const bf16_t* ws = a.w + (long)G * a.cog * a.cig_real * 9;       // fused group G: rows G*cog .. of the weight tensor
    for (int task = tid; task < a.cog * subs; task += 256) {
      const int r = task / subs, sub = task - r * subs;
      const bf16_t* p = ws + ((long)r * a.cig_real + sub * cw) * 9;
      lds_bf16_t* dst = As + r * Cfg::kAPitch + (r / a.cog_real) * a.cig_real + sub * cw;
      uint32_t d[36];
      if (cw == 8) {
#pragma unroll
        for (int q = 0; q < 9; ++q) {
          const uint4 v = *reinterpret_cast<const uint4*>(p + q * 8);
          d[4 * q] = v.x; d[4 * q + 1] = v.y; d[4 * q + 2] = v.z; d[4 * q + 3] = v.w;
        }
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
          uint32_t o[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int e0 = 9 * (2 * q) + tap, e1 = 9 * (2 * q + 1) + tap;
            o[q] = __builtin_amdgcn_perm(d[e1 / 2], d[e0 / 2], pick(e0 % 2, e1 % 2));
          }
          lds_store16(dst + tap * CB, make_uint4(o[0], o[1], o[2], o[3]));
        }
      } else {
#pragma unroll
        for (int q = 0; q < 9; ++q) {
          const uint2 v = *reinterpret_cast<const uint2*>(p + q * 4);
          d[2 * q] = v.x; d[2 * q + 1] = v.y;
        }
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
          uint32_t o[2];
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int e0 = 9 * (2 * q) + tap, e1 = 9 * (2 * q + 1) + tap;
            o[q] = __builtin_amdgcn_perm(d[e1 / 2], d[e0 / 2], pick(e0 % 2, e1 % 2));
          }
          lds_store8(dst + tap * CB, o[0], o[1]);
        }
      }
    }
  }
  __syncthreads();                                         // the zero fills are complete
  for (int ci0 = 0; ci0 < a.cig; ci0 += CB) {
    commit();
    __syncthreads();
    if (ci0 + CB < a.cig) prefetch(ci0 + CB);
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int tap_off = ((tap / 3) * a.PW + tap % 3) * PP;           // wave-uniform
#pragma unroll
      for (int g = 0; g < CB / 16; ++g) {
        bf16x8_t af[FM], bfr[FN];
#pragma unroll
        for (int i = 0; i < FM; ++i) af[i] = *(const lds_bf16x8_t*)(As + a_off + i * 32 * Cfg::kAPitch + tap * CB + g * 16);
#pragma unroll
        for (int j = 0; j < FN; ++j) bfr[j] = *(const lds_bf16x8_t*)(Ps + b_off[j] + tap_off + g * 16);
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
          for (int j = 0; j < FN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
      }
    }
    __syncthreads();
  }

  const long coff = (long)b * a.y_image + (long)G * a.y_group + (long)row0 * a.HoWo + p0;
  const long rvo = (long)G * a.cog + row0;
  gemm_epilogue<Cfg>(acc, (lds_f32_t*)smem_raw, a.y + coff, a.R ? a.R + coff : nullptr, a.HoWo, rows_left, cols_left,
                     a.ep, rvo, 0);
}

}  // namespace nf
