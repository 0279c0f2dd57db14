// Instantiation and launch of the tap-major 3x3 convolution kernels (conv_tap.h, bf16).
#include <atomic>
#include <cstdlib>

#include "conv_tap.h"
#include "gemm_launch.h"

namespace nf {

template <class Cfg, int VW, int NT, bool FUSED>
static nf_status launch_tap_kernel(long long total, int lds, const ConvPatchArgs& a, hipStream_t s) {
  auto kern = conv_tap_kernel<Cfg, VW, NT, FUSED>;
  if (lds > 64 * 1024) {
    static std::atomic<bool> opted_in{false};        // per kernel: idempotent, a benign race
    if (!opted_in.load(std::memory_order_acquire)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              160 * 1024) != hipSuccess)
        return NF_ELAUNCH;
      opted_in.store(true, std::memory_order_release);
    }
  }
  nf_launch(kern, dim3((unsigned)total), dim3(256), lds, s, a);
  return hipGetLastError() == hipSuccess ? NF_OK : NF_ELAUNCH;
}

template <class Cfg, bool FUSED = false>
static nf_status launch_tap(ConvPatchArgs& a, int B, hipStream_t s) {
  a.tiles_m = (a.cog + Cfg::kBM - 1) / Cfg::kBM;
  a.tiles_n = (a.HoWo + Cfg::kBN - 1) / Cfg::kBN;
  const long long total = (long long)a.tiles_m * a.tiles_n * a.nG * B;
  if (total <= 0 || total > 0x7fffffffLL) return NF_EUNSUPPORTED;
  a.PS = (a.PS + 7) / 8 * 8;
  const long long tasks = (long long)(kTapCB / 8) * (a.PS / a.PW) * a.cpr;     // patch tasks of the tallest tile
  const int nt = (int)((tasks + 255) / 256);
  const int lds = Cfg::lds_bytes(a.PS);
  if (lds > 160 * 1024) return NF_EUNSUPPORTED;
#define NF_TAP(VW_, NT_) return launch_tap_kernel<Cfg, VW_, NT_, FUSED>(total, lds, a, s)
  switch (a.VW) {
    case 8: if (nt == 1) NF_TAP(8, 1); if (nt == 2) NF_TAP(8, 2); break;     // 32 staging registers per task
    case 4: if (nt == 1) NF_TAP(4, 1); if (nt == 2) NF_TAP(4, 2); if (nt == 3) NF_TAP(4, 3); break;
    case 2: if (nt == 1) NF_TAP(2, 1); if (nt == 2) NF_TAP(2, 2); if (nt == 3) NF_TAP(2, 3); break;
    case 1: if (nt == 1) NF_TAP(1, 1); if (nt == 2) NF_TAP(1, 2); if (nt == 3) NF_TAP(1, 3); break;
  }
#undef NF_TAP
  return NF_EUNSUPPORTED;
}

// 3x3, dilation 1, pad <= kLPad, (fused) groups of 32 k channels.  The caller has filled everything but the
// tiling.  NF_EUNSUPPORTED = take another kernel.
nf_status launch_conv_tap_3x3(ConvPatchArgs& a, int B, hipStream_t s) {
  if (a.cig % kTapCB != 0 || ((uintptr_t)a.x & 15) != 0) return NF_EUNSUPPORTED;
  if (a.S > 1) {
    // fused narrow groups: one 32-channel block, at most 32 rows; weight runs are read 16 or 8 bytes at a time
    if (a.cig != kTapCB || a.cog > 32 || a.cig_real * a.S != kTapCB || a.cog_real * a.S != a.cog) return NF_EUNSUPPORTED;
    if (((uintptr_t)a.w & (a.cig_real >= 8 ? 15 : 7)) != 0) return NF_EUNSUPPORTED;
    ConvPatchArgs f = a;
    if (a.stride == 1) {
      const int rows = a.PS / a.PW;
      f.PW = a.PW + ((a.Wo - a.PW) % 16 + 16) % 16;       // see below
      f.PS = rows * f.PW;
    }
    return launch_tap<ConvTapCfg<32, 1, 4, 2>, true>(f, B, s);
  }
  if (((uintptr_t)a.w & 15) != 0) return NF_EUNSUPPORTED;
  static const int forced_bm = [] { const char* e = dev_getenv("NETFUSE_TAP_BM"); return e ? atoi(e) : 0; }();
  const long long per_row_tile = (long long)((a.HoWo + 127) / 128) * a.nG * B;
  auto tiles = [&](int bm) { return per_row_tile * ((a.cog + bm - 1) / bm); };
  // measured on the 3x3 layers of ResNet-50 at 32 merged models: a taller row tile copies the input patch
  // less often, which pays from about 400 workgroups up; stride 2 (four times the patch per output) prefers
  // it earlier, unless most of the 128 positions of a tile are padding (7x7 outputs)
  int bm = 32;
  if (a.cog > 64 && a.stride > 1 && tiles(128) >= 200) bm = 128;
  else if (a.cog > 32 && (tiles(64) >= 400 || (a.stride > 1 && a.HoWo >= 128 && tiles(64) >= 256))) bm = 64;
  if (forced_bm == 32 || forced_bm == 64 || forced_bm == 128) bm = forced_bm;
  ConvPatchArgs c = a;                                  // the caller's copy stays intact for a fallback
  if (a.stride == 1) {
    // 16 consecutive lanes read 16 consecutive output positions; their pixels are consecutive within an
    // output row and PW - Wo + 1 apart across a row end.  With the 80-byte pixel pitch, 16 pixels whose
    // indices are distinct modulo 16 hit 16 distinct bank groups, so a row pitch congruent to Wo modulo
    // 16 keeps the reads conflict free across row ends (measured: a third of the LDS cycles on 14x14 images
    // were bank conflicts without it).
    const int rows = a.PS / a.PW;
    c.PW = a.PW + ((a.Wo - a.PW) % 16 + 16) % 16;
    c.PS = rows * c.PW;
  }
  if (bm == 128) return launch_tap<ConvTapCfg<128, 2, 2, 1>>(c, B, s);
  if (bm == 64) return launch_tap<ConvTapCfg<64, 1, 4, 2>>(c, B, s);
  return launch_tap<ConvTapCfg<32, 1, 4, 2>>(c, B, s);
}

}  // namespace nf
