// Instantiation and launch of the patch-gather convolution kernels (3x3 and the 7x7 stem, bf16).
#include <atomic>

#include "conv_patch.h"
#include "conv_stem.h"
#include "gemm_launch.h"

namespace nf {

template <class Cfg, int VW, bool FUSED>
static nf_status launch_kernel(long long total, int lds, const ConvPatchArgs& a, hipStream_t s) {
  auto kern = conv_patch_kernel<Cfg, VW, FUSED>;
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
static nf_status launch_one(ConvPatchArgs& a, int B, hipStream_t s) {
  a.tiles_m = (a.cog + Cfg::kBM - 1) / Cfg::kBM;
  a.tiles_n = (a.HoWo + Cfg::kBN - 1) / Cfg::kBN;
  const long long total = (long long)a.tiles_m * a.tiles_n * a.nG * B;
  if (total <= 0 || total > 0x7fffffffLL) return NF_EUNSUPPORTED;
  a.PS = (a.PS + 7) / 8 * 8;                       // planes keep the 16-byte alignment of their rows
  if ((long long)Cfg::kCB * (a.PS / a.PW) * a.cpr > Cfg::kPatchTasksMax) return NF_EUNSUPPORTED;
  const int lds = Cfg::lds_bytes(a.PS);
  if (lds > 160 * 1024) return NF_EUNSUPPORTED;
  switch (a.VW) {
    case 8: return launch_kernel<Cfg, 8, FUSED>(total, lds, a, s);
    case 4: return launch_kernel<Cfg, 4, FUSED>(total, lds, a, s);
    case 2: return launch_kernel<Cfg, 2, FUSED>(total, lds, a, s);
    case 1: return launch_kernel<Cfg, 1, FUSED>(total, lds, a, s);
  }
  return NF_EUNSUPPORTED;
}

// 3x3, dilation 1, cig % 16 == 0, patch width <= 64.  The caller has filled everything but the tiling.
nf_status launch_conv_patch_3x3(ConvPatchArgs& a, int B, hipStream_t s) {
  // register budgets (last parameter) from measurements: three workgroups per CU pay for the 16-channel stages
  // and for the single-stage fused kernel, not for 32-channel stages looping over many blocks
  if (a.S > 1) return launch_one<ConvPatchCfg<32, 3, 3, 32, 1, 4, 3>, true>(a, B, s);   // fused narrow groups: one 32-channel block
  const long long per_row_tile = (long long)((a.HoWo + 127) / 128) * a.nG * B;
  auto tiles = [&](int bm) { return per_row_tile * ((a.cog + bm - 1) / bm); };
  // 32 channels per stage (half as many barriers) where the patch copy still fits 8 chunks per thread
  const bool deep = a.cig % 32 == 0 && a.cig >= 128 && 32LL * ((a.PS + a.PW - 1) / a.PW) * a.cpr <= 12 * 256;
  // measured on MI355X (M = 32 ResNet-50 layers): a taller row tile re-copies the input patch less often and
  // reuses every gathered B fragment for more output channels, which pays as long as about 400 workgroups
  // remain; stride-2 layers copy four times the patch per output and prefer 128 rows from 200 workgroups up
  if (a.cog > 64 && tiles(128) >= (a.stride > 1 ? 200 : 512)) return launch_one<ConvPatchCfg<128, 3, 3, 16, 2, 2>>(a, B, s);
  if (a.cog > 32 && tiles(64) >= 400)
    return deep ? launch_one<ConvPatchCfg<64, 3, 3, 32, 1, 4, 2>>(a, B, s) : launch_one<ConvPatchCfg<64, 3, 3, 16, 1, 4, 2>>(a, B, s);
  return deep ? launch_one<ConvPatchCfg<32, 3, 3, 32, 1, 4, 2>>(a, B, s) : launch_one<ConvPatchCfg<32, 3, 3, 16, 1, 4, 3>>(a, B, s);
}

// 7x7, stride 2, pad 3, 3 input channels per group.  The caller has filled everything but the tiling and
// has checked W % 8 == 0, 16-byte aligned x, and the patch width.
nf_status launch_conv_stem(ConvStemArgs& a, int B, hipStream_t s) {
  typedef ConvStemCfg<3> Cfg;
  a.tiles_m = (a.cog + Cfg::kBM - 1) / Cfg::kBM;
  a.tiles_n = (a.HoWo + Cfg::kBN - 1) / Cfg::kBN;
  const long long total = (long long)a.tiles_m * a.tiles_n * a.nG * B;
  if (total <= 0 || total > 0x7fffffffLL) return NF_EUNSUPPORTED;
  if (a.PW % 8 != 0 || a.PS % 8 != 0 || a.PS % a.PW != 0) return NF_EUNSUPPORTED;
  const int lds = Cfg::lds_bytes(a.PS);
  if (lds > 64 * 1024) return NF_EUNSUPPORTED;
  nf_launch((conv_stem_kernel<Cfg, 3>), dim3((unsigned)total), dim3(256), lds, s, a);
  return hipGetLastError() == hipSuccess ? NF_OK : NF_ELAUNCH;
}

}  // namespace nf
