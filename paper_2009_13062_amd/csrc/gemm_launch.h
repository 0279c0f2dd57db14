// Host-side launch plumbing of the bf16 MFMA contraction kernels.  The kernel template is
// instantiated per B-loader kind in its own translation unit (gemm_inst_*.hip) so the library
// builds in parallel; the C ABI file only sees launch_gemm_any().
#pragma once
#include <hip/hip_runtime.h>
#include <limits.h>

#include "gemm_mfma.h"
#include "nf_launch.h"

namespace nf {

struct GemmArgs {
  const bf16_t* A; const bf16_t* B; const bf16_t* R; bf16_t* C;
  const bf16_t* B_end;                     // one past the last element of the B operand (loaders that read past a row)
  long lda, ldb, ldc;
  long sA0, sA1, sB0, sB1, sC0, sC1;      // strides of the two batch coordinates (elements)
  int rows, cols, K, nz0, tiles_m, tiles_n;
  int touch_a;                             // direct-to-LDS kernels: pull the A rows into L2 at kernel start (see touch_a_rows)
  Epilogue ep;
  Im2colGeom geom;                         // implicit-B convolution only
};

struct GemmLaunch {
  GemmArgs a;
  int nz1;
  int weights_are_a;                       // convolution: A is the weight tensor; matmul (0): B is
};

enum TileId { T64x64 = 0, T32x128, T128x128w8, kNumTiles };
constexpr int kTileBM[kNumTiles] = {64, 32, 128};
constexpr int kTileBN[kNumTiles] = {64, 128, 128};

// Direct-to-LDS pipelined kernels for problems made of whole tiles (BM x BN, k-step, stages).
enum DmaTileId { D256x256k32s4 = 0, D128x128k32s4, D128x128k64s3w8, D128x384k32s4w12, D128x288k32s4w12, D128x96k64s4w12, kNumDmaTiles };
constexpr int kDmaBM[kNumDmaTiles] = {256, 128, 128, 128, 128, 128};
constexpr int kDmaBN[kNumDmaTiles] = {256, 128, 128, 384, 288, 96};
constexpr int kDmaBK[kNumDmaTiles] = {32, 32, 64, 32, 32, 64};
// dense, 16-byte aligned A and B; NF_EUNSUPPORTED if the problem is not a whole number of tiles
nf_status launch_gemm_dma(int cfg, GemmLaunch& L, hipStream_t s);

// Streaming kernels (gemm_stream.h): nsub consecutive column tiles per workgroup through one load pipeline,
// register epilogue.  Whole-tile problems with 8-byte aligned output rows; NF_EUNSUPPORTED otherwise.
enum StreamTileId { S128x96k64 = 0, S128x128k32, S128x288k32, S128x384k32, S256x256k32, S256x128k32, kNumStreamTiles };
constexpr int kStreamBM[kNumStreamTiles] = {128, 128, 128, 128, 256, 256};
constexpr int kStreamBN[kNumStreamTiles] = {96, 128, 288, 384, 256, 128};
constexpr int kStreamBK[kNumStreamTiles] = {64, 32, 32, 32, 32, 32};
nf_status launch_gemm_stream(int cfg, int nsub, GemmLaunch& L, hipStream_t s);
// The 256 x 256 streaming kernel on fragment-packed weights (B = output of launch_pack_fragments, sB0/sB1 its
// problem strides): rows and columns multiples of 256, K of 32, everything 16-byte aligned.
nf_status launch_gemm_stream_packed(int nsub, GemmLaunch& L, hipStream_t s);

// Fragment-packed weights (gemm_frag.h): B is the output of launch_pack_fragments, sB0/sB1 its problem strides
// (K x cols elements per problem); 128-row tiles of 96 / 288 / 384 columns (the encoder's widths: one tile per
// compute unit at 32 models) and of 128 / 256 columns (4 and 8 wavefronts; for widths the first three do not
// divide), and the 64-row forms of the first three.  NF_EUNSUPPORTED if the problem is not whole tiles, K not a whole number of pipeline rounds, or an
// operand not 16-byte aligned.
enum FragTileId { F96 = 0, F288, F384, F128, F256, F96h, F288h, F384h, kNumFragTiles };
constexpr int kNumFragMainTiles = 3;                             // F96, F288, F384 are tried first
constexpr int kNumFragFullTiles = 5;                             // the 128-row tiles; the rest are their 64-row forms
constexpr int kFragBN[kNumFragTiles] = {96, 288, 384, 128, 256, 96, 288, 384};
constexpr int kFragBM[kNumFragTiles] = {128, 128, 128, 128, 128, 64, 64, 64};
constexpr int kFragKUnit[kNumFragTiles] = {256, 128, 128, 128, 128, 256, 128, 128};      // K must be a multiple of this
nf_status launch_gemm_frag(int cfg, GemmLaunch& L, hipStream_t s);
// W[problems][K][Nout] -> fragment order (pack_kernels.h); K % 16 == 0, Nout % 32 == 0
nf_status launch_pack_fragments(const bf16_t* W, bf16_t* Wp, long long problems, int K, int Nout, hipStream_t s);

// BKIND: 8 / 4 / 1 = dense B read with that vector width; 0 = implicit (im2col) B.
// align_a: 16, 8, 4 or 2 = byte alignment of every A row start (and K a multiple of align_a/2).
template <int BKIND>
nf_status launch_gemm_bkind(int align_a, int tile, GemmLaunch& L, hipStream_t s);

struct ConvPatchArgs;
// 3x3 convolution through the LDS patch-gather kernel (conv_patch.h); see netfuse_conv2d for the conditions.
nf_status launch_conv_patch_3x3(ConvPatchArgs& a, int B, hipStream_t s);
// the same layers through the tap-major kernel (conv_tap.h) where it applies; NF_EUNSUPPORTED = it does not
nf_status launch_conv_tap_3x3(ConvPatchArgs& a, int B, hipStream_t s);
struct ConvStemArgs;
// 7x7 / stride 2 / pad 3 over 3 input channels per group (conv_stem.h)
nf_status launch_conv_stem(ConvStemArgs& a, int B, hipStream_t s);

}  // namespace nf
