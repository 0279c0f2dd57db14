// C ABI of the merged operators: argument validation on the host (before any HIP call), kernel
// selection by (storage type, shape class), launch with the model index folded into the grid.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>

#include "../../include/netfuse.h"
#include "attention_kernels.h"
#include "conv_patch.h"
#include "conv_stem.h"
#include "gemm_launch.h"
#include "gemm_mfma.h"
#include "generic_kernels.h"
#include "nf_common.h"
#include "norm_kernels.h"
#include "probe_kernels.h"

using namespace nf;

namespace {

inline bool is_dtype(int dt) { return dt == NF_F32 || dt == NF_BF16; }
inline bool is_act(int a) { return a == NF_ACT_NONE || a == NF_ACT_RELU || a == NF_ACT_GELU; }
inline bool aligned(const void* p, size_t a) { return p == nullptr || ((uintptr_t)p % a) == 0; }

// product of non-negative ints, saturating at LLONG_MAX
inline long long prod(std::initializer_list<long long> v) {
  long long r = 1;
  for (long long x : v) {
    if (x < 0) return -1;
    if (x != 0 && r > LLONG_MAX / x) return LLONG_MAX;
    r *= x;
  }
  return r;
}
constexpr long long kMaxElems = (1LL << 62);     // element counts must stay below this
constexpr long long kMaxGrid = 0x7fffffffLL;

}  // namespace

namespace nf {
LaunchTiming& launch_timing() {
  static thread_local LaunchTiming t = {nullptr, nullptr};
  return t;
}
}  // namespace nf

namespace {

inline nf_status launched() { return hipGetLastError() == hipSuccess ? NF_OK : NF_ELAUNCH; }

inline unsigned grid_for(long long total, int per_block, long long cap = 1 << 20) {
  long long g = (total + per_block - 1) / per_block;
  if (g > cap) g = cap;
  if (g < 1) g = 1;
  return (unsigned)g;
}

nf_status launch_gemm_any(int bkind, int align_a, int tile, GemmLaunch& L, hipStream_t s) {
  switch (bkind) {
    case 8: return launch_gemm_bkind<8>(align_a, tile, L, s);
    case 24: return launch_gemm_bkind<24>(align_a, tile, L, s);
    case 22: return launch_gemm_bkind<22>(align_a, tile, L, s);
    case 21: return launch_gemm_bkind<21>(align_a, tile, L, s);
    case 27: return launch_gemm_bkind<27>(align_a, tile, L, s);
    case 2: return launch_gemm_bkind<2>(align_a, tile, L, s);
    case 1: return launch_gemm_bkind<1>(align_a, tile, L, s);
    case 0: return launch_gemm_bkind<0>(align_a, tile, L, s);
  }
  return NF_EUNSUPPORTED;
}

// Optional override for tile-shape sweeps: NETFUSE_TILE=<index into TileId>, read once.
int forced_tile() {
  static const int v = [] {
    const char* e = dev_getenv("NETFUSE_TILE");
    if (!e || !*e) return -1;
    const int t = atoi(e);
    return (t >= 0 && t < kNumTiles) ? t : -1;
  }();
  return v;
}

// Optional override for sweeps of the direct-to-LDS kernels: NETFUSE_DMA=<index into DmaTileId>, or -1
// to disable them.
int forced_dma() {
  static const int v = [] {
    const char* e = dev_getenv("NETFUSE_DMA");
    if (!e || !*e) return -2;
    const int t = atoi(e);
    return (t >= -1 && t < kNumDmaTiles) ? t : -2;
  }();
  return v;
}

// Direct-to-LDS kernel for a dense, fully aligned problem made of whole tiles, or -1.  *cost_out receives the
// cost of the choice in the model's unit (operand elements loaded by the busiest CU).
int pick_dma(int rows, int cols, int K, long long problems, long long* cost_out = nullptr) {
  const int f = forced_dma();
  if (f == -1) return -1;
  auto fits = [&](int t) { return rows % kDmaBM[t] == 0 && cols % kDmaBN[t] == 0 && K % kDmaBK[t] == 0; };
  if (f >= 0) return fits(f) ? f : -1;
  // Measured on MI355X: these kernels are bound by what ONE compute unit can pull through its vector
  // memory path (about 22 GB/s per CU at HBM latency, 3x that for L2 hits), not by the matrix pipe, so
  // the cost of a configuration is the operand bytes the busiest CU has to load: its share of the tiles
  // times (A tile + B tile).  Wide tiles re-read the activation rows less often; a tile count that is a
  // whole multiple of the 256 CUs leaves none of them idle.
  constexpr long long kCUs = 256;
  int best = -1;
  long long best_cost = 0;
  for (int t = 0; t < kNumDmaTiles; ++t) {
    if (!fits(t)) continue;
    if (t == D128x128k64s3w8 && !(rows == 128 && (K >= 2048 || fits(D128x384k32s4w12)))) continue;   // long-K / narrow layers only
    const long long tiles = problems * (rows / kDmaBM[t]) * (cols / kDmaBN[t]);
    const long long per_cu = (tiles + kCUs - 1) / kCUs;
    long long cost = per_cu * ((long long)kDmaBM[t] + kDmaBN[t]) * K;
    if (kDmaBK[t] == 64) cost -= cost / 16;               // whole 128-byte lines of A per k-step: slightly cheaper than k32
    if (best < 0 || cost < best_cost) { best = t; best_cost = cost; }
  }
  if (cost_out) *cost_out = best_cost;
  return best;
}

// pick_dma(), unless the register-staged 64x64 tile is expected to be faster (kPreferSmallTile).
// Few merged models leave most CUs without a whole-tile workgroup; the 64x64 register-staged tile
// with its deep load pipeline then spreads the operand stream over more of them.  Same cost model,
// with the measured handicap of that kernel per byte (encoder layer at 8 models: the K = 3072
// matmul 25.6 -> 14.6 us, the 768 x 768 one 12.6 -> 11.0 us; at 32 models nothing changes).
constexpr int kPreferSmallTile = -2;
int pick_dma_or_small(int N, int Nout, int K, long long M) {
  long long dma_cost = 0;
  const int d = pick_dma(N, Nout, K, M, &dma_cost);
  if (d < 0) return -1;
  const long long t64 = M * ((N + 63) / 64) * ((Nout + 63) / 64);
  const long long reg_cost = (t64 + 255) / 256 * 128 * K;
  if (forced_dma() == -2 && forced_tile() < 0 && K % 256 == 0 && reg_cost * 13 < dma_cost * 10) return kPreferSmallTile;
  return d;
}

// Streaming kernel (gemm_stream.h) for a problem that pick_dma() routed to direct-to-LDS tile d, or -1.
// Measured on MI355X, 32 models (us, register epilogue / LDS-staged epilogue of the same tile):
//   GELU epilogues, 128 rows: 768 -> 3072  37.8 / 39.4;   512 rows, three 256x256 tiles per workgroup through
//   one pipeline: 105.6 / 119.1.  The barrier-free epilogue pays where the epilogue is VALU heavy; plain
//   bias / residual epilogues are as fast or faster through LDS (full-line stores), so they keep it --
//   except that 512-row problems whose 256x256 tiling leaves a quarter of the last round of workgroups
//   empty (768 -> 2304: 576 tiles) run as three 128x384 tiles per workgroup (82.7 / 88.4).
int pick_stream(int d, int N, int Nout, int K, long long M, int act, int* nsub) {
  *nsub = 1;
  if (d == D256x256k32s4) {
    const long long tiles = M * (N / 256) * (Nout / 256);
    if (act == NF_ACT_GELU) {
      if (tiles >= 3 * 256 && (Nout / 256) % 3 == 0) *nsub = 3;
      return S256x256k32;
    }
    if (tiles % 256 != 0 && N % 128 == 0 && Nout % 384 == 0 && (Nout / 384) % 3 == 0) {
      const long long t384 = M * (N / 128) * (Nout / 384);
      if (t384 % (3 * 256) == 0) { *nsub = 3; return S128x384k32; }
    }
    return -1;
  }
  if (d == D128x384k32s4w12 && act == NF_ACT_GELU) return S128x384k32;
  return -1;
}

// Developer override NETFUSE_STREAM="<StreamTileId>,<nsub>" (read at every call in builds with developer
// switches): force a streaming kernel and its number of column tiles per workgroup.
bool forced_stream(int* cfg, int* nsub) {
  const char* e = dev_getenv("NETFUSE_STREAM");
  if (!e || !*e) return false;
  return sscanf(e, "%d,%d", cfg, nsub) == 2 && *cfg >= 0 && *cfg < kNumStreamTiles && *nsub >= 1;
}

// Tile choice for the register-staged kernels.
int pick_tile(int rows, int cols, long long problems) {
  const int f = forced_tile();
  if (f >= 0) return f;
  auto tiles = [&](int t) {
    return problems * ((rows + kTileBM[t] - 1) / kTileBM[t]) * ((cols + kTileBN[t] - 1) / kTileBN[t]);
  };
  if (rows <= 32) return T32x128;
  // Measured over the pointwise layers of ResNet-50 / ResNeXt-50 at 16 and 32 merged models: the 8-wave
  // tile wins wherever it yields about a workgroup per CU (two when half of its columns are padding, as
  // on 7x7 images); below that, and for 64 rows, the 64x64 tile does.
  if (cols <= 64) return rows > 64 && tiles(T128x128w8) >= 512 ? T128x128w8 : T64x64;
  return rows > 64 && tiles(T128x128w8) >= 200 ? T128x128w8 : T64x64;
}

// largest alignment (16, 8, 4 or 2 bytes) shared by a pointer and a row pitch / stride set
int common_align(std::initializer_list<const void*> ptrs, std::initializer_list<long long> elem_strides) {
  int al = 16;
  for (const void* p : ptrs)
    while (al > 2 && ((uintptr_t)p % al) != 0) al /= 2;
  for (long long st : elem_strides)
    while (al > 2 && ((st * 2) % al) != 0) al /= 2;
  return al;
}

}  // namespace

// ==========================================================================================
extern "C" {

nf_status netfuse_time_next_launch(void* start_event, void* stop_event) {
  LaunchTiming& t = launch_timing();
  t.start = (hipEvent_t)start_event;
  t.stop = (hipEvent_t)stop_event;
  return NF_OK;
}

nf_status netfuse_probe_mfma(void* sink, int iters, double* flops, void* stream) {
  if (!sink || iters <= 0 || !flops) return NF_EINVAL;
  if (!aligned(sink, 4)) return NF_EINVAL;
  const int wgs = 256;                                        // one workgroup of 16 wavefronts per compute unit
  *flops = (double)wgs * kProbeWaves * iters * 4 * kProbeFlopsPerMfma;
  nf_launch(probe_mfma_kernel, dim3(wgs), dim3(kProbeWaves * kWave), 0, (hipStream_t)stream, (float*)sink, iters, 0);
  return launched();
}

nf_status netfuse_probe_hbm_read(const void* src, long long bytes, void* sink, void* stream) {
  if (!src || !sink || bytes < 16 || bytes % 16) return NF_EINVAL;
  if (!aligned(src, 16) || !aligned(sink, 4)) return NF_EINVAL;
  const size_t chunks = (size_t)bytes / 16;
  const size_t per_wg = (size_t)256 * kProbeReadUnroll;
  size_t wgs = (chunks + per_wg - 1) / per_wg;
  if (wgs > 256 * 8) wgs = 256 * 8;                           // eight workgroups per compute unit, grid-stride beyond
  nf_launch(probe_hbm_read_kernel, dim3((unsigned)wgs), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, chunks,
            (uint32_t*)sink, 0);
  return launched();
}

const char* netfuse_strerror(nf_status st) {
  switch (st) {
    case NF_OK: return "ok";
    case NF_EINVAL: return "invalid argument";
    case NF_EUNSUPPORTED: return "no kernel for these arguments";
    case NF_ELAUNCH: return "HIP launch failed";
  }
  return "unknown status";
}

nf_status netfuse_linear(const void* X, const void* W, const float* bias, const void* residual, void* Y,
                         int M, int N, int K, int Nout, nf_dtype dt, nf_act act, void* stream) {
  if (!X || !W || !Y) return NF_EINVAL;
  if (M <= 0 || N <= 0 || K <= 0 || Nout <= 0) return NF_EINVAL;
  if (!is_dtype(dt) || !is_act(act)) return NF_EINVAL;
  if (prod({M, N, K}) >= kMaxElems || prod({M, K, Nout}) >= kMaxElems || prod({M, N, Nout}) >= kMaxElems)
    return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(X, esz) || !aligned(W, esz) || !aligned(Y, esz) || !aligned(residual, esz) || !aligned(bias, 4))
    return NF_EINVAL;
  hipStream_t s = (hipStream_t)stream;

  if (dt == NF_BF16) {
    const int al_a = common_align({X}, {K, (long long)N * K});
    const int al_b = common_align({W}, {Nout, (long long)K * Nout});
    // vector width of the B loader: its chunks must not straddle the end of a row
    int bkind = 1;
    if (al_b == 16 && Nout % 8 == 0) bkind = 8;
    int al = al_a;
    while (al > 2 && (K % (al / 2)) != 0) al /= 2;
    GemmLaunch L;
    memset(&L, 0, sizeof(L));
    GemmArgs& a = L.a;
    a.A = (const bf16_t*)X; a.B = (const bf16_t*)W; a.R = (const bf16_t*)residual; a.C = (bf16_t*)Y;
    a.B_end = a.B + (long long)M * K * Nout;
    a.lda = K; a.ldb = Nout; a.ldc = Nout;
    a.sA0 = (long)N * K; a.sB0 = (long)K * Nout; a.sC0 = (long)N * Nout;
    a.rows = N; a.cols = Nout; a.K = K; a.nz0 = M;
    L.nz1 = 1;
    a.ep.col_bias = bias; a.ep.col_vec_stride0 = Nout;
    a.ep.act = act; a.ep.act_before_residual = 1;
    a.ep.vec_store = Nout % 8 == 0 && aligned(Y, 16) && aligned(residual, 16)  ? 2
                     : Nout % 4 == 0 && aligned(Y, 8) && aligned(residual, 8) ? 1 : 0;
    if (bkind == 8 && al == 16) {
      int scfg, snsub;
      if (forced_stream(&scfg, &snsub)) {
        const nf_status st = launch_gemm_stream(scfg, snsub, L, s);
        if (st != NF_EUNSUPPORTED) return st;
      }
      const int d = pick_dma_or_small(N, Nout, K, M);
      if (d == kPreferSmallTile) return launch_gemm_any(bkind, al, T64x64, L, s);
      if (d >= 0) {
        const int sc = pick_stream(d, N, Nout, K, M, act, &snsub);
        if (sc >= 0) {
          const nf_status st = launch_gemm_stream(sc, snsub, L, s);
          if (st != NF_EUNSUPPORTED) return st;
        }
        return launch_gemm_dma(d, L, s);
      }
    }
    return launch_gemm_any(bkind, al, pick_tile(N, Nout, M), L, s);
  }
  const int tiles_m = (N + 63) / 64, tiles_n = (Nout + 63) / 64;
  const long long total = prod({tiles_m, tiles_n, M});
  if (total > kMaxGrid) return NF_EUNSUPPORTED;
  nf_launch(linear_generic_kernel<float>, dim3((unsigned)total), dim3(256), 0, s, (const float*)X,
                     (const float*)W, bias, (const float*)residual, (float*)Y, N, K, Nout, (int)act, tiles_m,
                     tiles_n);
  return launched();
}

// The fragment-packed kernel for (N, K, Nout) at M models: the tile width that needs the fewest rounds of
// workgroups over the 256 compute units, weighted by its width (a round streams width x K weights per unit);
// ties go to the wider tile.  -1 if no tile fits.
#ifndef NF_FRAG_HALF_TILES
#define NF_FRAG_HALF_TILES 1
#endif
static int pick_frag(int N, int Nout, int K, int M) {
  static const int forced = [] { const char* e = dev_getenv("NETFUSE_FRAG"); return e ? atoi(e) : -1; }();
  auto fits = [&](int t) { return N % kFragBM[t] == 0 && Nout % kFragBN[t] == 0 && K % kFragKUnit[t] == 0; };
  if (forced >= 0 && forced < kNumFragTiles && fits(forced)) return forced;
  auto tiles_of = [&](int t) { return (long long)M * (N / kFragBM[t]) * (Nout / kFragBN[t]); };
  auto best_of = [&](int lo, int hi) {
    int best = -1;
    long long best_cost = 0;
    for (int t = lo; t < hi; ++t) {
      if (!fits(t)) continue;
      const long long cost = (tiles_of(t) + 255) / 256 * kFragBN[t];
      if (best < 0 || cost < best_cost || (cost == best_cost && kFragBN[t] > kFragBN[best])) { best = t; best_cost = cost; }
    }
    return best;
  };
  // the 12- and 9-wavefront tiles wherever one of them divides the width, else the 128 / 256 column ones
  int pick = best_of(0, kNumFragMainTiles);
  if (pick < 0) pick = best_of(kNumFragMainTiles, kNumFragFullTiles);
  // With fewer models the 128-row tiles leave compute units idle or need a second, half empty round.  The
  // 64-row form of a width doubles the workgroups; the two row tiles of a column tile run side by side and share
  // its weights through L2, so a compute unit's weight stream costs about half as much as one of its own
  // (factor 0.45).  Only where that gives one round of more than 128 workgroups.  Measured at 16 models and 128
  // rows (us): 3072 -> 768 32.7 -> 24.5, 768 -> 768 12.8 -> 10.0 (96 columns), 768 -> 2304 24.4 -> 18.4 (288 against 96),
  // 768 -> 3072 29.2 -> 23.2 (384 against 96); forward 1.38 -> 1.15 ms.  At 8 models they lose against what runs now.
  if (NF_FRAG_HALF_TILES) {
    long long best_cost = pick < 0 ? -1 : 100 * ((tiles_of(pick) + 255) / 256 * kFragBN[pick]);
    for (int t = kNumFragFullTiles; t < kNumFragTiles; ++t) {
      if (!fits(t) || tiles_of(t) <= 128 || tiles_of(t) > 256) continue;
      const long long cost = 45LL * kFragBN[t];
      if (best_cost < 0 || cost < best_cost) { pick = t; best_cost = cost; }
    }
  }
  return pick;
}

// The 256 x 256 streaming kernel on packed weights (several column tiles per workgroup through one pipeline;
// gemm_stream.h).  It takes the shapes the 128-row fragment kernel has no tile for (output widths that are
// multiples of 256 but not of 96, 288 or 384), and it is preferred where it measured faster: with a GELU
// epilogue and at least three tiles per compute unit (768 -> 3072 at 512 rows and 32 models: 102 against 107 us;
// without the GELU the fragment kernel is ahead: 75 against 88, 82 against 98, 32 against 39 us on the other
// three encoder shapes).  Returns the number of column tiles per workgroup, 0 = not applicable.
static int pick_packed_stream(int N, int Nout, int K, int M, int act, bool* preferred) {
  *preferred = false;
  if (N % 256 || Nout % 256 || K % 32) return 0;
  const int tn = Nout / 256;
  const long long tiles = (long long)M * (N / 256) * tn;
  // tiles a compute unit works through one after the other = rounds of workgroups x tiles per workgroup;
  // ties go to more tiles per workgroup (one launch ramp, epilogues under the next tile's loads)
  int best = 1;
  long long best_cost = 0;
  for (int n = 1; n <= tn; ++n) {
    if (tn % n) continue;
    const long long cost = ((tiles / n + 255) / 256) * n;
    if (n == 1 || cost <= best_cost) { best = n; best_cost = cost; }
  }
  *preferred = act == NF_ACT_GELU && tiles >= 3 * 256;
  return best;
}

int netfuse_linear_packed_supported(int M, int N, int K, int Nout, nf_dtype dt) {
  if (dt != NF_BF16 || M <= 0 || N <= 0 || K <= 0 || Nout <= 0) return 0;
  bool pref;
  const int f = pick_frag(N, Nout, K, M);
  if (f < 0) return pick_packed_stream(N, Nout, K, M, NF_ACT_NONE, &pref) > 0 ? 1 : 0;
  // With few models the 128-row tiles leave most compute units idle and netfuse_linear's small tiles win
  // (one encoder layer at 8 models: 0.088 ms packed against 0.074 ms; at 16 models packed is ahead): the answer
  // is "no" below half a workgroup per compute unit, although netfuse_linear_packed itself still runs there.
  const long long tiles = (long long)M * (N / kFragBM[f]) * (Nout / kFragBN[f]);
  return tiles >= 128 ? 1 : 0;
}

nf_status netfuse_linear_pack_weight(const void* W, void* Wp, int M, int K, int Nout, nf_dtype dt, void* stream) {
  if (!W || !Wp || W == Wp) return NF_EINVAL;
  if (M <= 0 || K <= 0 || Nout <= 0 || !is_dtype(dt)) return NF_EINVAL;
  if (K % 16 != 0 || Nout % 32 != 0) return NF_EINVAL;
  const long long total = prod({M, K, Nout});
  if (total >= kMaxElems) return NF_EINVAL;
  if (dt != NF_BF16) return NF_EUNSUPPORTED;
  if (!aligned(W, 2) || !aligned(Wp, 16)) return NF_EINVAL;
  return launch_pack_fragments((const bf16_t*)W, (bf16_t*)Wp, M, K, Nout, (hipStream_t)stream);
}

nf_status netfuse_linear_packed(const void* X, const void* Wp, const float* bias, const void* residual, void* Y,
                                int M, int N, int K, int Nout, nf_dtype dt, nf_act act, void* stream) {
  if (!X || !Wp || !Y) return NF_EINVAL;
  if (M <= 0 || N <= 0 || K <= 0 || Nout <= 0) return NF_EINVAL;
  if (!is_dtype(dt) || !is_act(act)) return NF_EINVAL;
  if (K % 16 != 0 || Nout % 32 != 0) return NF_EINVAL;
  if (prod({M, N, K}) >= kMaxElems || prod({M, K, Nout}) >= kMaxElems || prod({M, N, Nout}) >= kMaxElems)
    return NF_EINVAL;
  if (dt != NF_BF16) return NF_EUNSUPPORTED;
  if (!aligned(X, 2) || !aligned(Wp, 16) || !aligned(Y, 2) || !aligned(residual, 2) || !aligned(bias, 4))
    return NF_EINVAL;
  const int f = pick_frag(N, Nout, K, M);
  bool ps_preferred;
  const int ps = pick_packed_stream(N, Nout, K, M, act, &ps_preferred);
  if (f < 0 && ps <= 0) return NF_EUNSUPPORTED;
  GemmLaunch L;
  memset(&L, 0, sizeof(L));
  GemmArgs& a = L.a;
  a.A = (const bf16_t*)X; a.B = (const bf16_t*)Wp; a.R = (const bf16_t*)residual; a.C = (bf16_t*)Y;
  a.B_end = a.B + (long long)M * K * Nout;
  a.lda = K; a.ldb = 0; a.ldc = Nout;
  a.sA0 = (long)N * K; a.sB0 = (long)K * Nout; a.sC0 = (long)N * Nout;
  a.rows = N; a.cols = Nout; a.K = K; a.nz0 = M;
  L.nz1 = 1;
  a.ep.col_bias = bias; a.ep.col_vec_stride0 = Nout;
  a.ep.act = act; a.ep.act_before_residual = 1;
  if (ps > 0 && (ps_preferred || f < 0)) {
    a.ep.vec_store = 2;
    const nf_status st = launch_gemm_stream_packed(ps, L, (hipStream_t)stream);
    if (st != NF_EUNSUPPORTED || f < 0) return st;
  }
  return launch_gemm_frag(f, L, (hipStream_t)stream);
}

nf_status netfuse_linear_ragged(const void* X, const void* W, const float* bias, void* Y, int M, int N, int K,
                                const int* nout, nf_dtype dt, nf_act act, void* stream) {
  if (!X || !W || !Y || !nout) return NF_EINVAL;
  if (M <= 0 || N <= 0 || K <= 0) return NF_EINVAL;
  if (!is_dtype(dt) || !is_act(act)) return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(X, esz) || !aligned(W, esz) || !aligned(Y, esz) || !aligned(bias, 4)) return NF_EINVAL;
  if (prod({M, N, K}) >= kMaxElems) return NF_EINVAL;
  long long cols = 0, tiles = 0;
  for (int m = 0; m < M; ++m) {
    if (nout[m] <= 0) return NF_EINVAL;
    cols += nout[m];
    tiles += (long long)((N + 7) / 8) * ((nout[m] + 63) / 64);
    if (cols > INT_MAX || tiles > kMaxGrid) return NF_EINVAL;
  }
  if (prod({cols, K}) >= kMaxElems || prod({cols, N}) >= kMaxElems) return NF_EINVAL;
  if (M > kRaggedMaxModels) return NF_EUNSUPPORTED;
  RaggedTable tab;
  tab.tile_start[0] = 0; tab.col_start[0] = 0;
  for (int m = 0; m < M; ++m) {
    tab.tile_start[m + 1] = tab.tile_start[m] + ((N + 7) / 8) * ((nout[m] + 63) / 64);
    tab.col_start[m + 1] = tab.col_start[m] + nout[m];
  }
  for (int m = M + 1; m <= kRaggedMaxModels; ++m) { tab.tile_start[m] = tab.tile_start[M]; tab.col_start[m] = tab.col_start[M]; }
  hipStream_t s = (hipStream_t)stream;
  if (dt == NF_F32)
    nf_launch(linear_ragged_kernel<float>, dim3((unsigned)tiles), dim3(256), 0, s, (const float*)X, (const float*)W,
              bias, (float*)Y, M, N, K, (int)act, tab);
  else
    nf_launch(linear_ragged_kernel<bf16_t>, dim3((unsigned)tiles), dim3(256), 0, s, (const bf16_t*)X, (const bf16_t*)W,
              bias, (bf16_t*)Y, M, N, K, (int)act, tab);
  return launched();
}

nf_status netfuse_conv2d(const void* x, const void* w, const float* bias, const float* scale, const float* shift,
                         const void* residual, void* y, int M, int B, int Cin, int Cout, int g, int H, int W,
                         int KH, int KW, int stride, int pad, int dilation, nf_dtype dt, nf_act act,
                         void* stream) {
  if (!x || !w || !y) return NF_EINVAL;
  if (M <= 0 || B <= 0 || Cin <= 0 || Cout <= 0 || g <= 0 || H <= 0 || W <= 0 || KH <= 0 || KW <= 0)
    return NF_EINVAL;
  if (stride <= 0 || pad < 0 || dilation <= 0) return NF_EINVAL;
  if (Cin % g != 0 || Cout % g != 0) return NF_EINVAL;
  if ((scale == nullptr) != (shift == nullptr)) return NF_EINVAL;
  if (!is_dtype(dt) || !is_act(act)) return NF_EINVAL;
  const long long eh = (long long)H + 2LL * pad - (long long)dilation * (KH - 1) - 1;
  const long long ew = (long long)W + 2LL * pad - (long long)dilation * (KW - 1) - 1;
  if (eh < 0 || ew < 0) return NF_EINVAL;
  const long long Ho = eh / stride + 1, Wo = ew / stride + 1;
  const int cig = Cin / g, cog = Cout / g;
  const long long Ctot_in = (long long)M * Cin, Ctot_out = (long long)M * Cout;
  if (Ctot_in > INT_MAX || Ctot_out > INT_MAX || Ho * Wo > INT_MAX || (long long)H * W > INT_MAX ||
      prod({cig, KH, KW}) > INT_MAX || (long long)H + 2LL * pad > INT_MAX || (long long)W + 2LL * pad > INT_MAX)
    return NF_EINVAL;
  const long long n_in = prod({B, Ctot_in, H, W}), n_out = prod({B, Ctot_out, Ho, Wo});
  const long long n_w = prod({Ctot_out, cig, KH, KW});
  if (n_in >= kMaxElems || n_out >= kMaxElems || n_w >= kMaxElems) return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(x, esz) || !aligned(w, esz) || !aligned(y, esz) || !aligned(residual, esz) || !aligned(bias, 4) ||
      !aligned(scale, 4) || !aligned(shift, 4))
    return NF_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const int HoWo = (int)(Ho * Wo);
  const int Kdim = cig * KH * KW;

  static const bool no_mfma_conv = dev_getenv("NETFUSE_CONV_GENERIC") != nullptr;
  if (dt == NF_BF16 && !no_mfma_conv) {
    GemmLaunch L;
    memset(&L, 0, sizeof(L));
    GemmArgs& a = L.a;
    a.A = (const bf16_t*)w; a.B = (const bf16_t*)x; a.R = (const bf16_t*)residual; a.C = (bf16_t*)y;
    a.B_end = a.B + (long long)B * Ctot_in * H * W;
    a.lda = Kdim; a.ldc = HoWo;
    a.sA0 = (long)cog * Kdim; a.sA1 = 0;
    a.sB0 = (long)cig * H * W; a.sB1 = (long)Ctot_in * H * W;
    a.sC0 = (long)cog * HoWo; a.sC1 = (long)Ctot_out * HoWo;
    a.rows = cog; a.cols = HoWo; a.K = Kdim; a.nz0 = M * g;
    L.nz1 = B;
    L.weights_are_a = 1;
    a.ep.row_bias = bias; a.ep.row_scale = scale; a.ep.row_shift = shift;
    a.ep.row_vec_stride0 = cog; a.ep.row_vec_stride1 = 0;
    a.ep.act = act; a.ep.act_before_residual = 0;
    a.ep.vec_store = HoWo % 8 == 0 && aligned(y, 16) && aligned(residual, 16)  ? 2
                     : HoWo % 4 == 0 && aligned(y, 8) && aligned(residual, 8) ? 1
                     : HoWo <= 64 && ((long long)cog * HoWo) % 8 == 0 && aligned(y, 16) && aligned(residual, 16) ? 3 : 0;
    int al = common_align({w}, {Kdim});
    while (al > 2 && (Kdim % (al / 2)) != 0) al /= 2;
    const long long problems = (long long)M * g * B;
    const bool pointwise = KH == 1 && KW == 1 && stride == 1 && pad == 0;
    int tile = pick_tile(cog, HoWo, problems);
    // gathered B operand (strided or k x k taps): its loads are the expensive part, so a few output
    // positions are better served by tall tiles that gather them once per 128 output channels (measured)
    if (!pointwise && forced_tile() < 0 && HoWo <= 64 && cog >= 256) tile = T128x128w8;
    if (pointwise) {
      // a 1x1 convolution is a matrix product over the channel dimension with the H*W positions as
      // columns (the converse of Section 3.1's remark that a matmul is a 1x1 convolution)
      a.ldb = (long)H * W;
      const int al_b = common_align({x}, {(long long)H * W});
      int bkind = 1;
      if (al_b == 16 && HoWo % 8 == 0) bkind = 8;
      return launch_gemm_any(bkind, al, tile, L, s);
    }
    static const bool no_patch = dev_getenv("NETFUSE_NO_PATCH") != nullptr;
    if (!no_patch && KH == 7 && KW == 7 && stride == 2 && pad == 3 && dilation == 1 && cig == 3 && W % 8 == 0 &&
        aligned(x, 16)) {
      // the ResNet stem: a few input channels under a wide kernel (conv_stem.h)
      const int PWs = (std::max(8 + W, 2 * ((int)Wo - 1) + 12) + 7) / 8 * 8;     // copied columns and gathered segments fit
      const int span_s = (int)std::min<long long>(Ho, (126 + Wo) / Wo + 1);      // output rows one 128-position tile can touch
      const int PHs = (span_s - 1) * 2 + 7;
      ConvStemArgs c;
      memset(&c, 0, sizeof(c));
      c.x = (const bf16_t*)x; c.w = (const bf16_t*)w; c.R = (const bf16_t*)residual; c.y = (bf16_t*)y;
      c.cog = cog; c.nG = M * g; c.H = H; c.W = W; c.Ho = (int)Ho; c.Wo = (int)Wo; c.HoWo = HoWo;
      c.PW = PWs; c.PS = PHs * PWs; c.cpr = W / 8;
      c.x_group = (long)cig * H * W; c.x_image = (long)Ctot_in * H * W;
      c.y_group = (long)cog * HoWo; c.y_image = (long)Ctot_out * HoWo;
      c.ep = a.ep;
      c.ep.row_vec_stride0 = cog;
      const nf_status st = launch_conv_stem(c, B, s);
      if (st != NF_EUNSUPPORTED) return st;
    }
    // patch geometry (conv_patch.h): image column ix sits at patch column ix + 8; rows are copied in
    // chunks of VW pixels; a 128-position tile touches at most `span` output rows
    const int VW = W % 8 == 0 ? 8 : (W % 4 == 0 ? 4 : (W % 2 == 0 ? 2 : 1));
    const int maxcol = std::max(kLPad + W - 1, ((int)Wo - 1) * stride + KW - 1 - pad + kLPad);
    const int PWp = (maxcol + 1 + 7) / 8 * 8;
    const int span = (int)std::min<long long>(Ho, (126 + Wo) / Wo + 1);
    const int PHmax = (span - 1) * stride + KH;
    // narrow groups: fuse S = 32 / cig consecutive groups OF ONE MODEL into one 32-channel block
    // (block-diagonal weights).  The zero blocks are still multiplied with the neighbouring groups'
    // activations, and 0 * NaN = NaN, so a fused block never spans two models (g % S == 0): a non-finite
    // value in one model's input cannot reach another model's output.
    int S = 1;
    if (cig < 32 && 32 % cig == 0 && cig % 4 == 0 && (long long)(32 / cig) * cog <= 32 && g % (32 / cig) == 0 &&
        aligned(w, 8))
      S = 32 / cig;
    const int cig_e = S * cig, cog_e = S * cog;               // channels of the (fused) group a workgroup handles
    const long long patch_tasks = (long long)std::min(cig_e, 16) * PHmax * (W / VW);   // chunk copies per channel block
    const bool patch_ok = KH == 3 && KW == 3 && dilation == 1 && pad <= kLPad && aligned(x, 16) &&
                          ((S == 1 && cig % 16 == 0 && aligned(w, 16) && patch_tasks <= 12 * 256) ||
                           (S > 1 && 2 * patch_tasks <= 12 * 256));
    // the tap-major kernel (conv_tap.h) checks its own task and LDS bounds
    static const bool no_tap = dev_getenv("NETFUSE_NO_TAP") != nullptr;
    const bool tap_ok = !no_tap && KH == 3 && KW == 3 && dilation == 1 && pad <= kLPad && cig_e % 32 == 0;
    if (!no_patch && (patch_ok || tap_ok)) {
      // k x k: MFMA operands from an LDS copy of the zero-padded input patch (conv_tap.h, conv_patch.h)
      ConvPatchArgs c;
      memset(&c, 0, sizeof(c));
      c.x = (const bf16_t*)x; c.w = (const bf16_t*)w; c.R = (const bf16_t*)residual; c.y = (bf16_t*)y;
      c.cig = cig_e; c.cog = cog_e; c.nG = M * g / S; c.S = S; c.cig_real = cig; c.cog_real = cog;
      c.H = H; c.W = W; c.Ho = (int)Ho; c.Wo = (int)Wo; c.HoWo = HoWo;
      c.stride = stride; c.pad = pad;
      c.PW = PWp; c.VW = VW; c.cpr = W / VW;
      c.PS = PHmax * PWp;               // padded per kernel configuration at launch
      c.x_group = (long)cig_e * H * W; c.x_image = (long)Ctot_in * H * W;
      c.y_group = (long)cog_e * HoWo; c.y_image = (long)Ctot_out * HoWo;
      c.ep = a.ep;
      c.ep.row_vec_stride0 = cog_e;
      if (tap_ok) {
        const nf_status st = launch_conv_tap_3x3(c, B, s);
        if (st != NF_EUNSUPPORTED) return st;
      }
      if (patch_ok) {
        const nf_status st = launch_conv_patch_3x3(c, B, s);
        if (st != NF_EUNSUPPORTED) return st;           // else: the implicit-GEMM kernel below takes any shape
      }
    }
    a.geom.H = H; a.geom.W = W; a.geom.KH = KH; a.geom.KW = KW; a.geom.Wo = (int)Wo;
    a.geom.stride = stride; a.geom.pad = pad; a.geom.dil = dilation;
    int bkind = 0;
    if (KH == 1 && KW == 1 && pad == 0) {
      // projection shortcuts; stride 2 over an even width is read as aligned pixel pairs where the shape allows
      bkind = 2;
      const long long plane = (long long)H * W;
      if (stride == 2 && W == 2 * Wo) {
        if (Wo % 4 == 0 && plane % 8 == 0 && aligned(x, 16)) bkind = 24;
        else if (Wo % 2 == 0 && plane % 4 == 0 && aligned(x, 8)) bkind = 22;
        else if (Wo == 7 && Ho <= 8 && plane % 4 == 0 && aligned(x, 8)) bkind = 27;
        else if (aligned(x, 4)) bkind = 21;
      }
    }
    return launch_gemm_any(bkind, al, tile, L, s);
  }

  ConvGeom geo;
  geo.B = B; geo.Ctot_in = (int)Ctot_in; geo.Ctot_out = (int)Ctot_out; geo.cig = cig; geo.cog = cog;
  geo.H = H; geo.W = W; geo.KH = KH; geo.KW = KW; geo.Ho = (int)Ho; geo.Wo = (int)Wo;
  geo.stride = stride; geo.pad = pad; geo.dil = dilation;
  const unsigned grid = grid_for(n_out, 256);
  if (dt == NF_F32)
    nf_launch(conv2d_generic_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)x,
                       (const float*)w, bias, scale, shift, (const float*)residual, (float*)y, geo, (int)act,
                       (size_t)n_out);
  else
    nf_launch(conv2d_generic_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)x,
                       (const bf16_t*)w, bias, scale, shift, (const bf16_t*)residual, (bf16_t*)y, geo, (int)act,
                       (size_t)n_out);
  return launched();
}

nf_status netfuse_layernorm(const void* x, const void* residual, const float* gamma, const float* beta, void* y,
                            int M, int rows, int H, float eps, nf_merge_dim layout, nf_dtype dt, void* stream) {
  if (!x || !gamma || !beta || !y) return NF_EINVAL;
  if (M <= 0 || rows <= 0 || H <= 0) return NF_EINVAL;
  if (!(eps >= 0.f)) return NF_EINVAL;
  if (layout != NF_MERGE_BATCH && layout != NF_MERGE_CHANNEL) return NF_EINVAL;
  if (!is_dtype(dt)) return NF_EINVAL;
  if (prod({M, rows, H}) >= kMaxElems) return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(x, esz) || !aligned(y, esz) || !aligned(residual, esz) || !aligned(gamma, 4) || !aligned(beta, 4))
    return NF_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  const long long nrows = (long long)M * rows;
  const long long blocks = (nrows + 3) / 4;
  if (blocks > kMaxGrid) return NF_EUNSUPPORTED;
  const size_t va = 4 * esz;
  const bool vec = H % 4 == 0 && aligned(x, va) && aligned(y, va) && aligned(residual, va);
  const int ch = layout == NF_MERGE_CHANNEL;
  // rows that fit in registers: two per wavefront (they share the model's gamma and beta) once there are
  // enough rows to keep every CU busy that way (measured: 16384 rows of 768 11.8 -> 10.4 us, 4096 rows
  // 3.9 -> 4.7 us)
  static const int ln_forced = [] { const char* e = dev_getenv("NETFUSE_LN_ROWS"); return e ? atoi(e) : 0; }();
  const int ln_rows = ln_forced ? ln_forced : (nrows >= 16384 ? 2 : 1);
  if (vec && H <= kWave * 4 * 4 && (ln_rows == 2 || ln_rows == 4) && rows % ln_rows == 0) {
    const long long blocks_r = (nrows / ln_rows + 3) / 4;
#define NF_LNR(T, R)                                                                                      \
  nf_launch((layernorm_rows_kernel<T, 4, 4, R>), dim3((unsigned)blocks_r), dim3(256), 0, s,       \
                     (const T*)x, (const T*)residual, gamma, beta, (T*)y, M, rows, H, eps, ch)
    if (dt == NF_F32) { if (ln_rows == 2) NF_LNR(float, 2); else NF_LNR(float, 4); }
    else { if (ln_rows == 2) NF_LNR(bf16_t, 2); else NF_LNR(bf16_t, 4); }
#undef NF_LNR
    return launched();
  }
#define NF_LN(T, VEC, MAXIT)                                                                             \
  nf_launch((layernorm_kernel<T, VEC, MAXIT>), dim3((unsigned)blocks), dim3(256), 0, s,         \
                     (const T*)x, (const T*)residual, gamma, beta, (T*)y, M, rows, H, eps, ch)
  if (dt == NF_F32) {
    if (vec) NF_LN(float, 4, 4); else NF_LN(float, 1, 8);
  } else {
    if (vec) NF_LN(bf16_t, 4, 4); else NF_LN(bf16_t, 1, 8);
  }
#undef NF_LN
  return launched();
}

nf_status netfuse_batchnorm(const void* x, const float* gamma, const float* beta, const float* mean,
                            const float* var, const void* residual, void* y, int M, int B, int C, int HW,
                            float eps, nf_dtype dt, nf_act act, void* stream) {
  if (!x || !gamma || !beta || !mean || !var || !y) return NF_EINVAL;
  if (M <= 0 || B <= 0 || C <= 0 || HW <= 0) return NF_EINVAL;
  if (!(eps >= 0.f)) return NF_EINVAL;
  if (!is_dtype(dt) || !is_act(act)) return NF_EINVAL;
  const long long Ctot = (long long)M * C;
  if (Ctot > INT_MAX || prod({B, Ctot, HW}) >= kMaxElems) return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(x, esz) || !aligned(y, esz) || !aligned(residual, esz) || !aligned(gamma, 4) ||
      !aligned(beta, 4) || !aligned(mean, 4) || !aligned(var, 4))
    return NF_EINVAL;
  const long long rowsbc = (long long)B * Ctot;
  if (rowsbc > kMaxGrid) return NF_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  const long long n_el = prod({B, Ctot, HW});
  const int per = 16 / (int)esz;
  if (n_el % per == 0 && aligned(x, 16) && aligned(y, 16) && aligned(residual, 16) && n_el / per / 256 < kMaxGrid) {
    const long long chunks = n_el / per;
    const unsigned grid = (unsigned)((chunks + 255) / 256);
    if (dt == NF_F32)
      nf_launch(batchnorm_flat_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)x, gamma, beta, mean, var,
                (const float*)residual, (float*)y, (int)Ctot, HW, eps, (int)act, (size_t)chunks);
    else
      nf_launch(batchnorm_flat_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)x, gamma, beta, mean, var,
                (const bf16_t*)residual, (bf16_t*)y, (int)Ctot, HW, eps, (int)act, (size_t)chunks);
    return launched();
  }
  const unsigned gy = (unsigned)((HW + 1023) / 1024 > 64 ? 64 : (HW + 1023) / 1024);
  if (dt == NF_F32)
    nf_launch(batchnorm_kernel<float>, dim3((unsigned)rowsbc, gy), dim3(256), 0, s, (const float*)x,
                       gamma, beta, mean, var, (const float*)residual, (float*)y, (int)Ctot, HW, eps, (int)act);
  else
    nf_launch(batchnorm_kernel<bf16_t>, dim3((unsigned)rowsbc, gy), dim3(256), 0, s, (const bf16_t*)x,
                       gamma, beta, mean, var, (const bf16_t*)residual, (bf16_t*)y, (int)Ctot, HW, eps, (int)act);
  return launched();
}

nf_status netfuse_bn_fold(const float* gamma, const float* beta, const float* mean, const float* var, float* scale,
                          float* shift, int n, float eps, void* stream) {
  if (!gamma || !beta || !mean || !var || !scale || !shift) return NF_EINVAL;
  if (n <= 0 || !(eps >= 0.f)) return NF_EINVAL;
  if (!aligned(gamma, 4) || !aligned(beta, 4) || !aligned(mean, 4) || !aligned(var, 4) || !aligned(scale, 4) ||
      !aligned(shift, 4))
    return NF_EINVAL;
  nf_launch(bn_fold_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, gamma,
                     beta, mean, var, scale, shift, n, eps);
  return launched();
}

nf_status netfuse_attention(const void* Q, const void* K, const void* V, const float* mask, void* O, int M, int B,
                            int S, int heads, int d, long stride_m, long stride_row, float scale, nf_dtype dt,
                            void* stream) {
  if (!Q || !K || !V || !O) return NF_EINVAL;
  if (M <= 0 || B <= 0 || S <= 0 || heads <= 0 || d <= 0) return NF_EINVAL;
  if (!is_dtype(dt) || !(scale == scale)) return NF_EINVAL;
  const long long hd = (long long)heads * d;
  if (hd > INT_MAX) return NF_EINVAL;
  if (stride_row < hd) return NF_EINVAL;                              // heads of one row are side by side
  if (prod({B, S}) > INT_MAX / 2) return NF_EINVAL;
  if (stride_m < 0 || (M > 1 && stride_m < (long long)(B * (long long)S - 1) * stride_row + hd)) return NF_EINVAL;
  if (prod({M, B, S, hd}) >= kMaxElems || prod({M, stride_m}) >= kMaxElems) return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(Q, esz) || !aligned(K, esz) || !aligned(V, esz) || !aligned(O, esz) || !aligned(mask, 4))
    return NF_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  AttnArgs a;
  a.Q = Q; a.K = K; a.V = V; a.mask = mask; a.O = O;
  a.M = M; a.B = B; a.S = S; a.heads = heads; a.d = d;
  a.stride_m = stride_m; a.stride_row = stride_row; a.scale = scale;

  if (dt == NF_BF16 && d == kAttnD && stride_row % 8 == 0 && stride_m % 8 == 0 && aligned(Q, 16) &&
      aligned(K, 16) && aligned(V, 16) && aligned(O, 8)) {
    const int qblocks = (S + 127) / 128;
    const long long total = prod({M, B, heads, qblocks});
    if (total > kMaxGrid) return NF_EUNSUPPORTED;
    nf_launch(attention_mfma_d64_kernel, dim3((unsigned)total), dim3(256), 0, s, a, qblocks);
    return launched();
  }
  if (d > 256) return NF_EUNSUPPORTED;
  const long long waves = prod({M, B, heads, S});
  const long long blocks = (waves + 3) / 4;
  if (blocks > kMaxGrid) return NF_EUNSUPPORTED;
  const int dpl = (d + 63) / 64;
#define NF_ATT(T, DPL) \
  nf_launch((attention_generic_kernel<T, DPL>), dim3((unsigned)blocks), dim3(256), 0, s, a)
  if (dt == NF_F32) {
    if (dpl == 1) NF_ATT(float, 1); else if (dpl == 2) NF_ATT(float, 2); else NF_ATT(float, 4);
  } else {
    if (dpl == 1) NF_ATT(bf16_t, 1); else if (dpl == 2) NF_ATT(bf16_t, 2); else NF_ATT(bf16_t, 4);
  }
#undef NF_ATT
  return launched();
}

nf_status netfuse_attention_relpos(const void* Q, const void* K, const void* V, const void* Kr, const float* bias_w,
                                   const float* bias_r, const float* mask, void* O, int M, int B, int S, int heads,
                                   int d, long stride_m, long stride_row, float scale, nf_dtype dt, void* stream) {
  if (!Q || !K || !V || !Kr || !O) return NF_EINVAL;
  if (M <= 0 || B <= 0 || S <= 0 || heads <= 0 || d <= 0) return NF_EINVAL;
  if (!is_dtype(dt) || !(scale == scale)) return NF_EINVAL;
  const long long hd = (long long)heads * d;
  if (hd > INT_MAX || stride_row < hd) return NF_EINVAL;
  if (prod({B, S}) > INT_MAX / 2) return NF_EINVAL;
  if (stride_m < 0 || (M > 1 && stride_m < (long long)(B * (long long)S - 1) * stride_row + hd)) return NF_EINVAL;
  if (prod({M, B, S, hd}) >= kMaxElems || prod({M, stride_m}) >= kMaxElems || prod({M, 2, S, hd}) >= kMaxElems)
    return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(Q, esz) || !aligned(K, esz) || !aligned(V, esz) || !aligned(Kr, esz) || !aligned(O, esz) ||
      !aligned(mask, 4) || !aligned(bias_w, 4) || !aligned(bias_r, 4))
    return NF_EINVAL;
  if (d > 256) return NF_EUNSUPPORTED;
  const long long waves = prod({M, B, heads, S});
  const long long blocks = (waves + 3) / 4;
  if (blocks > kMaxGrid) return NF_EUNSUPPORTED;
  AttnRelArgs ra;
  AttnArgs& a = ra.a;
  a.Q = Q; a.K = K; a.V = V; a.mask = mask; a.O = O;
  a.M = M; a.B = B; a.S = S; a.heads = heads; a.d = d;
  a.stride_m = stride_m; a.stride_row = stride_row; a.scale = scale;
  ra.Kr = Kr; ra.bias_w = bias_w; ra.bias_r = bias_r;
  hipStream_t s = (hipStream_t)stream;
  if (dt == NF_BF16 && d == kAttnD && stride_row % 8 == 0 && stride_m % 8 == 0 && aligned(Q, 16) && aligned(K, 16) &&
      aligned(V, 16) && aligned(Kr, 16) && aligned(O, 8) && S <= (1 << 24)) {
    const int qblocks = (S + 127) / 128;
    const long long total = prod({M, B, heads, qblocks});
    if (total > kMaxGrid) return NF_EUNSUPPORTED;
    static std::atomic<bool> opted_in{false};          // 130 KB of LDS: one opt-in per process (idempotent)
    if (!opted_in.load(std::memory_order_acquire)) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(attention_relpos_mfma_d64_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kRelLdsBytes) != hipSuccess)
        return NF_ELAUNCH;
      opted_in.store(true, std::memory_order_release);
    }
    nf_launch(attention_relpos_mfma_d64_kernel, dim3((unsigned)total), dim3(256), kRelLdsBytes, s, ra, qblocks);
    return launched();
  }
  const int dpl = (d + 63) / 64;
#define NF_ATTR(T, DPL) nf_launch((attention_relpos_kernel<T, DPL>), dim3((unsigned)blocks), dim3(256), 0, s, ra)
  if (dt == NF_F32) {
    if (dpl == 1) NF_ATTR(float, 1); else if (dpl == 2) NF_ATTR(float, 2); else NF_ATTR(float, 4);
  } else {
    if (dpl == 1) NF_ATTR(bf16_t, 1); else if (dpl == 2) NF_ATTR(bf16_t, 2); else NF_ATTR(bf16_t, 4);
  }
#undef NF_ATTR
  return launched();
}

nf_status netfuse_maxpool2d(const void* x, void* y, int B, int Ctot, int H, int W, int k, int stride, int pad,
                            nf_dtype dt, void* stream) {
  if (!x || !y) return NF_EINVAL;
  if (B <= 0 || Ctot <= 0 || H <= 0 || W <= 0 || k <= 0 || stride <= 0 || pad < 0) return NF_EINVAL;
  if (pad >= k || !is_dtype(dt)) return NF_EINVAL;
  if ((long long)H + 2LL * pad < k || (long long)W + 2LL * pad < k) return NF_EINVAL;
  const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
  const long long n_in = prod({B, Ctot, H, W}), n_out = prod({B, Ctot, Ho, Wo});
  if (n_in >= kMaxElems || n_out >= kMaxElems) return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(x, esz) || !aligned(y, esz)) return NF_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  if (dt == NF_BF16 && k == 3 && stride == 2 && pad == 1 && W % 8 == 0 && aligned(x, 16) && aligned(y, 8)) {
    // Wo = W / 2 is a multiple of 4: four outputs per thread from 16-byte loads
    nf_launch(maxpool3x3s2_bf16_kernel, dim3(grid_for(n_out / 4, 256)), dim3(256), 0, s, (const bf16_t*)x,
                       (bf16_t*)y, H, W, Ho, Wo, (size_t)(n_out / 4));
    return launched();
  }
  const unsigned grid = grid_for(n_out, 256);
  if (dt == NF_F32)
    nf_launch(maxpool2d_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)x, (float*)y, H, W, Ho,
                       Wo, k, stride, pad, (size_t)n_out);
  else
    nf_launch(maxpool2d_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)x, (bf16_t*)y, H, W,
                       Ho, Wo, k, stride, pad, (size_t)n_out);
  return launched();
}

nf_status netfuse_avgpool_global(const void* x, void* y, int B, int Ctot, int HW, nf_dtype dt, void* stream) {
  if (!x || !y) return NF_EINVAL;
  if (B <= 0 || Ctot <= 0 || HW <= 0 || !is_dtype(dt)) return NF_EINVAL;
  if (prod({B, Ctot, HW}) >= kMaxElems) return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(x, esz) || !aligned(y, esz)) return NF_EINVAL;
  const long long nchan = (long long)B * Ctot;
  const long long blocks = (nchan + 3) / 4;
  if (blocks > kMaxGrid) return NF_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (HW <= 64) {
    const unsigned blocks16 = (unsigned)((nchan + 15) / 16);
    if (dt == NF_F32)
      nf_launch(avgpool_global_small_kernel<float>, dim3(blocks16), dim3(256), 0, s, (const float*)x,
                         (float*)y, (size_t)nchan, HW);
    else
      nf_launch(avgpool_global_small_kernel<bf16_t>, dim3(blocks16), dim3(256), 0, s, (const bf16_t*)x,
                         (bf16_t*)y, (size_t)nchan, HW);
    return launched();
  }
  if (dt == NF_F32)
    nf_launch(avgpool_global_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, (const float*)x,
                       (float*)y, (size_t)nchan, HW);
  else
    nf_launch(avgpool_global_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, s, (const bf16_t*)x,
                       (bf16_t*)y, (size_t)nchan, HW);
  return launched();
}

nf_status netfuse_merge_transpose(const void* src, void* dst, int M, int rows, int H, int to_channel, nf_dtype dt,
                                  void* stream) {
  if (!src || !dst || src == dst) return NF_EINVAL;
  if (M <= 0 || rows <= 0 || H <= 0 || !is_dtype(dt)) return NF_EINVAL;
  const long long total = prod({M, rows, H});
  if (total >= kMaxElems) return NF_EINVAL;
  const size_t esz = dt == NF_F32 ? 4 : 2;
  if (!aligned(src, esz) || !aligned(dst, esz)) return NF_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  // rows of H elements move as whole 16-byte vectors when they are made of them: the same index map over
  // H * esz / 16 vectors per row
  if (((size_t)H * esz) % 16 == 0 && aligned(src, 16) && aligned(dst, 16)) {
    const int Hv = (int)((size_t)H * esz / 16);
    const long long total_v = prod({M, rows, Hv});
    nf_launch(merge_transpose_kernel<uint4>, dim3(grid_for(total_v, 256)), dim3(256), 0, s, (const uint4*)src, (uint4*)dst,
              M, rows, Hv, to_channel != 0, (size_t)total_v);
    return launched();
  }
  const unsigned grid = grid_for(total, 256);
  if (dt == NF_F32)
    nf_launch(merge_transpose_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)src, (float*)dst,
                       M, rows, H, to_channel != 0, (size_t)total);
  else
    nf_launch(merge_transpose_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)src,
                       (bf16_t*)dst, M, rows, H, to_channel != 0, (size_t)total);
  return launched();
}

}  // extern "C"
