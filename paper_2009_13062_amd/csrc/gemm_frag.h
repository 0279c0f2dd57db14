// Merged matmul on FRAGMENT-PACKED weights (netfuse_linear_pack_weight): the weight operand goes from HBM
// straight into the registers of the one wavefront that multiplies it, already in the lane layout of the MFMA
// operand; only the activations (the small operand, re-read from L2) pass through LDS.
//
// Why: with the row-major [K][Nout] weight layout every weight fragment has to be transposed on its way into
// the MFMA operand, which on gfx950 is a transposing 8-byte LDS read.  Measured, LDS serves 16-byte reads at
// ~275 bytes per clock and compute unit but 8-byte reads (plain or transposing) at ~85, so at 128 rows per model
// the direct-to-LDS kernels (gemm_dma.h) spend about as long reading fragments back out of LDS as HBM needs to
// deliver the weights, and all waves do it in lock-step between two barriers.  Weights are static at inference
// (Section 3.1: the merged weight tensor is built once), so the transposition is done once, offline:
//
//   Wp[z][j][s][lane][e] = W[z][16 s + 8 (lane / 32) + e][32 j + lane % 32]     j < Nout/32, s < K/16, e < 8
//
// i.e. for every 32-column block j the K/16 operand fragments (1 KB each: 64 lanes x 16 bytes) follow one
// another down k.  A wavefront that owns column block j then streams one contiguous run of memory with
// plain 16-byte register loads (non-temporal: the weights are read once per forward pass), NS k-stages ahead.
//
// Workgroup = one (problem, tile of RB 32-row blocks -- 128 rows, or 64 where 128-row tiles would leave
// compute units idle --, tile of NB column blocks), NB x KG wavefronts: wavefront (q, j) owns
// column block j and, of every k-stage of 16 KG U columns of k, the U 16-k slices q U ... q U + U - 1; it
// multiplies them with all RB 32-row blocks of the A stage (RB 16-byte LDS reads per slice, shared by
// nobody: every weight fragment is used by exactly one wavefront, so nothing about B is ever shared).  With
// KG > 1 (narrow tiles: Nout = 768 gives one tile per compute unit only at 96 columns) the KG partial sums of a
// 32 x 32 block are added through LDS after the loop, in ascending k-group order, each wavefront finishing one
// row block.  The epilogue runs out of registers (gemm_stream.h).
//
// Waiting: a wavefront's vector-memory operations retire in issue order; per stage it issues NA direct-to-LDS
// loads of A and then U register loads of B, so "stage g is here" is vmcnt <= (stages issued since) x (NA + U).
// The loop is unrolled over the NS stages of the ring (static register slots) and compiled twice, for the
// wavefronts that issue one more A load per stage than the others, so that every count is a constant.
#pragma once
#include "gemm_stream.h"

namespace nf {

template <int NB, int KG, int U, int NS, int RB = 4>
struct FragCfg {
  static constexpr int kNB = NB, kKG = KG, kU = U, kNS = NS, kRB = RB;      // RB: 32-row blocks per tile
  static constexpr int kBM = 32 * RB, kBN = 32 * NB, kBK = 16 * KG * U;
  static_assert(KG == 1 || KG == RB, "with a split k every k-group finishes one 32-row block");
  static_assert(kBK == 32 || kBK == 64, "A stage rows of 64 or 128 bytes");
  static constexpr int kNW = NB * KG, kThreads = kNW * kWave;
  static constexpr int kARow = kBK * 2, kStageBytes = kBM * kARow;       // A stage: [128][BK] bf16, chunks permuted
  static constexpr int kABlocks = kStageBytes / 1024;                   // 1 KB direct-to-LDS loads per stage
  static constexpr int kNAHi = (kABlocks + kNW - 1) / kNW, kRem = kABlocks % kNW;   // waves < kRem (or all) issue kNAHi
  static constexpr int kACpr = kBK / 8, kARpi = 64 / kACpr;             // chunks per row, rows per load
  static constexpr int kARowsPer256 = 256 / kARow;
  __device__ static __forceinline__ int swz_a(int row) { return (row / kARowsPer256) % kACpr; }
  static constexpr int kLdsPipe = NS * kStageBytes;
  static constexpr int kLdsReduce = KG > 1 ? kNW * (KG - 1) * 4096 : 0;   // (KG-1) partial 32x32 fp32 blocks per wave
  static constexpr int kTouchOff = kLdsPipe > kLdsReduce ? kLdsPipe : kLdsReduce;     // 256 bytes per wave that nobody reads
  static constexpr int kLdsBytes = kTouchOff + kNW * 256;
  static_assert(kLdsBytes <= 160 * 1024, "LDS");
  static_assert((NS - 2) * (kNAHi + U) < 64, "vmcnt has 6 bits");
};

template <int R, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (R < N) {
    f(std::integral_constant<int, R>{});
    static_for<R + 1, N>(f);
  }
}

// One 128 x (32 NB) tile.  A: the tile's first row; Bw: this problem's packed weights at column block 0 of the
// tile (element pointer); C, R, col_bias at the tile's first column.  K a multiple of NS stages.
template <class Cfg, int NA>
__device__ __forceinline__ void gemm_frag_loop(const bf16_t* __restrict__ A, long lda, const bf16_t* __restrict__ bsrc,
                                               int nstage, lds_u8_t* smem, f32x16_t (&acc)[Cfg::kRB], int wave, int lane,
                                               int q, int a_touch_part, int a_touch_parts, int K) {
  constexpr int NS = Cfg::kNS, U = Cfg::kU, BK = Cfg::kBK, NW = Cfg::kNW, RB = Cfg::kRB;
  const int half = lane / 32, l32 = lane % 32;

  const bf16_t* asrc[NA > 0 ? NA : 1];
#pragma unroll
  for (int t = 0; t < NA; ++t) {
    const int blk = t * NW + wave;
    const int row = blk * Cfg::kARpi + lane / Cfg::kACpr;
    const int c = (lane % Cfg::kACpr) ^ Cfg::swz_a(row);
    asrc[t] = A + (long)row * lda + c * 8;
  }
  u32x4_t bq[NS][U];
  auto issue_stage = [&](int slot) {
    lds_u8_t* stage = smem + slot * Cfg::kStageBytes;
#pragma unroll
    for (int t = 0; t < NA; ++t) {
      __builtin_amdgcn_global_load_lds((glb_u8_t*)asrc[t], stage + (t * NW + wave) * 1024, 16, 0, 0);
      asrc[t] += BK;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      // Issued behind the compiler's back: its own wait-count bookkeeping gives up on register loads that are
      // consumed an iteration later (a full vmcnt(0) at every loop head); the waits are the explicit ones in
      // consume().  The destination registers are touched by nothing else until then.
      asm volatile("global_load_dwordx4 %0, %1, off nt" : "=&v"(bq[slot][u]) : "v"(bsrc + u * 512) : "memory");
    bsrc += (long)Cfg::kKG * U * 512;                       // the next stage's slices of this k-group
  };
  int a_off[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i) a_off[i] = (i * 32 + l32) * Cfg::kARow;
  const int a_swz = Cfg::swz_a(l32);

  // consume the stage in ring slot r; LEFT = stages issued after it that may still be in flight
  auto consume = [&](int r, auto left_tag) {
    constexpr int LEFT = decltype(left_tag)::value;
    wait_vmcnt<LEFT * (NA + U)>();
    __builtin_amdgcn_s_barrier();
    const lds_u8_t* stage = smem + r * Cfg::kStageBytes;
    bf16x8_t af[U][RB];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int i = 0; i < RB; ++i)
        af[u][i] = *(const lds_bf16x8_t*)(stage + a_off[i] + (((2 * (q * U + u) + half) ^ a_swz) * 16));
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bf16x8_t bf = __builtin_bit_cast(bf16x8_t, bq[r][u]);
#pragma unroll
      for (int i = 0; i < RB; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, af[u][i], acc[i], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

#pragma unroll
  for (int s = 0; s < NS - 1; ++s) issue_stage(s);
  if (a_touch_parts > 0) {
    // The touches of touch_a_rows (gemm_dma.h: this workgroup's share of the tile's A rows, pulled into L2 once
    // for all column tiles of the model), issued as direct-to-LDS loads into a dump area: with no destination
    // register there is nothing that has to wait for them before the loop starts (headline forward 1.668 ->
    // 1.659 ms).  They sit in the in-order queue in front of the last prologue stage, so the explicit counts
    // of consume() only become conservative until they have retired.
    const int rows_per = (Cfg::kBM + a_touch_parts - 1) / a_touch_parts;
    const int row_lo = a_touch_part * rows_per, row_hi = min(Cfg::kBM, row_lo + rows_per);
    const int nrow = row_hi - row_lo, n = nrow * (K / 64);
    lds_u8_t* dump = smem + Cfg::kTouchOff + wave * 256;
    for (int c0 = 0; c0 < n; c0 += Cfg::kThreads) {
      const int c = c0 + (int)threadIdx.x;                  // k-major: early k first
      if (c < n)
        __builtin_amdgcn_global_load_lds((glb_u8_t*)(A + (long)(row_lo + c % nrow) * lda + (c / nrow) * 64), dump, 4, 0, 0);
    }
  }

  // every macro step consumes NS stages; all but the last one refill each slot right after the slot before it
  // has been consumed (the barrier of step g proves that every wave is done with stage g-1)
  for (int g0 = 0; g0 + NS < nstage; g0 += NS) {
#pragma unroll
    for (int r = 0; r < NS; ++r) {
      consume(r, std::integral_constant<int, NS - 2>{});
      issue_stage((r + NS - 1) % NS);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // last macro step: only stage nstage-1 is still to be issued
  static_assert(NS >= 3, "ring");
  consume(0, std::integral_constant<int, NS - 2>{});
  issue_stage(NS - 1);
  __builtin_amdgcn_sched_barrier(0);
  static_for<0, NS - 1>([&](auto rr) {
    constexpr int R = decltype(rr)::value;
    consume(R + 1, std::integral_constant<int, NS - 2 - R>{});
  });
}

template <class Cfg>
__device__ __forceinline__ void gemm_frag_tile(const bf16_t* __restrict__ A, long lda, const bf16_t* __restrict__ Bw,
                                               int K, lds_u8_t* smem, bf16_t* C, const bf16_t* R, long ldc,
                                               const float* col_bias, int act, int a_touch_part, int a_touch_parts) {
  constexpr int NB = Cfg::kNB, KG = Cfg::kKG, U = Cfg::kU, RB = Cfg::kRB;
  const int lane = threadIdx.x % kWave;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int q = wave / NB, j = wave % NB;

  f32x16_t acc[RB];
#pragma unroll
  for (int i = 0; i < RB; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  // fragment (j, s) starts at ((j * K/16) + s) * 512 elements; this wave's first slice is s = q U
  const bf16_t* bsrc = Bw + ((long)j * (K / 16) + q * U) * 512 + lane * 8;
  const int nstage = K / Cfg::kBK;
  if (Cfg::kRem == 0 || wave < Cfg::kRem)
    gemm_frag_loop<Cfg, Cfg::kNAHi>(A, lda, bsrc, nstage, smem, acc, wave, lane, q, a_touch_part, a_touch_parts, K);
  else
    gemm_frag_loop<Cfg, Cfg::kNAHi - 1>(A, lda, bsrc, nstage, smem, acc, wave, lane, q, a_touch_part, a_touch_parts, K);

  if constexpr (KG == 1) {
    f32x16_t (&acc2)[RB][1] = reinterpret_cast<f32x16_t (&)[RB][1]>(acc);
    if (act == NF_ACT_GELU) reg_epilogue<RB, 1, NF_ACT_GELU>(acc2, C, R, ldc, col_bias, 0, 32 * j);
    else if (act == NF_ACT_RELU) reg_epilogue<RB, 1, NF_ACT_RELU>(acc2, C, R, ldc, col_bias, 0, 32 * j);
    else reg_epilogue<RB, 1, NF_ACT_NONE>(acc2, C, R, ldc, col_bias, 0, 32 * j);
  } else {
    // Partial sums of row block i go to wavefront (i, j): region of wave d = i NB + j, then [slot][r4][lane] x 16 B,
    // slot = the sender's k-group with the receiver's own left out.
    __builtin_amdgcn_s_barrier();                           // every wave is done reading the A stages
    lds_f32_t* red = (lds_f32_t*)smem;
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      if (i == q) continue;
      const int slot = q < i ? q : q - 1;
      lds_f32_t* dst = red + ((size_t)(i * NB + j) * (KG - 1) + slot) * 1024;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        *(lds_f32x4_t*)(dst + (r4 * 64 + lane) * 4) =
            f32x4v_t{acc[i][4 * r4], acc[i][4 * r4 + 1], acc[i][4 * r4 + 2], acc[i][4 * r4 + 3]};
    }
    __syncthreads();
    f32x16_t own, sum[1][1];
#pragma unroll
    for (int i = 0; i < RB; ++i)
      if (i == q) own = acc[i];
    const lds_f32_t* src = red + (size_t)wave * (KG - 1) * 1024;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum[0][0][r] = 0.f;
#pragma unroll
    for (int g = 0; g < KG; ++g) {                          // ascending k-group order
      if (g == q) {
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[0][0][r] += own[r];
      } else {
        const int slot = g < q ? g : g - 1;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4v_t p = *(const lds_f32x4_t*)(src + slot * 1024 + (r4 * 64 + lane) * 4);
          sum[0][0][4 * r4] += p.x; sum[0][0][4 * r4 + 1] += p.y; sum[0][0][4 * r4 + 2] += p.z; sum[0][0][4 * r4 + 3] += p.w;
        }
      }
    }
    if (act == NF_ACT_GELU) reg_epilogue<1, 1, NF_ACT_GELU>(sum, C, R, ldc, col_bias, 32 * q, 32 * j);
    else if (act == NF_ACT_RELU) reg_epilogue<1, 1, NF_ACT_RELU>(sum, C, R, ldc, col_bias, 32 * q, 32 * j);
    else reg_epilogue<1, 1, NF_ACT_NONE>(sum, C, R, ldc, col_bias, 32 * q, 32 * j);
  }
}

}  // namespace nf
