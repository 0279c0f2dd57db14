// bf16 MFMA contraction with a multi-stage, direct-to-LDS pipeline (gfx950): the kernel used when
// a problem is made of whole tiles (rows % BM == 0, cols % BN == 0, K % BK == 0, 16-byte aligned
// rows).  Same contract as gemm_mfma.h:  C[z][i][j] = sum_k A[z][i][k] * B[z][k][j] + epilogue,
// z = independent input-weight pairs folded into the grid.
//
// Global loads write straight into LDS (global_load_lds_dwordx4: each wavefront instruction moves
// 64 x 16 contiguous LDS bytes, every lane from its own global address), so no VGPR is spent on
// staging and NS-1 k-steps can be in flight per workgroup.  Because the LDS side of such a load is
// fixed (lane l -> byte 16 l of the 1 KB block), bank conflicts are avoided by permuting WHICH global
// 16-byte chunk a lane fetches (an XOR swizzle), not where it lands:
//   A tile [BM][BK] (k contiguous): chunk c of row r is stored at position c ^ s(r), s(r) = (r / 2) % 8
//     for 128-byte rows, (r / 4) % 4 for 64-byte rows, so the 16 rows hit by 16 neighbouring lanes of a
//     16-byte fragment read cover all 16 16-byte groups of the 64 banks.
//   B tile [BK][BN] (column contiguous): chunk c of row k is stored at position c ^ 4 (k % 4), so the
//     4 rows x 64 bytes touched by 32 neighbouring lanes of a transposing read (ds_read_b64_tr_b16)
//     fall into distinct banks (no permutation where the row pitch itself is 64 or 192 bytes modulo 256).
// Waiting is explicit: a thread's loads retire in order, so "stage kt has landed" is
// s_waitcnt vmcnt(loads issued after it); a workgroup barrier then publishes every thread's share
// and, at the same time, proves that the stage read in the previous step is free to be refilled.
#pragma once
#include "gemm_mfma.h"

namespace nf {

typedef __attribute__((address_space(3))) unsigned char lds_u8_t;
typedef __attribute__((address_space(1))) const unsigned char glb_u8_t;

// Cache policy of the weight loads (aux operand of global_load_lds: 1 = sc0, 2 = nt, 16 = sc1).  Weights are
// read exactly once per forward pass and are 20 times the size of the activations of a layer, so they are
// loaded non-temporal: they then do not displace the activations that the previous operator has just left in
// the memory-side cache (256 MB) and that the next one is about to read.  Measured on the operator sequence of
// one encoder layer at 32 models (us per kernel, default policy -> nt): 768 -> 2304 matmul 33.9 -> 28.2,
// 768 -> 3072 + GELU 45.0 -> 38.9, 3072 -> 768 45.1 -> 38.4, whole layer 167 -> 150; sc1 changes nothing.  A
// kernel timed alone in a loop does not show this: its own output then never leaves that cache.
#ifndef NF_B_CPOL
#define NF_B_CPOL 2
#endif
constexpr int kWeightCpol = NF_B_CPOL;

template <int BM, int BN, int BK, int WGM, int WGN, int NS>
struct DmaCfg {
  static_assert(BK == 32 || BK == 64, "k-step of 32 or 64");
  static constexpr int kBM = BM, kBN = BN, kBK = BK, kWGM = WGM, kWGN = WGN, kNS = NS;
  static constexpr int kNW = WGM * WGN, kThreads = kNW * kWave;
  static constexpr bool kRowConsts = false;              // matmul epilogues carry per-column constants only
  static constexpr int WM = BM / WGM, WN = BN / WGN, FM = WM / 32, FN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
  static constexpr int kARow = BK * 2, kBRow = BN * 2;                 // bytes per LDS row
  static constexpr int kABytes = BM * kARow, kBBytes = BK * kBRow, kStageBytes = kABytes + kBBytes;
  // A stage is kBlocks load instructions of 1 KB (A blocks first, then B), dealt to the wavefronts round
  // robin: wave w issues blocks w, w + kNW, ...; when kNW does not divide kBlocks the first kRem waves
  // issue one more than the others.
  static constexpr int kABlocks = kABytes / 1024, kBBlocks = kBBytes / 1024, kBlocks = kABlocks + kBBlocks;
  static_assert(kABlocks * 1024 == kABytes && kBBlocks * 1024 == kBBytes, "tiles are whole 1 KB blocks");
  static constexpr int kMaxPer = (kBlocks + kNW - 1) / kNW, kRem = kBlocks % kNW;
  static_assert(NS >= 3, "NS-1 stages are in flight while one is multiplied");
  static_assert((NS - 2) * kMaxPer < 64, "vmcnt has 6 bits");
  static constexpr int kEpiPitch = BN + 4;
  static constexpr int kLdsEpi = WGM * 32 * kEpiPitch * (int)sizeof(float);
  static constexpr int kLdsPipe = NS * kStageBytes;
  static constexpr int kLdsBytes = kLdsPipe > kLdsEpi ? kLdsPipe : kLdsEpi;
  static_assert(kLdsBytes <= 160 * 1024, "pipeline stages and epilogue staging must fit the 160 KB of LDS");
  static constexpr int kACpr = BK / 8, kARpi = 64 / kACpr;              // A: chunks per row, rows per instruction
  static constexpr int kBCpr = BN / 8;                                  // B: chunks per row (rows need not divide 64)
  static_assert(BN % 32 == 0, "whole 32-column MFMA blocks");
  // LDS serves 256 bytes per clock (64 banks): a 16-byte read is processed 16 lanes at a time, a
  // transposing 8-byte read 32 lanes at a time, and the lanes of one such group must cover distinct banks.
  static constexpr int kARowsPer256 = 256 / kARow;                      // A rows that share one bank span
  __device__ static __forceinline__ int swz_a(int row) { return (row / kARowsPer256) % kACpr; }
  // B rows whose pitch is 64 or 192 bytes modulo 256 (BN = 96, 288) need no permutation: four consecutive
  // k rows already start 64 bytes apart in the banks.  Otherwise chunk ^= 4 (k % 4), which stays in the row
  // when rows are whole groups of 16 chunks.
  static constexpr bool kBNatural = kBRow % 256 == 64 || kBRow % 256 == 192;
  static_assert(kBNatural || kBCpr % 16 == 0, "B rows are permuted in units of 16 chunks");
  static constexpr int kBSwz = kBNatural ? 0 : 4;
};

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their "don't wait" maxima).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// only the LDS / scalar-memory counter constrained (vmcnt left at its maximum)
__device__ __forceinline__ void wait_lgkmcnt0() {
  __builtin_amdgcn_s_waitcnt((63 & 15) | ((63 >> 4) << 14) | (7 << 4) | (0 << 8));
}

// The A operand of a weight-streaming matmul is small (the model's activation rows) but is re-read by
// every column tile and k-step, and it was written by the previous operator, so it starts out in no L2.
// Each of the `parts` workgroups that share an A tile (the column tiles of one model and row tile, which run
// on one XCD) reads one part of its rows once, right after its first pipeline stages are on their way,
// k-ascending, and discards the data: the rows are then L2 hits for every later k-step of all of them.
// Measured on the 12-layer encoder at 32 models: 768 -> 3072 matmul 42.7 -> 37.9 us, 768 -> 2304 32.4 -> 28.9,
// whole forward 1.855 -> 1.733 ms.  (Timed alone in a loop on a never rewritten input the kernels do not
// show this: the input then stays in L2 from one launch to the next.)
// Only launches whose workgroups are all resident at once (one per compute unit) and whose A operands fit
// the L2 of an XCD beside the weight stream do this: 512 x 3072 activations per model (four models per XCD:
// 12 MB against 4 MB of L2) measured 10 % slower with it, as did launches of several rounds of workgroups.
// At 3 MB per XCD (128 x 3072 per model, the 3072 -> 768 matmul) it still pays, if less: 41.2 -> 39.0 us behind
// the matmul that wrote the operand (34 us on a never rewritten one: part of the lines is evicted by the
// weight stream before its use).
#ifndef NF_A_TOUCH
#define NF_A_TOUCH 1
#endif
// (A rolling variant for larger operands -- one wavefront touching each k-slab a few steps ahead of the
// pipeline -- measured slower: 3072 -> 768 at 128 rows 44 -> 58 us; the cold touches sit in that wavefront's
// in-order memory queue in front of its own pipeline stages.)
inline bool touch_a_pays(long long workgroups, long long a_elems_per_problem, long long problems) {
  const long long per_xcd = (problems + kNumXcd - 1) / kNumXcd * a_elems_per_problem * 2;      // bytes
  return workgroups <= 256 && per_xcd <= (3 << 20);
}
template <class Cfg>
__device__ __forceinline__ void touch_a_rows(const bf16_t* A, long lda, int K, int part, int parts) {
#if NF_A_TOUCH
  if (parts <= 0) return;
  const int rows_per = (Cfg::kBM + parts - 1) / parts;
  const int row_lo = part * rows_per, row_hi = min(Cfg::kBM, row_lo + rows_per);
  const int cpr = K / 64;                                  // 128-byte lines per row
  const int n = (row_hi - row_lo) * cpr;
  for (int c = threadIdx.x; c < n; c += Cfg::kThreads) {
    const int r = row_lo + c % (row_hi - row_lo), kc = c / (row_hi - row_lo);      // k-major: early k first
    uint32_t v = *(const volatile uint32_t*)(A + (long)r * lda + kc * 64);
    asm volatile("" ::"v"(v));
  }
#endif
}

template <class Cfg>
__device__ __forceinline__ void gemm_dma_tile(const bf16_t* __restrict__ A, long lda, const bf16_t* __restrict__ B,
                                              long ldb, int K, lds_u8_t* smem, bf16_t* C, const bf16_t* R,
                                              long ldc, const Epilogue& ep, long row_vec_off, long col_vec_off,
                                              int a_touch_part = 0, int a_touch_parts = 0) {
  constexpr int FM = Cfg::FM, FN = Cfg::FN, NS = Cfg::kNS, BK = Cfg::kBK;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / Cfg::kWGN, wn = wave % Cfg::kWGN;
  const int half = lane / 32, l32 = lane % 32, l16 = lane % 16;

  // ---- what this lane fetches: the global address of its 16-byte chunk of each of its blocks, advanced
  // by one k-step after every issue (stages are issued in order)
  const bf16_t* src[Cfg::kMaxPer];
  long inc[Cfg::kMaxPer];
#pragma unroll
  for (int t = 0; t < Cfg::kMaxPer; ++t) {
    const int blk = t * Cfg::kNW + wave;
    if (blk < Cfg::kABlocks) {
      const int row = blk * Cfg::kARpi + lane / Cfg::kACpr;
      const int c = (lane % Cfg::kACpr) ^ Cfg::swz_a(row);
      src[t] = A + (long)row * lda + c * 8;
      inc[t] = BK;
    } else {
      const int flat = (blk - Cfg::kABlocks) * 64 + lane;    // chunk index in the row-major [BK][BN] LDS tile
      const int krow = flat / Cfg::kBCpr;
      const int c = (flat % Cfg::kBCpr) ^ (Cfg::kBSwz * (krow % 4));
      src[t] = B + (long)krow * ldb + c * 8;
      inc[t] = (long)BK * ldb;
    }
  }
  const bool extra = Cfg::kRem == 0 || wave < Cfg::kRem;     // this wave issues kMaxPer loads per stage (else one less)
  auto issue_stage = [&](int kt) {
    lds_u8_t* stage = smem + (kt % NS) * Cfg::kStageBytes;
#pragma unroll
    for (int t = 0; t < Cfg::kMaxPer; ++t) {
      if (t + 1 < Cfg::kMaxPer || extra)
        {
          // A blocks (activations, re-read by every column tile of the model) keep the default policy;
          // B blocks (weights, read exactly once per forward pass) take kWeightCpol
          if (t * Cfg::kNW + wave < Cfg::kABlocks)
            __builtin_amdgcn_global_load_lds((glb_u8_t*)src[t], stage + (t * Cfg::kNW + wave) * 1024, 16, 0, 0);
          else
            __builtin_amdgcn_global_load_lds((glb_u8_t*)src[t], stage + (t * Cfg::kNW + wave) * 1024, 16, 0, kWeightCpol);
        }
      src[t] += inc[t];
    }
  };
  // stage kt has landed once at most the loads of the NS-2 younger stages are pending
  auto wait_landed = [&]() {
    if (extra) wait_vmcnt<(NS - 2) * Cfg::kMaxPer>(); else wait_vmcnt<(NS - 2) * (Cfg::kMaxPer - 1)>();
  };

  // ---- where this lane reads its fragments (byte offsets inside a stage, k-step part added later)
  int a_off[FM], b_off[FN][2];
#pragma unroll
  for (int i = 0; i < FM; ++i) a_off[i] = (wm * Cfg::WM + i * 32 + l32) * Cfg::kARow;
  const int a_swz = Cfg::swz_a(l32);                  // row offsets above are multiples of 32: same swizzle
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int hl = 0; hl < 2; ++hl) {
      const int kr = 8 * half + l16 / 4 + 4 * hl;     // row inside a 16-k step; kr % 4 = l16 / 4
      const int n = wn * Cfg::WN + j * 32 + ((lane / 16) % 2) * 16 + (l16 % 4) * 4;
      b_off[j][hl] = Cfg::kABytes + kr * Cfg::kBRow + (((n / 8) ^ (Cfg::kBSwz * (l16 / 4))) * 16) + ((n / 4) % 2) * 8;
    }
  // byte offset of the kk-th 16-k step of a stage's B region
  auto b_step = [](int kk) {
    return kk * 16 * Cfg::kBRow;
  };

  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = K / BK;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < nk) issue_stage(s);
  touch_a_rows<Cfg>(A, lda, K, a_touch_part, a_touch_parts);

  for (int kt = 0; kt < nk; ++kt) {
    // near the end fewer stages were issued, so wait for everything
    if (kt + NS - 2 < nk) wait_landed(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    const lds_u8_t* stage = smem + (kt % NS) * Cfg::kStageBytes;
    // All fragments of the k-step are read BEFORE the next stage's loads are issued: LDS reads that a
    // wave issues behind its own fresh direct-to-LDS loads are held up by them (measured: 20 % of the
    // kernel on weight-streaming shapes), whereas the loads lose nothing by starting one LDS latency later.
    bf16x8_t af[BK / 16][FM], bfr[BK / 16][FN];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
      for (int i = 0; i < FM; ++i)
        af[kk][i] = *(const lds_bf16x8_t*)(stage + a_off[i] + (((2 * kk + half) ^ a_swz) * 16));
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(stage + b_off[j][0] + b_step(kk)));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(stage + b_off[j][1] + b_step(kk)));
        const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bfr[kk][j] = __builtin_bit_cast(bf16x8_t, both);
      }
    }
    // The multiplications start as soon as the fragments of the first 16-k slice are there; the next stage's
    // loads are issued behind the last slice (they refill the stage read in step kt-1).
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk][j], af[kk][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (kt + NS - 1 < nk) issue_stage(kt + NS - 1);
    __builtin_amdgcn_sched_barrier(0);
  }
  __syncthreads();   // every wave is done with the last stage before the epilogue reuses LDS
  gemm_epilogue<Cfg>(acc, (lds_f32_t*)smem, C, R, ldc, Cfg::kBM, Cfg::kBN, ep, row_vec_off, col_vec_off);
}

}  // namespace nf
