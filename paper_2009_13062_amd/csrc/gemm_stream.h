// Streaming form of the direct-to-LDS bf16 MFMA contraction (gemm_dma.h) for the merged matmul: one
// workgroup computes NSUB consecutive column tiles of one (problem, row tile) through ONE continuous load
// pipeline, and each tile's epilogue runs out of registers while the next tile's operands are already
// landing in LDS.
//
// Why: measured on MI355X, a weight-streaming matmul (128 rows per model) spends a quarter to a third of
// its time in the epilogue of its single tile per compute unit -- bias, GELU and the bf16 conversion are
// 60-80 VALU clocks per element with nothing else in flight, and the staging of the accumulators through
// LDS adds four workgroup barriers -- while the same operand stream without any epilogue runs at the rate of
// a plain read kernel (6 TB/s).  Here
//   * the epilogue touches no LDS and no barrier: a lane owns groups of 4 consecutive columns of a row (the
//     accumulators are computed transposed); the two lanes of a row swap half of their groups so that each
//     holds 8 consecutive columns, loads 16 bytes of residual, converts and stores 16 bytes;
//   * the load pipeline never drains between the tiles of a workgroup: the stage counter runs over
//     NSUB x K/BK steps, the source pointers jump to the next tile after a tile's last k-step, so
//     NS-1 stages of the NEXT tile are in flight during an epilogue, and every wave starts the next tile
//     as soon as it is done with its own part of the epilogue;
//   * the A operand (the model's activation rows) is re-read per column tile, from L2.
// Bit-for-bit the same result as the other contraction kernels: same k order, same epilogue arithmetic.
#pragma once
#include "gemm_dma.h"

namespace nf {

// Epilogue of one whole BM x BN tile straight from the accumulators (layout: see gemm_mfma.h): a lane holds,
// per 32 x 32 block, four groups of 4 consecutive columns of its row (columns 8 q + 4 half + 0..3).  The two
// lanes of a row (lane and lane + 32) swap one group per pair of groups, after the activation, so that each
// ends up with 8 consecutive columns: residual and output then move 16 bytes per lane (8-byte stores
// measured 1.4x the algorithmic write traffic: partially written sectors reaching HBM).
// Needs 16-byte aligned rows of C and R (ldc % 8 == 0) and a 16-byte aligned column-constant vector.
// acc[i][j] is the 32 x 32 block at rows row_base + 32 i, columns col_base + 32 j of the tile that C, R and col_bias
// point at.
template <int FM, int FN, int ACT>
__device__ __forceinline__ void reg_epilogue(f32x16_t (&acc)[FM][FN], bf16_t* C, const bf16_t* R, long ldc,
                                             const float* col_bias, int row_base, int col_base) {
  const int lane = threadIdx.x % kWave;
  const int half = lane / 32, l32 = lane % 32;
  // Row blocks outermost: the column blocks of a row block are stored one right after the other, so the 64-byte
  // halves of a 128-byte output line (two neighbouring column blocks of one wavefront) reach L2 close together.
  // With the column blocks outermost they were four row blocks of epilogue arithmetic apart, and L2 wrote a
  // third of the lines back half filled: 135.7 MB written for a 100.7 MB output (768 -> 3072 + GELU at 512 rows
  // and 32 models), 120 us against 108 us this way.
  float4 cball[FN][4];
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q)
      cball[j][q] = col_bias ? *reinterpret_cast<const float4*>(col_bias + col_base + j * 32 + q * 8 + half * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int colb = col_base + j * 32;
      float4 (&cb)[4] = cball[j];
      // this lane's two 8-column pieces: columns colb + 16 qq + 8 half + 0..7
      const long off = (long)(row_base + i * 32 + l32) * ldc + colb + half * 8;
      uint4 rr[2];
#pragma unroll
      for (int qq = 0; qq < 2; ++qq)
        rr[qq] = R ? *reinterpret_cast<const uint4*>(R + off + qq * 16) : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
      for (int qq = 0; qq < 2; ++qq) {
        float own[4], send[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // group 2 qq + half stays (its other half comes from the partner), group 2 qq + 1 - half is sent
          const float b0[4] = {cb[2 * qq].x, cb[2 * qq].y, cb[2 * qq].z, cb[2 * qq].w};
          const float b1[4] = {cb[2 * qq + 1].x, cb[2 * qq + 1].y, cb[2 * qq + 1].z, cb[2 * qq + 1].w};
          // (an accumulator is never -0 -- it starts at +0 and (+0) + (-0) = +0 -- so neither is the sum, and the
          // "+ 0, x 1 + 0" steps with which the other epilogues normalise a -0 would change no bit here)
          const float v0 = act_const<ACT>(acc[i][j][(2 * qq) * 4 + e] + b0[e]);
          const float v1 = act_const<ACT>(acc[i][j][(2 * qq + 1) * 4 + e] + b1[e]);
          own[e] = half ? v1 : v0;
          send[e] = half ? v0 : v1;
        }
        float recv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) recv[e] = __shfl_xor(send[e], 32, kWave);
        // columns within the piece: the lower lane's group sits at 4 half' ... : half 0 holds columns 0..3 of its
        // group and receives 4..7; half 1 holds 4..7 and receives 0..3
        float v[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = half ? recv[e] : own[e];
          v[4 + e] = half ? own[e] : recv[e];
        }
        const uint32_t w[4] = {rr[qq].x, rr[qq].y, rr[qq].z, rr[qq].w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          o[e] = pack_bf16x2(v[2 * e] + __uint_as_float(w[e] << 16), v[2 * e + 1] + __uint_as_float(w[e] & 0xffff0000u));
        *reinterpret_cast<uint4*>(C + off + qq * 16) = make_uint4(o[0], o[1], o[2], o[3]);
      }
    }
  }
}

template <class Cfg, int ACT>
__device__ __forceinline__ void stream_epilogue_act(f32x16_t (&acc)[Cfg::FM][Cfg::FN], bf16_t* C, const bf16_t* R,
                                                    long ldc, const float* col_bias) {
  const int wave = threadIdx.x / kWave;
  reg_epilogue<Cfg::FM, Cfg::FN, ACT>(acc, C, R, ldc, col_bias, (wave / Cfg::kWGN) * Cfg::WM, (wave % Cfg::kWGN) * Cfg::WN);
}

// A, B, C, R, col_bias point at the workgroup's first tile; consecutive tiles are b_tile_stride elements
// apart in B and Cfg::kBN columns apart in C, R and col_bias.  act is applied before the residual.
//
// PB (fragment-packed weights, pack_kernels.h): B points at the first fragment of the workgroup's first column
// block; a stage's B part is the (BN / 32) x (BK / 16) fragments of 1 KB of the tile's column blocks and the
// stage's k slices, each fetched by one direct-to-LDS load (64 lanes x 16 contiguous bytes) and read back as it
// lies with one 16-byte LDS read per lane: no transposing read (a third of the rate of 16-byte reads) and
// no bank conflicts by construction.  ldb is unused; b_tile_stride = BN x K elements.
template <class Cfg, bool PB = false>
__device__ __forceinline__ void gemm_stream_tiles(const bf16_t* __restrict__ A, long lda, const bf16_t* __restrict__ B,
                                                  long ldb, long b_tile_stride, int K, int nsub, lds_u8_t* smem,
                                                  bf16_t* C, const bf16_t* R, long ldc, const float* col_bias,
                                                  int act, int a_touch_part = 0, int a_touch_parts = 0) {
  constexpr int FM = Cfg::FM, FN = Cfg::FN, NS = Cfg::kNS, BK = Cfg::kBK;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / Cfg::kWGN, wn = wave % Cfg::kWGN;
  const int half = lane / 32, l32 = lane % 32, l16 = lane % 16;
  const int nk = K / BK;

  // ---- what this lane fetches (as gemm_dma_tile), plus the pointer jump after a tile's last k-step
  const bf16_t* src[Cfg::kMaxPer];
  long inc[Cfg::kMaxPer], jump[Cfg::kMaxPer];
#pragma unroll
  for (int t = 0; t < Cfg::kMaxPer; ++t) {
    const int blk = t * Cfg::kNW + wave;
    if (blk < Cfg::kABlocks) {
      const int row = blk * Cfg::kARpi + lane / Cfg::kACpr;
      const int c = (lane % Cfg::kACpr) ^ Cfg::swz_a(row);
      src[t] = A + (long)row * lda + c * 8;
      inc[t] = BK;
      jump[t] = -(long)(nk - 1) * BK;                        // back to k = 0 of the same rows
    } else if constexpr (PB) {
      const int bb = blk - Cfg::kABlocks;                    // fragment (column block bb / (BK/16), slice bb % (BK/16))
      src[t] = B + ((long)(bb / (BK / 16)) * (K / 16) + bb % (BK / 16)) * 512 + lane * 8;
      inc[t] = (BK / 16) * 512;
      jump[t] = b_tile_stride - (long)(nk - 1) * inc[t];
    } else {
      const int flat = (blk - Cfg::kABlocks) * 64 + lane;
      const int krow = flat / Cfg::kBCpr;
      const int c = (flat % Cfg::kBCpr) ^ (Cfg::kBSwz * (krow % 4));
      src[t] = B + (long)krow * ldb + c * 8;
      inc[t] = (long)BK * ldb;
      jump[t] = b_tile_stride - (long)(nk - 1) * inc[t];
    }
  }
  const bool extra = Cfg::kRem == 0 || wave < Cfg::kRem;
  int kt_issue = 0;                                          // k-step, within its tile, of the next stage to issue
  auto issue_stage = [&](int g) {
    lds_u8_t* stage = smem + (g % NS) * Cfg::kStageBytes;
    const bool last = kt_issue == nk - 1;
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
      src[t] += last ? jump[t] : inc[t];
    }
    kt_issue = last ? 0 : kt_issue + 1;
  };
  // Stage g has landed once at most the loads of the NS-2 younger stages are pending.  Memory operations of
  // a wave retire in issue order, so the epilogue's own loads and stores, which are younger than the stages
  // in flight at that time, only make this fixed threshold more conservative.
  auto wait_landed = [&]() {
    if (extra) wait_vmcnt<(NS - 2) * Cfg::kMaxPer>(); else wait_vmcnt<(NS - 2) * (Cfg::kMaxPer - 1)>();
  };

  int a_off[FM], b_off[FN][2];
#pragma unroll
  for (int i = 0; i < FM; ++i) a_off[i] = (wm * Cfg::WM + i * 32 + l32) * Cfg::kARow;
  const int a_swz = Cfg::swz_a(l32);
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int hl = 0; hl < 2; ++hl) {
      const int kr = 8 * half + l16 / 4 + 4 * hl;
      const int n = wn * Cfg::WN + j * 32 + ((lane / 16) % 2) * 16 + (l16 % 4) * 4;
      b_off[j][hl] = Cfg::kABytes + kr * Cfg::kBRow + (((n / 8) ^ (Cfg::kBSwz * (l16 / 4))) * 16) + ((n / 4) % 2) * 8;
    }
  auto b_step = [](int kk) {
    return kk * 16 * Cfg::kBRow;
  };
  int bp_off[FN];                                            // PB: this lane's 16 bytes of column block j, slice 0
#pragma unroll
  for (int j = 0; j < FN; ++j) bp_off[j] = Cfg::kABytes + (wn * FN + j) * (BK / 16) * 1024 + lane * 16;

  const int total = nsub * nk;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < total) issue_stage(s);
  touch_a_rows<Cfg>(A, lda, K, a_touch_part, a_touch_parts);

  int g = 0;
  for (int sub = 0; sub < nsub; ++sub) {
    f32x16_t acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int kt = 0; kt < nk; ++kt, ++g) {
      if (g + NS - 2 < total) wait_landed(); else wait_vmcnt<0>();
      __builtin_amdgcn_s_barrier();
      const lds_u8_t* stage = smem + (g % NS) * Cfg::kStageBytes;
      bf16x8_t af[BK / 16][FM], bfr[BK / 16][FN];
#pragma unroll
      for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
        for (int i = 0; i < FM; ++i)
          af[kk][i] = *(const lds_bf16x8_t*)(stage + a_off[i] + (((2 * kk + half) ^ a_swz) * 16));
#pragma unroll
        for (int j = 0; j < FN; ++j) {
          if constexpr (PB) {
            bfr[kk][j] = *(const lds_bf16x8_t*)(stage + bp_off[j] + kk * 1024);
          } else {
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(stage + b_off[j][0] + b_step(kk)));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(stage + b_off[j][1] + b_step(kk)));
            const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            bfr[kk][j] = __builtin_bit_cast(bf16x8_t, both);
          }
        }
      }
      // The multiplications start as soon as the fragments of the first 16-k slice are there; the next stage's
      // loads are issued behind the last slice (they refill the stage read in step g-1).
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
      if (g + NS - 1 < total) issue_stage(g + NS - 1);
      __builtin_amdgcn_sched_barrier(0);
    }
    const long c0 = (long)sub * Cfg::kBN;
    const float* cb = col_bias ? col_bias + c0 : nullptr;
    const bf16_t* Rt = R ? R + c0 : nullptr;
    if (act == NF_ACT_GELU) stream_epilogue_act<Cfg, NF_ACT_GELU>(acc, C + c0, Rt, ldc, cb);
    else if (act == NF_ACT_RELU) stream_epilogue_act<Cfg, NF_ACT_RELU>(acc, C + c0, Rt, ldc, cb);
    else stream_epilogue_act<Cfg, NF_ACT_NONE>(acc, C + c0, Rt, ldc, cb);
  }
}

}  // namespace nf
