// bf16 MFMA contraction core shared by the merged matmul and the merged convolution.
//
//   C[z][i][j] = sum_k A[z][i][k] * B[z][k][j]     fp32 accumulation, one fused epilogue
//
// z runs over the independent input-weight pairs (models, or models x groups x images): the
// model index is a grid coordinate, never a loop inside a tile, so no tile ever mixes two models.
//
// A is row-major with k contiguous (activation rows of the matmul; weight rows of a convolution).
// B is "k-major": element (k, j) has j contiguous in memory (the matmul's W[K][Nout]; a
// convolution's input planes, where j runs over output positions).  Both are copied to LDS in the
// layout they have in memory -- A tile [BM][64], B tile [64][BN] -- so global loads and LDS stores
// are plain 16-byte copies.  The MFMA wants 8 consecutive k per lane for both operands: A
// fragments are 16-byte LDS reads; B fragments use gfx950's transposing LDS read
// (ds_read_b64_tr_b16), which hands each lane of a 16-lane group 4 consecutive k of one column.
//
// Workgroup = 4 or 8 wavefronts.  Wave (wm, wn) owns a (BM/WGM) x (BN/WGN) block of the
// tile as FM x FN MFMA 32x32x16 accumulators, computed TRANSPOSED (the instruction's A operand is
// the B fragment) so that a lane ends up with 4 consecutive output columns of one row: the
// epilogue can then move 16 bytes at a time.  K advances in steps of 64 with the next step's
// global loads in flight (registers) while the current one is multiplied out of LDS; LDS is
// double buffered so one barrier per step suffices.
//
// Epilogue: per-row / per-column constants and the activation are applied to the accumulators,
// which pass through LDS (fp32) to turn the MFMA layout into full rows; each thread then adds
// the residual (read 16 bytes at a time), rounds once to bf16 and stores 16 bytes.
#pragma once
#include "nf_common.h"

namespace nf {

// Pointers into LDS carry their address space explicitly: a generic pointer makes the compiler
// emit flat loads, which count against the global-memory counter too and serialise the prefetch.
typedef __attribute__((address_space(3))) bf16_t lds_bf16_t;
typedef __attribute__((address_space(3))) float lds_f32_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4v_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4_t lds_u32x4_t;
typedef __attribute__((address_space(3))) u32x2_t lds_u32x2_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((address_space(3))) bf16x8_t lds_bf16x8_t;
typedef __attribute__((address_space(3))) f32x4v_t lds_f32x4_t;

__device__ __forceinline__ void lds_store16(lds_bf16_t* p, uint4 v) { *(lds_u32x4_t*)p = u32x4_t{v.x, v.y, v.z, v.w}; }
__device__ __forceinline__ void lds_store8(lds_bf16_t* p, uint32_t a, uint32_t b) { *(lds_u32x2_t*)p = u32x2_t{a, b}; }

constexpr int kBK = 64;             // k extent of one LDS stage
// LDS has 64 banks (256 bytes per clock): a 16-byte read is served 16 lanes at a time, a transposing
// 8-byte read 32 lanes at a time, and the lanes served together must fall into distinct banks.
constexpr int kPitchA = kBK + 8;    // A tile row pitch (elements): 144 B = 9 x 16 B, so 16 consecutive rows
                                    // start in 16 different 16-byte bank groups
constexpr int kPadB = 32;           // B tile row pitch = BN + 32 elements: pitch mod 256 B = 64 B (BN a multiple
                                    // of 128) or 192 B (BN = 64), so the 4 rows x 64 B touched by 32 lanes of a
                                    // transposing read tile the 256 bytes exactly

struct Epilogue {
  const float* row_bias;    // [z][i] or null      (convolution bias per output channel)
  const float* row_scale;   // [z][i] or null      (folded batch norm), with row_shift
  const float* row_shift;
  const float* col_bias;    // [z][j] or null      (matmul bias per output feature)
  long row_vec_stride0, row_vec_stride1;   // z = z1 * nz0 + z0 -> offset z0*stride0 + z1*stride1
  long col_vec_stride0, col_vec_stride1;
  int act;
  int act_before_residual;  // matmul: act(.) + residual;  convolution: act(. + residual)
  int vec_store;            // 2: C (and residual) rows are 16-byte aligned and cols % 8 == 0; 1: 8-byte aligned
                            // and cols % 4 == 0 (e.g. 14 x 14 planes); 3: ldc == cols <= 64, so every tile spans
                            // whole rows, and 32 rows start 16-byte aligned (e.g. 7 x 7 planes); 0: element by element
};

// ------------------------------------------------------------------------------------------
// A tile loader: [BM][64] from a row-major matrix, 16-byte chunks; chunk c -> row c/8, k-chunk c%8,
// so 8 neighbouring lanes read and write 128 contiguous bytes.
// ALIGN = guaranteed byte alignment of every row start (K is then a multiple of ALIGN/2).
// FULL = the tile lies inside the matrix and K % 64 == 0: no predicates at all (needs ALIGN 16).
// ------------------------------------------------------------------------------------------
// WNT: the operand is read once per forward pass (matmul weights) and is loaded non-temporal.
template <bool WNT> __device__ __forceinline__ uint4 ld16(const void* p) {
  if constexpr (WNT) return ldnt16(p); else return *reinterpret_cast<const uint4*>(p);
}

template <int ALIGN>
__device__ __forceinline__ uint4 load_k8(const bf16_t* p, int k, int klim) {
  uint4 r = make_uint4(0, 0, 0, 0);
  if constexpr (ALIGN == 16) {
    if (k < klim) r = *reinterpret_cast<const uint4*>(p);
  } else if constexpr (ALIGN == 8) {
    uint2 a = make_uint2(0, 0), b = make_uint2(0, 0);
    if (k < klim) a = *reinterpret_cast<const uint2*>(p);
    if (k + 4 < klim) b = *reinterpret_cast<const uint2*>(p + 4);
    r = make_uint4(a.x, a.y, b.x, b.y);
  } else {
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = (k + e < klim) ? (uint32_t)p[e] : 0u;
    r = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
  }
  return r;
}

template <int BM, int ALIGN, bool FULL, int NT>
struct ATileLoader {
  static constexpr int kChunks = BM * (kBK / 8);
  static constexpr int kPer = kChunks / NT;
  static_assert(kChunks % NT == 0, "tile too small for the workgroup");
  const bf16_t* base;   // A + problem offset + row0*lda
  long lda;
  int rows_left;        // rows of the problem from row0 on
  int K;
  struct Regs { uint4 v[kPer]; };     // one k-step of this thread's share, in flight or landed

  __device__ __forceinline__ void fetch(Regs& regs, int k0, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int c = tid + t * NT;
      const int r = c / 8, kc = (c % 8) * 8;
      if constexpr (FULL) {
        regs.v[t] = *reinterpret_cast<const uint4*>(base + (long)r * lda + k0 + kc);
      } else {
        regs.v[t] = r < rows_left ? load_k8<ALIGN>(base + (long)r * lda + k0 + kc, k0 + kc, K) : make_uint4(0, 0, 0, 0);
      }
    }
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int c = tid + t * NT;
      lds_store16(lds + (c / 8) * kPitchA + (c % 8) * 8, regs.v[t]);
    }
  }
};

// ------------------------------------------------------------------------------------------
// B tile loader, dense k-major matrix B[k][j] (row pitch ldb): [64][BN] copied as is.
// VEC = 8: rows aligned to 16 bytes and cols % 8 == 0; VEC = 1: any rows.
// ------------------------------------------------------------------------------------------
template <int BN, int VEC, bool FULL, int NT, bool WNT = false>
struct BDenseLoader {
  static constexpr int kPitch = BN + kPadB;
  // VEC = 1 (rows that start at any 2-byte address, e.g. 7x7 = 49 positions per channel) still moves 8
  // elements per access: the global side is an unaligned 16-byte load, the LDS side is aligned.  The
  // elements such a chunk reads past the last valid column belong to the next row; they only feed output
  // columns that are never stored.  Only the chunk that would cross the END of the operand (`end`) is read
  // element by element.
  static_assert(VEC == 8 || VEC == 1, "16-byte aligned rows or any rows");
  static constexpr int kW = 8;                           // elements per task
  static constexpr int kPerRow = BN / kW;
  static constexpr int kTasks = kBK * kPerRow;
  static constexpr int kPer = kTasks / NT;
  static_assert(kTasks % NT == 0, "tile too small for the workgroup");
  static constexpr int kDw = 4;
  const bf16_t* base;   // B + problem offset + col0
  const bf16_t* end;    // one past the last element of the whole B operand (VEC = 1 only)
  long ldb;
  int cols_left, K;
  struct Regs { uint32_t v[kPer][kDw]; };
  struct __attribute__((packed, aligned(2))) unaligned16 { uint4 v; };

  __device__ __forceinline__ void fetch(Regs& regs, int k0, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      const int k = k0 + task / kPerRow, j = (task % kPerRow) * kW;
      const bf16_t* p = base + (long)k * ldb + j;
      const bool live = FULL || (k < K && j < cols_left);
      if constexpr (VEC == 8) {
        const uint4 v = live ? ld16<WNT>(p) : make_uint4(0, 0, 0, 0);
        regs.v[t][0] = v.x; regs.v[t][1] = v.y; regs.v[t][2] = v.z; regs.v[t][3] = v.w;
      } else {
        uint4 v = make_uint4(0, 0, 0, 0);
        if (live) {
          if (p + 8 <= end) {
            v = reinterpret_cast<const unaligned16*>(p)->v;
          } else {
            uint32_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = p + e < end ? (uint32_t)p[e] : 0u;
            v = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
          }
        }
        regs.v[t][0] = v.x; regs.v[t][1] = v.y; regs.v[t][2] = v.z; regs.v[t][3] = v.w;
      }
    }
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      lds_bf16_t* dst = lds + (task / kPerRow) * kPitch + (task % kPerRow) * kW;
      lds_store16(dst, make_uint4(regs.v[t][0], regs.v[t][1], regs.v[t][2], regs.v[t][3]));
    }
  }
};

// Geometry of the implicit B matrix of a convolution: row k = (ci, ky, kx) of one group, column
// j = output position (oy, ox); element = x[channel0 + ci][oy*stride + ky*dil - pad][ox*stride + kx*dil - pad]
// or zero outside the image (Appendix A Eq. 1, cross-correlation on the zero-padded input).
struct Im2colGeom {
  int H, W, KH, KW, Wo, stride, pad, dil;
};

// B tile loader gathering from the input planes: task = one k row x 8 consecutive output positions
// (consecutive ox of one output row read consecutive-or-strided input pixels of one input row).
template <int BN, int NT>
struct BIm2colLoader {
  static constexpr int kPitch = BN + kPadB;
  static constexpr int kPerRow = BN / 8;
  static constexpr int kTasks = kBK * kPerRow;
  static constexpr int kPer = kTasks / NT;
  static_assert(kTasks % NT == 0, "tile too small for the workgroup");
  const bf16_t* xg;     // first input plane of this group and image
  Im2colGeom g;
  int cols_left, K, col0;
  struct Regs { uint4 v[kPer]; };

  __device__ __forceinline__ void fetch(Regs& regs, int k0, int tid) const {
    const int khw = g.KH * g.KW;
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      const int k = k0 + task / kPerRow, j = (task % kPerRow) * 8;
      uint32_t h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = 0u;
      if (k < K && j < cols_left) {
        const int ci = k / khw, rem = k - ci * khw;
        const int ky = rem / g.KW, kx = rem - ky * g.KW;
        const bf16_t* plane = xg + (long)ci * g.H * g.W;
        const int p = col0 + j;
        int oy = p / g.Wo, ox = p - oy * g.Wo;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int iy = oy * g.stride - g.pad + ky * g.dil, ix = ox * g.stride - g.pad + kx * g.dil;
          if (j + e < cols_left && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W) h[e] = (uint32_t)plane[(long)iy * g.W + ix];
          if (++ox == g.Wo) { ox = 0; ++oy; }
        }
      }
      regs.v[t] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      lds_store16(lds + (task / kPerRow) * kPitch + (task % kPerRow) * 8, regs.v[t]);
    }
  }
};

// B tile loader of a strided pointwise convolution (1x1 kernel, no padding: the projection shortcuts):
// element (k, p) = x[k][(p / Wo) * stride][(p % Wo) * stride], always inside the image.  Task = one k row x
// 8 consecutive output positions; one division per task, no bounds checks on the image.
template <int BN, int NT>
struct BStridedPointwiseLoader {
  static constexpr int kPitch = BN + kPadB;
  static constexpr int kPerRow = BN / 8;
  static constexpr int kTasks = kBK * kPerRow;
  static constexpr int kPer = kTasks / NT;
  static_assert(kTasks % NT == 0, "tile too small for the workgroup");
  const bf16_t* xg;     // first input plane of this group and image
  Im2colGeom g;
  int cols_left, K, col0;
  struct Regs { uint4 v[kPer]; };

  __device__ __forceinline__ void fetch(Regs& regs, int k0, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      const int k = k0 + task / kPerRow, j = (task % kPerRow) * 8;
      uint32_t h[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) h[e] = 0u;
      if (k < K && j < cols_left) {
        const bf16_t* plane = xg + (long)k * g.H * g.W;
        const int p = col0 + j;
        int oy = p / g.Wo, ox = p - oy * g.Wo;
        int off = (oy * g.W + ox) * g.stride;
        const int row_step = (g.W - g.Wo) * g.stride;      // from the end of one output row to the start of the next
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (j + e < cols_left) h[e] = (uint32_t)plane[off];
          off += g.stride;
          if (++ox == g.Wo) { ox = 0; off += row_step; }
        }
      }
      regs.v[t] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      lds_store16(lds + (task / kPerRow) * kPitch + (task % kPerRow) * 8, regs.v[t]);
    }
  }
};

// The same for stride 2 over an image of even width W = 2 Wo, read as (even, odd) pixel pairs: pair
// oy * W + ox of a plane holds input pixel (2 oy, 2 ox) in its low half, so VW consecutive output
// positions of one row are VW consecutive pairs, fetched with one 4*VW-byte load (VW = 4 or 2, dividing
// Wo, hence no group straddles a row) and narrowed by byte permutes.  The caller guarantees the alignment:
// plane pitch and base multiples of 2*VW elements.
template <int BN, int VW, int NT>
struct BStride2PairLoader {
  static_assert(VW == 4 || VW == 2, "pairs per load");
  static constexpr int kPitch = BN + kPadB;
  static constexpr int kPerRow = BN / 8;
  static constexpr int kTasks = kBK * kPerRow;
  static constexpr int kPer = kTasks / NT;
  static_assert(kTasks % NT == 0, "tile too small for the workgroup");
  const bf16_t* xg;     // first input plane of this group and image
  Im2colGeom g;
  int cols_left, K, col0;
  struct Regs { uint4 v[kPer]; };

  __device__ __forceinline__ void fetch(Regs& regs, int k0, int tid) const {
    constexpr uint32_t kLowHalves = 0x05040100u;     // perm(hi, lo): low 16 bits of lo, then low 16 bits of hi
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      const int k = k0 + task / kPerRow, j = (task % kPerRow) * 8;
      uint32_t o[4] = {0u, 0u, 0u, 0u};
      if (k < K && j < cols_left) {
        const uint32_t* plane = reinterpret_cast<const uint32_t*>(xg + (long)k * g.H * g.W);
        const int p = col0 + j;
        int oy = p / g.Wo, ox = p - oy * g.Wo;
#pragma unroll
        for (int q = 0; q < 8 / VW; ++q) {
          if (j + q * VW < cols_left) {            // the output count is a multiple of VW: whole groups only
            const uint32_t* src = plane + oy * g.W + ox;
            if constexpr (VW == 4) {
              const uint4 v = *reinterpret_cast<const uint4*>(src);
              o[2 * q] = __builtin_amdgcn_perm(v.y, v.x, kLowHalves);
              o[2 * q + 1] = __builtin_amdgcn_perm(v.w, v.z, kLowHalves);
            } else {
              const uint2 v = *reinterpret_cast<const uint2*>(src);
              o[q] = __builtin_amdgcn_perm(v.y, v.x, kLowHalves);
            }
          }
          ox += VW;
          if (ox == g.Wo) { ox = 0; ++oy; }
        }
      }
      regs.v[t] = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      lds_store16(lds + (task / kPerRow) * kPitch + (task % kPerRow) * 8, regs.v[t]);
    }
  }
};

// ------------------------------------------------------------------------------------------
// Branch-free loaders of the deep pipeline (gemm_tile_deep): every fetch issues the same loads on every
// lane, so the number of loads in flight is known at compile time and a wait for one k-step leaves the
// younger steps pending.  Rows and column chunks outside the problem are redirected to the last valid
// one instead of being skipped; what they produce lands in rows / columns of C that are never stored.
// Requirements (checked by the caller): K a multiple of the k-step, A rows 16-byte aligned, B rows of
// at least 8 elements.
// ------------------------------------------------------------------------------------------
template <int BM, int NT>
struct ADeepLoader {
  static constexpr int kChunks = BM * (kBK / 8);
  static constexpr int kPer = kChunks / NT;
  static_assert(kChunks % NT == 0, "tile too small for the workgroup");
  const bf16_t* src[kPer];              // this thread's chunks at k = 0
  struct Regs { uint4 v[kPer]; };
  __device__ __forceinline__ void init(const bf16_t* base, long lda, int rows_left, int tid) {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int c = tid + t * NT;
      const int r = min(c / 8, rows_left - 1);
      src[t] = base + (long)r * lda + (c % 8) * 8;
    }
  }
  __device__ __forceinline__ void fetch(Regs& regs, int k0, int) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) regs.v[t] = *reinterpret_cast<const uint4*>(src[t] + k0);
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int c = tid + t * NT;
      lds_store16(lds + (c / 8) * kPitchA + (c % 8) * 8, regs.v[t]);
    }
  }
};

template <int BN, bool ALIGNED, int NT, bool WNT = false>
struct BDeepLoader {
  static constexpr int kPitch = BN + kPadB;
  static constexpr int kPerRow = BN / 8;
  static constexpr int kTasks = kBK * kPerRow;
  static constexpr int kPer = kTasks / NT;
  static_assert(kTasks % NT == 0, "tile too small for the workgroup");
  const bf16_t* src[kPer];              // this thread's chunks at k = 0
  long step;                            // elements per k-step: kBK * ldb
  // !ALIGNED: rows start at any 2-byte address and the last chunk of a row may run into the next row.
  // Only in the last row of the whole operand would it run past the end: that one load is pulled back to
  // `limit` (last address a full chunk may start at) and the elements it should have brought are put into
  // LDS one by one by finish(), after the last k-step is committed.
  const bf16_t* limit;
  const bf16_t* tail_src;               // valid elements of that chunk, or null when the tile does not reach the end
  int tail_n, tail_col;
  struct Regs { uint4 v[kPer]; };
  struct __attribute__((packed, aligned(2))) unaligned16 { uint4 v; };
  // first column of the last chunk that holds a valid column
  static __device__ __forceinline__ int last_chunk(int cols_left) { return (min(cols_left, BN) - 1) & ~7; }
  // ldb >= 8, K a multiple of kBK; `end` = one past the last element of the whole operand
  __device__ __forceinline__ void init(const bf16_t* base, long ldb, int cols_left, int K, const bf16_t* end, int tid) {
    step = (long)kBK * ldb;
    const int lastc = last_chunk(cols_left);
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      const int j = min((task % kPerRow) * 8, lastc);
      src[t] = base + (long)(task / kPerRow) * ldb + j;
    }
    if constexpr (!ALIGNED) {
      limit = end - 8;
      const bf16_t* last = base + (long)(K - 1) * ldb + lastc;    // with ldb >= 8 no other chunk can cross the end
      tail_src = last > limit ? last : nullptr;
      tail_n = (int)(end - last);
      tail_col = lastc;
    }
  }
  __device__ __forceinline__ void fetch(Regs& regs, int k0, int) const {
    const long off = (long)(k0 / kBK) * step;
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      if constexpr (ALIGNED) {
        regs.v[t] = ld16<WNT>(src[t] + off);
      } else {
        const bf16_t* p = src[t] + off;
        regs.v[t] = reinterpret_cast<const unaligned16*>(p < limit ? p : limit)->v;
      }
    }
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int tid) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      lds_store16(lds + (task / kPerRow) * kPitch + (task % kPerRow) * 8, regs.v[t]);
    }
  }
  // after the commit of the last k-step into `lds`, before the barrier that publishes it
  __device__ __forceinline__ void finish(lds_bf16_t* lds, int tid) const {
    if constexpr (!ALIGNED) {
      if (tail_src == nullptr) return;
      // the thread that committed the pulled-back chunk overwrites it (LDS writes of one thread stay in order)
#pragma unroll
      for (int t = 0; t < kPer; ++t)
        if (tid + t * NT == (kBK - 1) * kPerRow + tail_col / 8)
          for (int e = 0; e < tail_n; ++e) lds[(kBK - 1) * kPitch + tail_col + e] = tail_src[e];
    }
  }
};

// Branch-free B loader of a stride-2 pointwise convolution over an image of even width W = 2 Wo, for the
// deep pipeline: the image is read as (even, odd) pixel pairs (see BStride2PairLoader), VW pairs per load
// (VW = 4, 2 or 1; VW divides Wo, and plane pitch and base are multiples of 2*VW elements).  The pair
// offsets of this thread's 8 / VW loads per task are fixed at init; output positions past the end of the
// image are redirected to the last group of VW.
template <int BN, int VW, int NT>
struct BPairDeepLoader {
  static_assert(VW == 4 || VW == 2 || VW == 1, "pairs per load");
  static constexpr int kPitch = BN + kPadB;
  static constexpr int kPerRow = BN / 8;
  static constexpr int kTasks = kBK * kPerRow;
  static constexpr int kPer = kTasks / NT;
  static constexpr int kLoads = 8 / VW;             // per task
  static_assert(kTasks % NT == 0, "tile too small for the workgroup");
  typedef typename std::conditional<VW == 4, uint4, typename std::conditional<VW == 2, uint2, uint32_t>::type>::type raw_t;
  const uint32_t* planes;                // first input plane of this group and image, as pairs
  int off[kPer][kLoads];                 // pair offsets at k = 0
  int step;                              // pairs per k-step: kBK * H * W / 2
  struct Regs { raw_t v[kPer][kLoads]; };
  __device__ __forceinline__ void init(const bf16_t* xg, const Im2colGeom& g, int col0, int cols_left, int tid) {
    planes = reinterpret_cast<const uint32_t*>(xg);
    const int plane = g.H * g.W / 2;
    step = kBK * plane;
    const int p_last = col0 + cols_left - VW;        // first position of the last whole group
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      const int krow = task / kPerRow, j = (task % kPerRow) * 8;
#pragma unroll
      for (int q = 0; q < kLoads; ++q) {
        const int p = min(col0 + j + q * VW, p_last);
        const int oy = p / g.Wo, ox = p - oy * g.Wo;
        off[t][q] = krow * plane + oy * g.W + ox;
      }
    }
  }
  __device__ __forceinline__ void fetch(Regs& regs, int k0, int) const {
    const uint32_t* base = planes + (long)(k0 / kBK) * step;
#pragma unroll
    for (int t = 0; t < kPer; ++t)
#pragma unroll
      for (int q = 0; q < kLoads; ++q) regs.v[t][q] = *reinterpret_cast<const raw_t*>(base + off[t][q]);
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int tid) const {
    constexpr uint32_t kLowHalves = 0x05040100u;     // perm(hi, lo): low 16 bits of lo, then low 16 bits of hi
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      uint32_t o[4];
      if constexpr (VW == 4) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          o[2 * q] = __builtin_amdgcn_perm(regs.v[t][q].y, regs.v[t][q].x, kLowHalves);
          o[2 * q + 1] = __builtin_amdgcn_perm(regs.v[t][q].w, regs.v[t][q].z, kLowHalves);
        }
      } else if constexpr (VW == 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) o[q] = __builtin_amdgcn_perm(regs.v[t][q].y, regs.v[t][q].x, kLowHalves);
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) o[q] = __builtin_amdgcn_perm(regs.v[t][2 * q + 1], regs.v[t][2 * q], kLowHalves);
      }
      lds_store16(lds + (task / kPerRow) * kPitch + (task % kPerRow) * 8, make_uint4(o[0], o[1], o[2], o[3]));
    }
  }
  __device__ __forceinline__ void finish(lds_bf16_t*, int) const {}
};

// The same for 7 output columns (a 14-wide input: the last projection shortcut of a 224 x 224 ResNet), where
// groups of 8 consecutive output positions would straddle rows and every position would cost its own load:
// task = one (k row, output row): the 7 pixel pairs of input row 2 oy are contiguous (28 bytes at an 8-byte
// aligned address: three 8-byte loads and one of 4), and their low halves go to LDS columns 7 oy .. 7 oy + 6
// with 2-byte writes.  The whole image is one column tile (at most 8 output rows); LDS columns past the
// image are never written and only feed output columns that are never stored.
template <int BN, int NT>
struct BRow7DeepLoader {
  static constexpr int kPitch = BN + kPadB;
  static constexpr int kWo = 7, kMaxHo = 8;
  static constexpr int kPer = (kBK * kMaxHo + NT - 1) / NT;
  static_assert(BN >= kWo * kMaxHo, "the image fits one column tile");
  const uint32_t* planes;                // first input plane of this group and image, as pairs
  int off[kPer];                         // pair offset of the task's input row at k = 0
  int dst[kPer];                         // LDS element offset of its 7 columns, or -1: nothing to commit
  int step;                              // pairs per k-step
  struct Regs { uint32_t v[kPer][kWo]; };
  __device__ __forceinline__ void init(const bf16_t* xg, const Im2colGeom& g, int Ho, int tid) {
    planes = reinterpret_cast<const uint32_t*>(xg);
    const int plane = g.H * g.W / 2;
    step = kBK * plane;
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int task = tid + t * NT;
      const int krow = task / Ho, oy = task - krow * Ho;
      const bool live = krow < kBK;
      off[t] = live ? krow * plane + oy * g.W : 0;
      dst[t] = live ? krow * kPitch + oy * kWo : -1;
    }
  }
  __device__ __forceinline__ void fetch(Regs& regs, int k0, int) const {
    const uint32_t* base = planes + (long)(k0 / kBK) * step;
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const uint32_t* p = base + off[t];
      const uint2 a = *reinterpret_cast<const uint2*>(p), b = *reinterpret_cast<const uint2*>(p + 2),
                  c = *reinterpret_cast<const uint2*>(p + 4);
      regs.v[t][0] = a.x; regs.v[t][1] = a.y; regs.v[t][2] = b.x; regs.v[t][3] = b.y;
      regs.v[t][4] = c.x; regs.v[t][5] = c.y; regs.v[t][6] = p[6];
    }
  }
  __device__ __forceinline__ void commit(const Regs& regs, lds_bf16_t* lds, int) const {
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      if (dst[t] < 0) continue;
#pragma unroll
      for (int i = 0; i < kWo; ++i) lds[dst[t] + i] = (bf16_t)regs.v[t][i];
    }
  }
  __device__ __forceinline__ void finish(lds_bf16_t*, int) const {}
};

// ------------------------------------------------------------------------------------------
// The tile main loop and epilogue
// ------------------------------------------------------------------------------------------
template <int BM, int BN, int WGM, int WGN, int DEPTH = 1>
struct TileCfg {
  static constexpr int kDepth = DEPTH;     // k-steps of global loads in flight per thread (see gemm_tile_deep)
  static_assert(WGM * WGN == 4 || WGM * WGN == 8, "4 or 8 wavefronts per workgroup");
  static constexpr int kBM = BM, kBN = BN, kWGM = WGM, kWGN = WGN;
  static constexpr int kThreads = WGM * WGN * kWave;
  static constexpr bool kRowConsts = true;               // convolution epilogues carry per-row scale/shift
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int FM = WM / 32, FN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile is made of 32x32 MFMA blocks");
  static constexpr int kPitchB = BN + kPadB;
  static constexpr int kLdsA = BM * kPitchA, kLdsB = kBK * kPitchB;       // elements per stage
  static constexpr int kLdsPipe = 2 * (kLdsA + kLdsB) * (int)sizeof(bf16_t);
  // epilogue staging: one 32-row block of every wave row at a time, fp32, padded rows
  static constexpr int kEpiPitch = BN + 4;
  static constexpr int kLdsEpi = WGM * 32 * kEpiPitch * (int)sizeof(float);
  static constexpr int kLdsBytes = kLdsPipe > kLdsEpi ? kLdsPipe : kLdsEpi;
};

#ifndef NF_REG_EPILOGUE
#define NF_REG_EPILOGUE 1
#endif

template <int ACT>
__device__ __forceinline__ float act_const(float v) {
  if constexpr (ACT == NF_ACT_RELU) return v > 0.f ? v : (v != v ? v : 0.f);
  else if constexpr (ACT == NF_ACT_GELU) return gelu_erf(v);
  else return v;
}

// ACT1: activation applied to the accumulator side (before the residual), ACT2: after the residual.
// HALVES: the body for ep.vec_store == 1 (8-byte accesses, each half of an 8-column chunk whole or absent) and
// == 3 (flat mode, see below); otherwise 16-byte accesses or, for ep.vec_store == 0, single elements.
template <class Cfg, int ACT1, int ACT2, bool HALVES>
__device__ __forceinline__ void gemm_epilogue_act(f32x16_t (&acc)[Cfg::FM][Cfg::FN], lds_f32_t* const Es, bf16_t* C,
                                                  const bf16_t* R, long ldc, int rows_left, int cols_left,
                                                  const Epilogue& ep, long row_vec_off, long col_vec_off) {
  constexpr int FM = Cfg::FM, FN = Cfg::FN;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / Cfg::kWGN, wn = wave % Cfg::kWGN;
  const int half = lane / 32, l32 = lane % 32;
  constexpr int kEP = Cfg::kEpiPitch;
  constexpr int kChunksPerRow = Cfg::kBN / 8;
  constexpr int kPassChunks = Cfg::kWGM * 32 * kChunksPerRow;
  constexpr int kPer = (kPassChunks + Cfg::kThreads - 1) / Cfg::kThreads;

  // per-column constants of this lane (4 consecutive columns per 8-column group), fetched once, all
  // loads in flight together
  float cb[FN][4][4];
  if (FN >= 3 && ep.col_bias != nullptr && cols_left >= Cfg::kBN && ((uintptr_t)(ep.col_bias + col_vec_off) & 15) == 0) {
    // wide wave tiles (where the scalar form costs 48+ predicated loads per lane; measured slower on narrow
    // ones), whole tile, 16-byte aligned vector: one 16-byte load per 4 columns, no per-column predicate
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 v = *reinterpret_cast<const float4*>(ep.col_bias + col_vec_off + wn * Cfg::WN + j * 32 + q * 8 + half * 4);
        cb[j][q][0] = v.x; cb[j][q][1] = v.y; cb[j][q][2] = v.z; cb[j][q][3] = v.w;
      }
  } else {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int col = wn * Cfg::WN + j * 32 + q * 8 + half * 4 + e;
          cb[j][q][e] = (ep.col_bias != nullptr && col < cols_left) ? ep.col_bias[col_vec_off + col] : 0.f;
        }
  }

  // per-row constants of this lane for every pass, fetched together: one memory round trip instead of one
  // per pass (short-K layers are a chain of such round trips).  Configurations whose callers never pass row
  // constants (Cfg::kRowConsts == false: the whole-tile matmul kernels) keep the per-pass form, which costs
  // them nothing and leaves their register allocation alone.
  float rbs[FM], rss[FM], rts[FM];
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    rbs[i] = 0.f; rss[i] = 1.f; rts[i] = 0.f;
    if constexpr (Cfg::kRowConsts) {
      const int row = wm * Cfg::WM + i * 32 + l32;           // this lane's row in the tile
      if (row < rows_left) {
        if (ep.row_bias) rbs[i] = ep.row_bias[row_vec_off + row];
        if (ep.row_scale) { rss[i] = ep.row_scale[row_vec_off + row]; rts[i] = ep.row_shift[row_vec_off + row]; }
      }
    }
  }

#pragma unroll
  for (int i = 0; i < FM; ++i) {
    {
      float rb = rbs[i], rs = rss[i], rt = rts[i];
      if constexpr (!Cfg::kRowConsts) {
        const int row = wm * Cfg::WM + i * 32 + l32;
        if (row < rows_left) {
          if (ep.row_bias) rb = ep.row_bias[row_vec_off + row];
          if (ep.row_scale) { rs = ep.row_scale[row_vec_off + row]; rt = ep.row_shift[row_vec_off + row]; }
        }
      }
      lds_f32_t* erow = Es + (wm * 32 + l32) * kEP + wn * Cfg::WN + half * 4;
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4v_t v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = act_const<ACT1>(fmaf(acc[i][j][q * 4 + e] + cb[j][q][e] + rb, rs, rt));
          *(lds_f32x4_t*)(erow + j * 32 + q * 8) = v;
        }
    }
    __syncthreads();
    if constexpr (HALVES) {
      if (ep.vec_store == 3) {
        // Flat mode: the tile spans whole rows (ldc == cols_left), so the 32 rows of each wave row are one
        // contiguous, 16-byte aligned run of 32 * ldc elements in C and R; it is written 8 elements per
        // thread regardless of where the rows begin (rows of 49 elements start at odd 2-byte addresses).
        const int ld = (int)ldc;
        const int cps = (32 * ld + 7) / 8;                         // chunks per run
        for (int c = tid; c < Cfg::kWGM * cps; c += Cfg::kThreads) {
          const int sp = c / cps, f0 = (c - sp * cps) * 8;
          const int first = sp * Cfg::WM + i * 32;                   // first tile row of the run
          const int n_el = max(0, min(32, rows_left - first)) * ld;
          if (f0 >= n_el) continue;
          int r = f0 / ld, col = f0 - r * ld;
          float v[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            v[e] = f0 + e < n_el ? Es[(sp * 32 + r) * kEP + col] : 0.f;
            if (++col == ld) { col = 0; ++r; }
          }
          const long o0 = (long)first * ldc + f0;
          if (f0 + 8 <= n_el) {
            uint4 w4 = make_uint4(0, 0, 0, 0);
            if (R != nullptr) w4 = *reinterpret_cast<const uint4*>(R + o0);
            const uint32_t w[4] = {w4.x, w4.y, w4.z, w4.w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float a0 = act_const<ACT2>(v[2 * e] + __uint_as_float(w[e] << 16));
              const float a1 = act_const<ACT2>(v[2 * e + 1] + __uint_as_float(w[e] & 0xffff0000u));
              o[e] = pack_bf16x2(a0, a1);
            }
            *reinterpret_cast<uint4*>(C + o0) = make_uint4(o[0], o[1], o[2], o[3]);
          } else {
            for (int e = 0; f0 + e < n_el; ++e) {
              float x = v[e];
              if (R) x += bf16_to_f32(R[o0 + e]);
              C[o0 + e] = f32_to_bf16(act_const<ACT2>(x));
            }
          }
        }
        __syncthreads();
        continue;
      }
    }
    // this thread's chunks of the pass: residual loads first (all in flight), then LDS -> bf16 -> HBM
    uint4 rr[kPer];
    long off[kPer];
    bool live[kPer];
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      const int c = tid + t * Cfg::kThreads;
      const int prow = c / kChunksPerRow, col = (c % kChunksPerRow) * 8;
      const int row = (prow / 32) * Cfg::WM + i * 32 + (prow % 32);
      live[t] = (kPassChunks % Cfg::kThreads == 0 || c < kPassChunks) && row < rows_left && col < cols_left;
      off[t] = (long)row * ldc + col;
      rr[t] = make_uint4(0, 0, 0, 0);
      if constexpr (HALVES) {
        if (live[t] && R != nullptr) {
          const uint2 lo = *reinterpret_cast<const uint2*>(R + off[t]);
          uint2 hi = make_uint2(0, 0);
          if (col + 4 < cols_left) hi = *reinterpret_cast<const uint2*>(R + off[t] + 4);
          rr[t] = make_uint4(lo.x, lo.y, hi.x, hi.y);
        }
      } else {
        if (live[t] && R != nullptr && ep.vec_store) rr[t] = *reinterpret_cast<const uint4*>(R + off[t]);
      }
    }
#pragma unroll
    for (int t = 0; t < kPer; ++t) {
      if (!live[t]) continue;
      const int c = tid + t * Cfg::kThreads;
      const int prow = c / kChunksPerRow, col = (c % kChunksPerRow) * 8;
      const lds_f32_t* src = Es + prow * kEP + col;
      const f32x4v_t v0 = *(const lds_f32x4_t*)src, v1 = *(const lds_f32x4_t*)(src + 4);
      float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
      if (HALVES || ep.vec_store) {
        const uint32_t w[4] = {rr[t].x, rr[t].y, rr[t].z, rr[t].w};
        uint32_t o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float a0 = act_const<ACT2>(v[2 * e] + __uint_as_float(w[e] << 16));
          const float a1 = act_const<ACT2>(v[2 * e + 1] + __uint_as_float(w[e] & 0xffff0000u));
          o[e] = pack_bf16x2(a0, a1);
        }
        if constexpr (HALVES) {
          *reinterpret_cast<uint2*>(C + off[t]) = make_uint2(o[0], o[1]);
          if (col + 4 < cols_left) *reinterpret_cast<uint2*>(C + off[t] + 4) = make_uint2(o[2], o[3]);
        } else {
          *reinterpret_cast<uint4*>(C + off[t]) = make_uint4(o[0], o[1], o[2], o[3]);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (col + e >= cols_left) break;
          float x = v[e];
          if (R) x += bf16_to_f32(R[off[t] + e]);
          C[off[t] + e] = f32_to_bf16(act_const<ACT2>(x));
        }
      }
    }
    __syncthreads();
  }
}

// The same epilogue straight from the accumulators, for outputs whose rows are 16-byte aligned and whole
// 8-column pieces (ep.vec_store == 2) and that carry no per-column constants (every convolution): no staging
// through LDS and no workgroup barrier.  A lane holds, per 32 x 32 block, four groups of 4 consecutive columns
// of its row (columns 8 q + 4 half + 0..3); the two lanes of a row (lane, lane + 32) swap one group per pair of
// groups so that each ends up with 8 consecutive columns: residual and output then move 16 bytes per lane.
// Same arithmetic in the same order as the staged form, element by element: the two give the same bits.
// TAIL4 (ep.vec_store == 1: rows 8-byte aligned, widths multiples of 4, e.g. 14 x 14 planes): the 16-byte accesses
// then sit on 8-byte boundaries, and the last piece of a row may be its first 4 columns only (8 bytes).
template <class Cfg, int ACT1, int ACT2, bool TAIL4 = false>
__device__ __forceinline__ void gemm_epilogue_regs(f32x16_t (&acc)[Cfg::FM][Cfg::FN], bf16_t* C, const bf16_t* R,
                                                   long ldc, int rows_left, int cols_left, const Epilogue& ep,
                                                   long row_vec_off) {
  constexpr int FM = Cfg::FM, FN = Cfg::FN;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int wm = wave / Cfg::kWGN, wn = wave % Cfg::kWGN;
  const int half = lane / 32, l32 = lane % 32;
  float rbs[FM], rss[FM], rts[FM];
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    rbs[i] = 0.f; rss[i] = 1.f; rts[i] = 0.f;
    const int row = wm * Cfg::WM + i * 32 + l32;
    if (row < rows_left) {
      if (ep.row_bias) rbs[i] = ep.row_bias[row_vec_off + row];
      if (ep.row_scale) { rss[i] = ep.row_scale[row_vec_off + row]; rts[i] = ep.row_shift[row_vec_off + row]; }
    }
  }
  // this lane's residual pieces (columns colb + 16 qq + 8 half + 0..7 of its FM rows), all requested together
  uint4 rr[FM][FN][2];
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    const int row = wm * Cfg::WM + i * 32 + l32;
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int qq = 0; qq < 2; ++qq) {
        const int col = wn * Cfg::WN + j * 32 + 16 * qq + 8 * half;
        rr[i][j][qq] = make_uint4(0u, 0u, 0u, 0u);
        if (R != nullptr && row < rows_left && col < cols_left) {
          if (!TAIL4 || col + 8 <= cols_left) {
            rr[i][j][qq] = *reinterpret_cast<const uint4*>(R + (long)row * ldc + col);
          } else {
            const uint2 lo = *reinterpret_cast<const uint2*>(R + (long)row * ldc + col);
            rr[i][j][qq] = make_uint4(lo.x, lo.y, 0u, 0u);
          }
        }
      }
  }
#pragma unroll
  for (int i = 0; i < FM; ++i) {
    const int row = wm * Cfg::WM + i * 32 + l32;
    const bool row_ok = row < rows_left;
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int qq = 0; qq < 2; ++qq) {
        float own[4], send[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // group 2 qq + half stays (its other half comes from the partner), group 2 qq + 1 - half is sent
          const float v0 = act_const<ACT1>(fmaf(acc[i][j][(2 * qq) * 4 + e] + 0.f + rbs[i], rss[i], rts[i]));
          const float v1 = act_const<ACT1>(fmaf(acc[i][j][(2 * qq + 1) * 4 + e] + 0.f + rbs[i], rss[i], rts[i]));
          own[e] = half ? v1 : v0;
          send[e] = half ? v0 : v1;
        }
        float v[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float recv = __shfl_xor(send[e], 32, kWave);
          v[e] = half ? recv : own[e];
          v[4 + e] = half ? own[e] : recv;
        }
        const int col = wn * Cfg::WN + j * 32 + 16 * qq + 8 * half;
        if (row_ok && col < cols_left) {
          const uint32_t w[4] = {rr[i][j][qq].x, rr[i][j][qq].y, rr[i][j][qq].z, rr[i][j][qq].w};
          uint32_t o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float a0 = act_const<ACT2>(v[2 * e] + __uint_as_float(w[e] << 16));
            const float a1 = act_const<ACT2>(v[2 * e + 1] + __uint_as_float(w[e] & 0xffff0000u));
            o[e] = pack_bf16x2(a0, a1);
          }
          if (!TAIL4 || col + 8 <= cols_left) *reinterpret_cast<uint4*>(C + (long)row * ldc + col) = make_uint4(o[0], o[1], o[2], o[3]);
          else *reinterpret_cast<uint2*>(C + (long)row * ldc + col) = make_uint2(o[0], o[1]);
        }
      }
  }
}

// ------------------------------------------------------------------------------------------
// Epilogue shared by the contraction kernels.  acc[i][j] holds rows wm*WM + 32 i .. and columns
// wn*WN + 32 j .. of the tile, transposed: register r of lane l is row (l % 32), column
// 8 (r/4) + 4 (l/32) + r % 4 of the 32x32 block.  One 32-row block of every wave row per pass goes
// through LDS (Es, fp32) so that rows leave the workgroup 16 bytes per lane.  All threads of the
// workgroup must call it, after a barrier that ends every other use of the LDS behind Es.
// The activation is a wave-uniform switch around fully specialised bodies.
// ------------------------------------------------------------------------------------------
template <class Cfg>
__device__ __forceinline__ void gemm_epilogue(f32x16_t (&acc)[Cfg::FM][Cfg::FN], lds_f32_t* const Es, bf16_t* C,
                                              const bf16_t* R, long ldc, int rows_left, int cols_left,
                                              const Epilogue& ep, long row_vec_off, long col_vec_off) {
#define NF_EPI(A1, A2)                                                                                          \
  do {                                                                                                          \
    if (NF_REG_EPILOGUE && Cfg::kRowConsts && ep.vec_store == 2 && ep.col_bias == nullptr)                       \
      gemm_epilogue_regs<Cfg, A1, A2>(acc, C, R, ldc, rows_left, cols_left, ep, row_vec_off);                   \
    else if (NF_REG_EPILOGUE && Cfg::kRowConsts && ep.vec_store == 1 && ep.col_bias == nullptr)                  \
      gemm_epilogue_regs<Cfg, A1, A2, true>(acc, C, R, ldc, rows_left, cols_left, ep, row_vec_off);             \
    else if (ep.vec_store == 1 || ep.vec_store == 3)                                                                 \
      gemm_epilogue_act<Cfg, A1, A2, true>(acc, Es, C, R, ldc, rows_left, cols_left, ep, row_vec_off, col_vec_off); \
    else                                                                                                        \
      gemm_epilogue_act<Cfg, A1, A2, false>(acc, Es, C, R, ldc, rows_left, cols_left, ep, row_vec_off, col_vec_off); \
  } while (0)
  if (ep.act == NF_ACT_NONE) NF_EPI(NF_ACT_NONE, NF_ACT_NONE);
  else if (ep.act_before_residual) {
    if (ep.act == NF_ACT_GELU) NF_EPI(NF_ACT_GELU, NF_ACT_NONE); else NF_EPI(NF_ACT_RELU, NF_ACT_NONE);
  } else {
    if (ep.act == NF_ACT_GELU) NF_EPI(NF_ACT_NONE, NF_ACT_GELU); else NF_EPI(NF_ACT_NONE, NF_ACT_RELU);
  }
#undef NF_EPI
}

// DEEP: the loaders are branch free and K is a multiple of Cfg::kDepth k-steps; Cfg::kDepth steps of
// loads are kept in flight in a ring of register slots.
template <class Cfg, bool DEEP = false, class ALoader, class BLoader>
__device__ __forceinline__ void gemm_tile(ALoader& la, BLoader& lb, int K, lds_bf16_t* smem,
                                          bf16_t* C, const bf16_t* R, long ldc, int rows_left,
                                          int cols_left, const Epilogue& ep, long row_vec_off,
                                          long col_vec_off) {
  constexpr int FM = Cfg::FM, FN = Cfg::FN;
  const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
  const int wm = wave / Cfg::kWGN, wn = wave % Cfg::kWGN;   // this wave's block of the tile
  lds_bf16_t* const As = smem;                       // stage s of A at As + s * kLdsA
  lds_bf16_t* const Bs = smem + 2 * Cfg::kLdsA;      // stage s of B at Bs + s * kLdsB

  // acc[i][j]: rows wm*WM + 32 i .. of C, columns wn*WN + 32 j ..; held transposed:
  // register r of lane l is row (l % 32), column 8 (r/4) + 4 (l/32) + r % 4 of the 32x32 block.
  f32x16_t acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // A fragment of lane l: row l % 32 of a 32-row block, k = 8 (l/32) .. + 7 of a 16-step.
  // B fragment of lane l: column l % 32 of a 32-column block, same k; fetched as two transposing
  // reads of 4 k each.  In a 16-lane group, lane i points at row (i/4), columns 4 (i%4) .. + 3 of
  // the 4 x 16 block the group transposes, and receives the 4 rows of column i.
  const int half = lane / 32, l32 = lane % 32, l16 = lane % 16;
  const int a_off = (wm * Cfg::WM + l32) * kPitchA + half * 8;
  const int b_off = (half * 8 + l16 / 4) * Cfg::kPitchB + wn * Cfg::WN + ((lane / 16) % 2) * 16 + (l16 % 4) * 4;

  auto multiply_stage = [&](int stage) {
    const lds_bf16_t* a_lds = As + stage * Cfg::kLdsA + a_off;
    const lds_bf16_t* b_lds = Bs + stage * Cfg::kLdsB + b_off;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8_t af[FM], bfr[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) af[i] = *(const lds_bf16x8_t*)(a_lds + i * 32 * kPitchA + kk * 16);
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const lds_bf16_t* p = b_lds + kk * 16 * Cfg::kPitchB + j * 32;
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p);
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p + 4 * Cfg::kPitchB));
        const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bfr[j] = __builtin_bit_cast(bf16x8_t, both);
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
  };

  // Software pipeline: while k-step kt is multiplied out of LDS stage kt % 2, the global loads of
  // step kt+1 are in flight into registers; they are committed to the other stage afterwards.
  const int nk = (K + kBK - 1) / kBK;
  if constexpr (DEEP) {
    // While step kt is multiplied out of LDS, the loads of steps kt+1 .. kt+D sit in D register slots.
    // The steady loop is unrolled D times (static slot indices; D even, so the LDS stage is static too)
    // and issues unconditionally, so the wait before each commit is for exactly one step; the last D
    // steps drain the ring without issuing.
    constexpr int D = Cfg::kDepth;
    static_assert(D >= 2 && D % 2 == 0, "even depth");
    typename ALoader::Regs ra[D];
    typename BLoader::Regs rb[D];
#pragma unroll
    for (int u = 0; u < D; ++u) {
      la.fetch(ra[u], u * kBK, tid);
      lb.fetch(rb[u], u * kBK, tid);
    }
    la.commit(ra[0], As, tid);
    lb.commit(rb[0], Bs, tid);
    __syncthreads();
    int kt0 = 0;
    for (; kt0 + D < nk; kt0 += D) {
#pragma unroll
      for (int u = 0; u < D; ++u) {
        la.fetch(ra[u], (kt0 + u + D) * kBK, tid);        // slot u is free: its step went to LDS one step ago
        lb.fetch(rb[u], (kt0 + u + D) * kBK, tid);
        __builtin_amdgcn_sched_barrier(0);                 // the loads go out before anything waits
        multiply_stage(u & 1);
        la.commit(ra[(u + 1) % D], As + ((u + 1) & 1) * Cfg::kLdsA, tid);
        lb.commit(rb[(u + 1) % D], Bs + ((u + 1) & 1) * Cfg::kLdsB, tid);
        __syncthreads();
      }
    }
#pragma unroll
    for (int u = 0; u < D; ++u) {
      multiply_stage(u & 1);
      if (u + 1 < D) {
        la.commit(ra[u + 1], As + ((u + 1) & 1) * Cfg::kLdsA, tid);
        lb.commit(rb[u + 1], Bs + ((u + 1) & 1) * Cfg::kLdsB, tid);
        if (u + 2 == D) lb.finish(Bs + ((u + 1) & 1) * Cfg::kLdsB, tid);      // that was the last k-step
      }
      __syncthreads();
    }
    gemm_epilogue<Cfg>(acc, (lds_f32_t*)smem, C, R, ldc, rows_left, cols_left, ep, row_vec_off, col_vec_off);
    return;
  }
  typename ALoader::Regs ra;
  typename BLoader::Regs rb;
  la.fetch(ra, 0, tid);
  lb.fetch(rb, 0, tid);
  la.commit(ra, As, tid);
  lb.commit(rb, Bs, tid);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
      la.fetch(ra, (kt + 1) * kBK, tid);
      lb.fetch(rb, (kt + 1) * kBK, tid);
    }
    multiply_stage(cur);
    if (kt + 1 < nk) {
      la.commit(ra, As + (cur ^ 1) * Cfg::kLdsA, tid);
      lb.commit(rb, Bs + (cur ^ 1) * Cfg::kLdsB, tid);
    }
    __syncthreads();
  }

  gemm_epilogue<Cfg>(acc, (lds_f32_t*)smem, C, R, ldc, rows_left, cols_left, ep, row_vec_off, col_vec_off);
}

}  // namespace nf
