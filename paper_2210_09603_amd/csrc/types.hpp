// Element and vector types, kernel parameters, LDS swizzles and the matrix-core wrappers shared by every kernel
// of the library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace hidet {

using f16 = _Float16;
using bf16 = __bf16;
typedef f16 f16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef f16 f16x4 __attribute__((ext_vector_type(4)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

enum : int { L_KC = 0, L_MC = 1 };                    // operand contiguity
// how a chunk is fetched from global memory; LD_IM2COL_TAP is the img2col gather over a K axis ordered (kh, kw, ic)
// with ic fastest (weights repacked to match), so that a K tile lies within one filter tap
enum : int { LD_VEC = 0, LD_ELEM = 1, LD_IM2COL = 2, LD_IM2COL_TAP = 3 };
enum : int { MAP_PLAIN = 0, MAP_NCHW = 1 };           // output index map
enum : int { SCHED_SIMPLE = 0, SCHED_PINGPONG = 1, SCHED_AHEAD = 2, SCHED_KSPLIT = 3 };  // main-loop schedule

// Division of a non-negative 31-bit integer by a divisor fixed at launch: floor(n / d) =
// (n * mul) >> shift with mul = ceil(2^shift / d), shift = 31 + ceil(log2 d), which is exact for
// every 0 <= n < 2^31 (Granlund and Montgomery, "Division by invariant integers using
// multiplication", Theorem 4.2).  Two instructions instead of the forty-odd of a hardware-less
// 32-bit division; the img2col gather divides for every chunk it fetches.
struct FastDiv {
  unsigned int mul;
  unsigned int shift;
#if defined(__HIPCC__)
  __host__ __device__
#endif
  int div(int n) const {
    return (int)(((unsigned long long)(unsigned int)n * mul) >> shift);
  }
};

inline FastDiv make_fastdiv(long long d) {
  FastDiv f;
  unsigned int l = 0;
  while ((1LL << l) < d) ++l;
  f.shift = 31 + l;
  const unsigned __int128 one = 1;
  f.mul = (unsigned int)(((one << f.shift) + (unsigned __int128)d - 1) / (unsigned __int128)d);
  return f;
}

// Geometry of the implicit-GEMM convolution.  The GEMM column index enumerates output positions row by
// row with every output row padded to OWP = roundup(OW, 8) columns: n = (image * OH + oh) * OWP + ow.  A
// 16-byte chunk of the img2col matrix (8 consecutive n at 16 bits) then never leaves its output row, so
// for stride 1 it is 8 consecutive pixels of one input row -- one load instead of eight.  Columns with
// ow >= OW are dummies: their products are computed and never stored.
struct ConvGeom {
  int IC, H, W, KH, KW, sh, sw, ph, pw, OH, OW, OWP;
  int numel_x;                         // elements of the input tensor (bounds of the whole-chunk loads)
  FastDiv d_khw, d_kw, d_owp, d_oh;    // dividers by KH*KW, KW, OWP, OH
  int HW;                              // H * W
  FastDiv d_ic;                        // divider by IC (tap-major K order: k = (kh * KW + kw) * IC + ic)
};

struct GemmParams {
  const void* A;
  const void* B;
  void* C;
  const void* bias;
  const void* residual;
  int M, N, K;
  long long lda, ldb, ldc, ldr;
  long long strideA, strideB, strideC, strideR;
  float alpha;
  int bias_axis;  // 0 none, 1 per column, 2 per row
  int relu;
  int vec_store;  // groups of 4 consecutive output columns are contiguous in memory and may use one access:
                  // 0 no, 1 yes at element alignment, 2 yes and every group is aligned to 4 elements,
                  // 3 as 2 and the groups are written through the L2 (row-major 16-bit output with rows >= 4 KB apart)
  int tiles_m, tiles_n, group;
  int total_blocks;
  int k_slices;     // > 1: parallel reduction on K -- workgroup z of a tile works on K range [z*k_slice_len, ...)
  int k_slice_len;  // and writes raw fp32 partial sums to slice z of the workspace (C points at the workspace)
  int relu_a, relu_b;   // fused input prologue: the operand's elements pass through ReLU on their way into LDS
  int out_map;          // MAP_PLAIN kernels: 0 row-major [M][ldc], 1 head split (see row_offset / col_offset)
  int map_seq, map_d;   // head split: rows per sequence, columns per head
  int map_heads;        // head split: N / map_d
  FastDiv d_seq, d_hd;  // dividers by map_seq and map_d
  ConvGeom g;           // img2col geometry (LD_IM2COL) and NCHW map (MAP_NCHW)
  long long out_inner;  // MAP_NCHW: OH*OW
  long long out_outer;  // MAP_NCHW: OC*OH*OW
};

// ---------------------------------------------------------------------------------------------
// LDS swizzles.  Tiles are stored without padding; bank conflicts are avoided by XOR-ing the
// chunk index with a function of the row, which keeps every row a permutation of itself.
//   KC tiles are read with one 16-byte read per lane: consecutive lanes read the same chunk
//   column of consecutive rows, so consecutive rows must land in different bank groups.
//   MC tiles are read with the transposing 8-byte read: a group of 16 lanes reads 4 consecutive
//   k rows x 32 bytes, so those 4 rows must land in different bank groups.
// Any per-row permutation is correct (loads and fragment reads apply the same one); these were
// chosen with an LDS micro-benchmark so that the fragment reads run at the LDS peak
// (256 B/clk for 16-byte reads, about 160 B/clk for the transposing read).
// ---------------------------------------------------------------------------------------------
template <int CPR, int MI>
__device__ __forceinline__ constexpr int swz_kc(int row) {
  // Chosen per MFMA shape from measurements (LDS micro-benchmark and the SQ_LDS_BANK_CONFLICT counter
  // of the running kernel): in the 32x32 fragment read the 32 lanes of a half-wave are 32 consecutive
  // rows of one chunk column; in the 16x16 read they are 16 consecutive rows times two adjacent chunk
  // columns.  Rows that start at the same bank must spread over all chunk positions in the first case
  // and must keep the two columns apart in the second.
  if constexpr (MI == 32) {
    if constexpr (CPR >= 16) return row & 15;
    if constexpr (CPR == 8) return (row & 7) ^ ((row >> 3) & 1);
    if constexpr (CPR == 4) return ((row >> 1) & 3) ^ ((row >> 3) & 1);
  } else {
    if constexpr (CPR >= 16) return ((row & 1) * 3) | ((row & 6) << 1);
    if constexpr (CPR == 8) return (((row >> 1) & 1) * 3) | (((row >> 2) & 1) << 2);
    if constexpr (CPR == 4) return ((row >> 2) & 1) * 3;
  }
  return 0;
}
template <int CPR, int MI>
__device__ __forceinline__ constexpr int swz_mc(int k) {
  if constexpr (CPR >= 16 && MI == 32) {
    return (0xCA60 >> (4 * (k & 3))) & 15;  // k % 4 -> 0, 6, 10, 12 (a lookup packed into one constant)
  }
  if constexpr (CPR >= 16 && MI == 16) {
    // one 16x16 transposing read touches k rows kb..kb+3 and kb+8..kb+11 in the same cycle
    return 2 * ((k & 3) | (((k >> 3) & 1) << 2));
  }
  if constexpr (CPR == 8) return (k & 3) * 2;
  if constexpr (CPR == 4) return ((k >> 1) & 1) * 2;
  return 0;
}

// ---------------------------------------------------------------------------------------------
// Matrix-core wrappers.  D = A.B + C with A: MI x k, B: k x MI; lane l supplies row (l % MI) of A
// and column (l % MI) of B, both for the k group (l / MI).
// ---------------------------------------------------------------------------------------------
template <int MI>
struct AccT;
template <>
struct AccT<32> {
  using type = f32x16;
};
template <>
struct AccT<16> {
  using type = f32x4;
};

__device__ __forceinline__ f32x16 mfma_op(f16x8 a, f16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma_op(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_op(f16x8 a, f16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_op(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma_op(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma_op(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

template <typename T>
struct FragT;  // what one lane feeds to one MFMA
template <>
struct FragT<f16> {
  using type = f16x8;
};
template <>
struct FragT<bf16> {
  using type = bf16x8;
};
template <>
struct FragT<float> {
  using type = float;
};

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(f16 v) { return (float)v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename TO>
__device__ __forceinline__ TO from_f32(float v) {
  return (TO)v;  // fp32 -> fp16/bf16 conversions round to nearest even
}

}  // namespace hidet
