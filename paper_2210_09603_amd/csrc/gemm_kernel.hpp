// The scheduled matrix-multiplication tensor program (Hidet paper, Sections 2.2, 3.1, 5.1) for
// CDNA4 / gfx950, written once as a template over a tile configuration.
//
//   step 1  block-level task mapping: one workgroup per BM x BN tile of C (x batch)
//   step 2  cooperative, predicated global -> LDS loads of a BM x BK tile of A and a BK x BN tile
//           of B; the lane -> element assignment is the task mapping repeat(n,1) o spatial(r,c)
//           of the paper's cooperative-loading example.  Prologue operators (plain, transposed,
//           img2col gather) are fused here: they only change how an element's address is formed.
//   step 3  double buffering: the next tile travels global -> registers while the matrix cores
//           work on the current LDS buffer, and is written to the other buffer afterwards
//           (gemm_kernel).  The large-tile schedule (gemm_kernel_pingpong) goes further: a ring
//           of four LDS stages filled by direct global -> LDS loads three stages ahead, and the
//           two wavefronts of every SIMD half a step apart, one on the matrix cores while the
//           other reads LDS.
//   step 4  wave-level task mapping spatial(WAVES_M, WAVES_N) o repeat(FM, FN) of MFMA tiles,
//           fp32 accumulators in registers
//   step 5  fused epilogue on the accumulators (alpha, bias, residual, ReLU, cast) and predicated
//           store through an index map (row-major C, or NCHW for convolution)
//
// Conventions inside this file: an operand tile is "KC" when K is its contiguous dimension
// (row-major A, transposed B) and "MC" when the M/N dimension is contiguous (row-major B,
// transposed A, img2col matrix).  A "chunk" is 16 bytes: 8 fp16/bf16 or 4 fp32 elements along
// the contiguous dimension.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "taskmap.hpp"

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
enum : int { LD_VEC = 0, LD_ELEM = 1, LD_IM2COL = 2 };  // how a chunk is fetched from global memory
enum : int { MAP_PLAIN = 0, MAP_NCHW = 1 };           // output index map
enum : int { SCHED_SIMPLE = 0, SCHED_PINGPONG = 1 };  // main-loop schedule

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
                  // 0 no, 1 yes at element alignment, 2 yes and every group is aligned to 4 elements
  int tiles_m, tiles_n, group;
  int total_blocks;
  int k_slices;     // > 1: parallel reduction on K -- workgroup z of a tile works on K range [z*k_slice_len, ...)
  int k_slice_len;  // and writes raw fp32 partial sums to slice z of the workspace (C points at the workspace)
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

// ---------------------------------------------------------------------------------------------
// Tile configuration: everything the template needs, plus derived constants.
// ---------------------------------------------------------------------------------------------
template <typename T_, typename TO_, int BM_, int BN_, int BK_, int WAVES_M_, int WAVES_N_, int MI_, int LA_, int LB_,
          int MODE_A_, int MODE_B_, int MAPPER_, int SCHED_ = SCHED_SIMPLE>
struct GemmConfig {
  using T = T_;
  using TO = TO_;
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, MI = MI_;
  static constexpr int LA = LA_, LB = LB_, MODE_A = MODE_A_, MODE_B = MODE_B_, MAPPER = MAPPER_, SCHED = SCHED_;
  static constexpr bool IS_F32 = sizeof(T) == 4;
  static constexpr int VEC = 16 / (int)sizeof(T);
  static constexpr int NWAVES = WAVES_M * WAVES_N;
  static constexpr int NT = NWAVES * 64;
  static constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;  // wave tile
  static constexpr int FM = WTM / MI, FN = WTN / MI;            // MFMA tiles per wave: repeat(FM, FN)
  static constexpr int KGROUPS = 64 / MI;                       // k groups across the lanes of one MFMA
  static constexpr int KSTEP = IS_F32 ? KGROUPS : 8 * KGROUPS;  // k extent of one MFMA
  static constexpr int KS = BK / KSTEP;
  static constexpr int A_BYTES = BM * BK * (int)sizeof(T);
  static constexpr int B_BYTES = BN * BK * (int)sizeof(T);
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int STAGES = (SCHED == SCHED_PINGPONG) ? 4 : 2;
  // per-wave transposition regions of the epilogue: MI rows of the wave tile in fp32, rows padded by 16 bytes
  static constexpr int EPI_BYTES = NWAVES * MI * (WTN * 4 + 16);
  static constexpr int LDS_BYTES = STAGES * STAGE_BYTES > EPI_BYTES ? STAGES * STAGE_BYTES : EPI_BYTES;
  static constexpr int NL_A = BM * BK / VEC / NT;  // chunks per thread per tile
  static constexpr int NL_B = BN * BK / VEC / NT;
  static_assert(BM % (WAVES_M * MI) == 0 && BN % (WAVES_N * MI) == 0, "wave tiles must be whole MFMA tiles");
  static_assert(BK % KSTEP == 0, "BK must be a multiple of the MFMA k extent");
  static_assert(NL_A >= 1 && NL_B >= 1 && NL_A * NT * VEC == BM * BK && NL_B * NT * VEC == BN * BK,
                "every thread must load the same whole number of chunks");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS capacity of a gfx950 compute unit");
};

// Cooperative-load task mapping of one operand tile: which chunk (row, chunk-in-row) of the tile
// thread `t` loads as its q-th load.  The grid is (rows, chunks per row) of the tile as stored.
template <int ROWS, int CPR, int NT>
struct LoadMapRowMajor {
  // consecutive threads walk along a row first: repeat(n, 1) o spatial(NT / CPR, CPR)
  static_assert(NT % CPR == 0 && (ROWS * CPR) % NT == 0 && ROWS % (NT / CPR) == 0, "tile does not split evenly");
  using Map = tmap::Compose<tmap::Repeat<ROWS * CPR / NT, 1>, tmap::Spatial<NT / CPR, CPR>>;
  __device__ static constexpr tmap::Task task(int t, int q) { return Map::task(t, q); }
};
template <int ROWS, int CPR, int NT, bool WIDE = (ROWS > NT)>
struct LoadMapColMajor;  // consecutive threads walk down the rows first (grid is (chunk, row))
template <int ROWS, int CPR, int NT>
struct LoadMapColMajor<ROWS, CPR, NT, false> {
  static_assert(NT % ROWS == 0 && CPR % (NT / ROWS) == 0, "tile does not split evenly");
  using Map = tmap::Compose<tmap::Repeat<CPR * ROWS / NT, 1>, tmap::Spatial<NT / ROWS, ROWS>>;
  __device__ static constexpr tmap::Task task(int t, int q) {
    const tmap::Task x = Map::task(t, q);
    return tmap::Task{x.j, x.i};
  }
};
template <int ROWS, int CPR, int NT>
struct LoadMapColMajor<ROWS, CPR, NT, true> {
  static_assert(ROWS % NT == 0, "tile does not split evenly");
  using Map = tmap::Compose<tmap::Repeat<CPR, ROWS / NT>, tmap::Spatial<1, NT>>;
  __device__ static constexpr tmap::Task task(int t, int q) {
    const tmap::Task x = Map::task(t, q);
    return tmap::Task{x.j, x.i};
  }
};

// ---------------------------------------------------------------------------------------------
// One operand (A or B) of one workgroup: global source + LDS tile.
//   ROWS   extent of the tile along M (for A) or N (for B)
//   LAYOUT L_KC: element (r, k) at src[r*ld + k];  L_MC: element (k, r) at src[k*ld + r]
// LDS layout, 16-bit types: same orientation as the source, chunk-swizzled (see swz_*).
// LDS layout, fp32: always [k][r] (each lane reads a single float per MFMA, consecutive lanes
// read consecutive r), so a KC source is transposed on its way into LDS.
// ---------------------------------------------------------------------------------------------
template <typename T, int ROWS, int BK, int LAYOUT, int MODE, int NT, int MI>
struct Operand {
  static constexpr bool IS_F32 = sizeof(T) == 4;
  static constexpr int VEC = 16 / (int)sizeof(T);
  static constexpr int CPR = (LAYOUT == L_KC) ? BK / VEC : ROWS / VEC;  // chunks per stored row
  static constexpr int SROWS = (LAYOUT == L_KC) ? ROWS : BK;             // stored rows
  static constexpr int NL = ROWS * BK / VEC / NT;
  static constexpr int KGROUPS = 64 / MI;
  using LoadMap = typename std::conditional<(IS_F32 && LAYOUT == L_KC), LoadMapColMajor<SROWS, CPR, NT>,
                                            LoadMapRowMajor<SROWS, CPR, NT>>::type;
  using Frag = typename FragT<T>::type;

  const T* src;      // origin of this workgroup's panel: row r0 (KC) or column r0 (MC), k = 0
  long long ld;
  int rows_left;     // valid extent along ROWS from the panel origin (may exceed ROWS, may be <= 0)
  int K;             // extent of this workgroup's K range
  int kofs;          // global k index where that range starts (needed by the img2col gather)
  int r0;            // global row/column of the panel origin (needed by the img2col gather)

  // ---- global -> registers ------------------------------------------------------------------
  __device__ __forceinline__ u32x4 gather(int q, int sr, int sc, int k0, const ConvGeom& g) const {
    // Element by element, zero-filled: any alignment, any edge.  Every load is issued unconditionally
    // from a clamped (always valid) address and the predicate is applied to the value, so the VEC loads
    // of a chunk are in flight together instead of waiting for one another behind branches.
    T tmp[VEC];
    if constexpr (MODE == LD_IM2COL) {
      // stored row sr = k index (ic, kh, kw); the chunk = VEC consecutive output positions of one output
      // row.  What depends on the positions was prepared by init(); what depends on k is computed here.
      const int kk = k0 + sr;
      const int k = kofs + kk;
      const int ic = g.d_khw.div(k), rem = k - ic * (g.KH * g.KW);
      const int kh = g.d_kw.div(rem), kw = rem - kh * g.KW;
      const int xy = pxy[q];
      const int ih = (int)(short)(xy & 0xffff) + kh, iwf = (xy >> 16) + kw;  // input row, input column of element 0
      const int cnt = pcnt[q];                                               // real positions in the chunk
      const bool row_ok = kk < K && (unsigned)ih < (unsigned)g.H;
      const int start = pofs[q] + (ic * g.H + kh) * g.W + kw;                // element offset of (ih, iwf)
      if (g.sw <= 2 && g.numel_x >= 2 * VEC) {  // (a tensor smaller than the window has no valid window)
        // Strides 1 and 2: element e is input pixel (ih, iwf + e * sw), so the chunk lies in one window of
        // VEC * sw consecutive pixels.  Pixels left of the row (padding), right of it, and positions past
        // the end of the output row read as zero: keep e in [lo, hi).
        const int sw = g.sw;
        int lo = iwf < 0 ? (-iwf + sw - 1) / sw : 0;
        int hi = iwf < g.W ? (g.W - 1 - iwf) / sw + 1 : 0;
        hi = hi < cnt ? hi : cnt;
        if (!row_ok) hi = 0;
        const bool any = hi > lo;
        const bool inside = start >= 0 && start + VEC * sw <= g.numel_x;  // the whole window lies in the tensor
        if (any && !inside) {
          // first or last pixels of the tensor: the window would leave the allocation
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            const bool ok = e >= lo && e < hi;
            const T v = src[ok ? start + e * sw : 0];
            tmp[e] = ok ? v : (T)0.0f;
          }
          return __builtin_bit_cast(u32x4, tmp);
        }
        // unconditional loads from a valid address; the mask makes them exact
        const T* win = src + ((any && inside) ? start : 0);
        u32x4 v = reinterpret_cast<const Unaligned*>(win)->v;
        if (sw == 2) {
          const u32x4 w = reinterpret_cast<const Unaligned*>(win + VEC)->v;
          if constexpr (IS_F32) {
            v = u32x4{v[0], v[2], w[0], w[2]};
          } else {  // even 16-bit elements of the 16 loaded
            v = u32x4{(v[0] & 0xffffu) | (v[1] << 16), (v[2] & 0xffffu) | (v[3] << 16),
                      (w[0] & 0xffffu) | (w[1] << 16), (w[2] & 0xffffu) | (w[3] << 16)};
          }
        }
        if (!any) lo = hi = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          if constexpr (IS_F32) {
            v[i] = (i >= lo && i < hi) ? v[i] : 0u;
          } else {
            const unsigned int m_lo = (2 * i >= lo && 2 * i < hi) ? 0x0000ffffu : 0u;
            const unsigned int m_hi = (2 * i + 1 >= lo && 2 * i + 1 < hi) ? 0xffff0000u : 0u;
            v[i] &= (m_lo | m_hi);
          }
        }
        return v;
      }
      // Other strides: element e is input pixel (ih, iwf + e * sw); one clamped load per element.
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const int iw = iwf + e * g.sw;
        const bool ok = row_ok && e < cnt && (unsigned)iw < (unsigned)g.W;
        const T v = src[ok ? start + e * g.sw : 0];
        tmp[e] = ok ? v : (T)0.0f;
      }
    } else {
      // Element mode: rows are not 16-byte aligned (odd leading dimension, offset pointer).  A chunk that lies
      // entirely inside the matrix is still fetched with one 16-byte load -- the address is only element
      // aligned, which global loads accept on this target -- and only chunks that straddle an edge fall back
      // to one predicated load per element.
      long long base;
      int valid;  // elements of the chunk inside the matrix
      bool whole;  // the 16 bytes of the chunk may be read at once
      if constexpr (LAYOUT == L_KC) {
        base = (long long)sr * ld + (k0 + sc);
        valid = sr < rows_left ? K - (k0 + sc) : 0;
        // a chunk that sticks out along K is read whole and masked below, unless it ends the last row
        whole = valid >= VEC || (valid > 0 && (kofs + k0 + sc + VEC <= ld || sr < rows_left - 1));
      } else {
        base = (long long)(k0 + sr) * ld + sc;
        valid = k0 + sr < K ? rows_left - sc : 0;
        // a chunk that sticks out along M/N may be read whole (see init) unless it ends the last row
        whole = valid >= VEC || (valid > 0 && (r0 + sc + VEC <= ld || k0 + sr < K - 1));
      }
      if (valid <= 0) return u32x4{0u, 0u, 0u, 0u};
      if (whole) {
        u32x4 v = reinterpret_cast<const Unaligned*>(src + base)->v;
        if constexpr (LAYOUT == L_KC) {
          // along K what lies beyond the matrix must contribute exact zeros
          if (valid < VEC) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              if constexpr (IS_F32)
                v[i] = valid > i ? v[i] : 0u;
              else
                v[i] &= valid >= 2 * i + 2 ? 0xffffffffu : (valid == 2 * i + 1 ? 0x0000ffffu : 0u);
            }
          }
        }
        return v;
      }
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        const bool ok = e < valid;
        const T v = src[ok ? base + e : 0];
        tmp[e] = ok ? v : (T)0.0f;
      }
    }
    return __builtin_bit_cast(u32x4, tmp);
  }

  // Vector mode (LD_VEC): the host guarantees 16-byte aligned rows and that no chunk straddles the
  // edge of the matrix (K, resp. the M/N extent, is a multiple of the chunk length).  Chunks that lie
  // outside the matrix along M/N are redirected to the last valid row / chunk: they only feed output
  // rows or columns that are never stored, so any finite or non-finite value is harmless there.
  // Along K a chunk outside the matrix must read as zero; that can only happen in the last K tile.
  int off[NL];  // element offset of each chunk from `src` at k = 0 (vector mode only)
  // Element mode: the same idea at element alignment.  eoff = offset of the chunk at k = 0, nv = how many
  // of its VEC elements lie inside the matrix along M/N (a property of the chunk, not of the K tile).
  // Chunks entirely outside are redirected to a chunk inside (nv = VEC; they feed outputs that are never
  // stored).  A chunk that straddles the M/N edge is still read whole: the bytes past the edge are the
  // padding of the row or the beginning of the next row -- valid memory, and values that only reach
  // outputs that are never stored.  The exception is the last row of the operand, where "past the edge"
  // may be past the allocation: nv = -(valid elements) marks such chunks, and the one row concerned is
  // fetched element by element (so is everything in a matrix narrower than one chunk, 0 <= nv < VEC).
  static constexpr int NE = (MODE == LD_ELEM) ? NL : 1;
  long long eoff[NE];
  int nv[NE];
  struct __attribute__((packed, aligned(sizeof(T)))) Unaligned {
    u32x4 v;
  };
  // img2col mode only, per chunk: offset of the input pixel (image, oh*sh - ph, ow*sw - pw) of channel 0 that
  // element 0 of the chunk reads at (kh, kw) = (0, 0) (may be negative), that pixel's row and column packed as
  // two signed 16-bit fields, and how many of the chunk's positions are real (ow < OW and inside the matrix).
  static constexpr int NP = (MODE == LD_IM2COL) ? NL : 1;
  int pofs[NP];
  int pxy[NP];
  int pcnt[NP];

  __device__ __forceinline__ void init(int tid, const ConvGeom& g) {
    if constexpr (MODE == LD_IM2COL) {
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        const tmap::Task t = LoadMap::task(tid, q);
        const int sc = t.j * VEC;
        const int p = r0 + sc;                       // GEMM column of element 0
        const int r = g.d_owp.div(p), ow = p - r * g.OWP;  // r = image * OH + oh
        const int img = g.d_oh.div(r), oh = r - img * g.OH;
        const int ih0 = oh * g.sh - g.ph, iw0 = ow * g.sw - g.pw;
        pofs[q] = (img * g.IC * g.H + ih0) * g.W + iw0;
        pxy[q] = (ih0 & 0xffff) | (iw0 << 16);
        int cnt = g.OW - ow;
        cnt = cnt < rows_left - sc ? cnt : rows_left - sc;
        pcnt[q] = cnt < 0 ? 0 : (cnt > VEC ? VEC : cnt);
      }
    }
    if constexpr (MODE == LD_ELEM) {
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        const tmap::Task t = LoadMap::task(tid, q);
        const int sr = t.i, sc = t.j * VEC;
        if constexpr (LAYOUT == L_KC) {
          const int r = sr < rows_left ? sr : rows_left - 1;
          eoff[q] = (long long)r * ld + sc;
          nv[q] = VEC;
        } else {
          const int rem = rows_left - sc;
          int c = sc, n = rem;
          if (rem >= VEC) {
            n = VEC;
          } else if (rem > 0) {
            n = (r0 + sc + VEC <= ld) ? VEC : -rem;  // the padding of the row covers the over-read
          } else {
            n = rows_left >= VEC ? VEC : 0;  // a matrix narrower than one chunk has nowhere to redirect to
            c = rows_left >= VEC ? rows_left - VEC : 0;
          }
          eoff[q] = (long long)sr * ld + c;
          nv[q] = n;
        }
      }
    }
    if constexpr (MODE == LD_VEC) {
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        const tmap::Task t = LoadMap::task(tid, q);
        const int sr = t.i, sc = t.j * VEC;
        if constexpr (LAYOUT == L_KC) {
          const int r = sr < rows_left ? sr : rows_left - 1;
          off[q] = r * (int)ld + sc;
        } else {
          const int c = sc + VEC <= rows_left ? sc : rows_left - VEC;
          off[q] = sr * (int)ld + c;
        }
      }
    }
  }

  // Direct global -> LDS loads (vector mode, 16-bit types).  Lane l of a wave writes its 16 bytes at
  // LDS[base + 16*l], so the LDS side of the cooperative load is fixed -- thread t's q-th load fills
  // stored position q*NT + t of the tile -- and the swizzle moves to the global side: the thread
  // fetches the logical chunk that belongs at that position.  The instruction is issued through
  // inline assembly and tracked by hand with s_waitcnt vmcnt(n): the schedule that uses it keeps
  // several stages in flight and waits for the oldest only.
  int doff[NL];
  __device__ __forceinline__ void init_direct(int tid) {
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const int pos = q * NT + tid;
      const int row = pos / CPR, pc = pos % CPR;
      const int lc = pc ^ ((LAYOUT == L_KC) ? swz_kc<CPR, MI>(row) : swz_mc<CPR, MI>(row));
      if constexpr (LAYOUT == L_KC) {
        const int r = row < rows_left ? row : rows_left - 1;
        doff[q] = r * (int)ld + lc * VEC;
      } else {
        const int c = lc * VEC + VEC <= rows_left ? lc * VEC : rows_left - VEC;
        doff[q] = row * (int)ld + c;
      }
    }
  }
  // `tile_lds`: LDS byte address of the tile; `wave`: wave index (both wave-uniform).
  __device__ __forceinline__ void load_direct(unsigned tile_lds, int wave, int k0) const {
    const T* base = (LAYOUT == L_KC) ? src + k0 : src + (long long)k0 * ld;
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const T* g = base + doff[q];
      const unsigned dst = tile_lds + (unsigned)((q * NT + wave * 64) * 16);
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(dst) : "memory");
    }
  }

  // A K tile that lies entirely inside the matrix: no predicates at all in vector mode.
  __device__ __forceinline__ void load_full(u32x4 (&regs)[NL], int tid, int k0, const ConvGeom& g) const {
    if constexpr (MODE == LD_VEC) {
      const T* base = (LAYOUT == L_KC) ? src + k0 : src + (long long)k0 * ld;
#pragma unroll
      for (int q = 0; q < NL; ++q) regs[q] = *reinterpret_cast<const u32x4*>(base + off[q]);
    } else if constexpr (MODE == LD_ELEM) {
      const T* base = (LAYOUT == L_KC) ? src + k0 : src + (long long)k0 * ld;
#pragma unroll
      for (int q = 0; q < NL; ++q) {
        const tmap::Task t = LoadMap::task(tid, q);
        if (nv[q] == VEC || (nv[q] < 0 && k0 + t.i < K - 1)) {
          regs[q] = reinterpret_cast<const Unaligned*>(base + eoff[q])->v;
        } else {
          const int cnt = nv[q] < 0 ? -nv[q] : nv[q];
          T tmp[VEC];
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            const bool ok = e < cnt;
            const T v = base[ok ? eoff[q] + e : eoff[q]];
            tmp[e] = ok ? v : (T)0.0f;
          }
          regs[q] = __builtin_bit_cast(u32x4, tmp);
        }
      }
    } else {
      load_edge(regs, tid, k0, g);
    }
  }

  // The last, partial K tile (and every tile of the element-wise modes).
  __device__ __forceinline__ void load_edge(u32x4 (&regs)[NL], int tid, int k0, const ConvGeom& g) const {
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const tmap::Task t = LoadMap::task(tid, q);
      const int sr = t.i, sc = t.j * VEC;  // stored row, first stored column of the chunk
      if constexpr (MODE == LD_VEC) {
        const T* base = (LAYOUT == L_KC) ? src + k0 : src + (long long)k0 * ld;
        const bool inside = (LAYOUT == L_KC) ? (k0 + sc < K) : (k0 + sr < K);
        u32x4 v = {0u, 0u, 0u, 0u};
        if (inside) v = *reinterpret_cast<const u32x4*>(base + off[q]);
        regs[q] = v;
      } else {
        regs[q] = gather(q, sr, sc, k0, g);
      }
    }
  }

  // ---- registers -> LDS ---------------------------------------------------------------------
  __device__ __forceinline__ void store(const u32x4 (&regs)[NL], int tid, unsigned char* tile) const {
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const tmap::Task t = LoadMap::task(tid, q);
      if constexpr (!IS_F32) {
        const int swz = (LAYOUT == L_KC) ? swz_kc<CPR, MI>(t.i) : swz_mc<CPR, MI>(t.i);
        *reinterpret_cast<u32x4*>(tile + (t.i * CPR + (t.j ^ swz)) * 16) = regs[q];
      } else if constexpr (LAYOUT == L_MC) {
        *reinterpret_cast<u32x4*>(tile + (t.i * CPR + t.j) * 16) = regs[q];
      } else {
        // fp32, KC source: row t.i, k = 4*t.j + e  ->  LDS [k][row]
        unsigned int* w = reinterpret_cast<unsigned int*>(tile);
#pragma unroll
        for (int e = 0; e < 4; ++e) w[(t.j * 4 + e) * ROWS + t.i] = regs[q][e];
      }
    }
  }

  // ---- LDS -> MFMA fragment -----------------------------------------------------------------
  // Fragment `f` (rows f*MI .. f*MI+MI-1 of the wave's sub-tile starting at row `w0`), k step `ks`.
  __device__ __forceinline__ Frag fragment(const unsigned char* tile, int lane, int w0, int f, int ks) const {
    if constexpr (IS_F32) {
      const int k = ks * KGROUPS + lane / MI;
      const int r = w0 + f * MI + lane % MI;
      return reinterpret_cast<const float*>(tile)[k * ROWS + r];
    } else if constexpr (LAYOUT == L_KC) {
      const int r = w0 + f * MI + lane % MI;
      const int c = ks * KGROUPS + lane / MI;
      const u32x4 v = *reinterpret_cast<const u32x4*>(tile + (r * CPR + (c ^ swz_kc<CPR, MI>(r))) * 16);
      return __builtin_bit_cast(Frag, v);
    } else {
      // transposing read: within each group of 16 lanes, lane s supplies the address of 4
      // elements (k = kb + s/4, columns cb + 4*(s%4) ..+3) and receives column cb + s, k = kb..kb+3
      const int b = lane / 16, s = lane % 16;
      int kb, cb;
      if constexpr (MI == 32) {
        kb = ks * 16 + 8 * (b / 2);
        cb = w0 + f * 32 + 16 * (b % 2);
      } else {
        kb = ks * 32 + 8 * b;
        cb = w0 + f * 16;
      }
      const int k = kb + s / 4;
      const int col = cb + 4 * (s % 4);
      u32x2 h[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int kk = k + 4 * i;
        const unsigned char* addr = tile + (kk * CPR + ((col / 8) ^ swz_mc<CPR, MI>(kk))) * 16 + (col % 8) * 2;
        const i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) i16x4*)(const_cast<unsigned char*>(addr)));
        h[i] = __builtin_bit_cast(u32x2, v);
      }
      const u32x4 v = {h[0][0], h[0][1], h[1][0], h[1][1]};
      return __builtin_bit_cast(Frag, v);
    }
  }
};

// Output index maps (the index half of an epilogue, Section 5.2).  All of them are separable,
//     offset(m, n) = row_offset(m) + col_offset(n),
// so a lane that keeps its columns computes the column part once and the row part once per row:
//   plain        m * ldc                    + n
//   NCHW (conv)  m * OH*OW                  + image * OC*OH*OW + oh * OW + ow   (n = (image * OH + oh) * OWP + ow)
//   head split   ((b * heads) * seq + s) * d + h * seq * d + f                  (m = b*seq + s, n = h*d + f;
//                the reshape-matmul-transpose sub-graph of transformer models, Section 3.2)
// DYN = false compiles the run-time choice between plain and head split out of MAP_PLAIN kernels (the
// large-tile schedule is built that way: its register budget is tight enough that the extra live values
// cost several percent of its main loop).
template <int MAPPER, bool DYN = true>
__device__ __forceinline__ long long col_offset(const GemmParams& p, int n) {
  if constexpr (MAPPER == MAP_NCHW) {
    const int r = p.g.d_owp.div(n), ow = n - r * p.g.OWP;
    const int img = p.g.d_oh.div(r), oh = r - img * p.g.OH;
    return (long long)img * p.out_outer + oh * p.g.OW + ow;
  } else {
    if (DYN && p.out_map != 0) {
      const int h = p.d_hd.div(n);
      return (long long)h * p.map_seq * p.map_d + (n - h * p.map_d);
    }
    return n;
  }
}
template <int MAPPER, bool DYN = true>
__device__ __forceinline__ long long row_offset(const GemmParams& p, int m, long long ld) {
  if constexpr (MAPPER == MAP_NCHW) {
    return (long long)m * p.out_inner;
  } else {
    if (DYN && p.out_map != 0) {
      const int b = p.d_seq.div(m), s = m - b * p.map_seq;
      return ((long long)b * p.map_heads * p.map_seq + s) * p.map_d;
    }
    return (long long)m * ld;
  }
}

// How many of the 4 columns n .. n+3 are real outputs (the rest lie beyond N, or -- convolution -- in the
// padding of an output row).
template <int MAPPER>
__device__ __forceinline__ int group_valid(const GemmParams& p, int n) {
  int left = p.N - n;
  if constexpr (MAPPER == MAP_NCHW) {
    const int r = p.g.d_owp.div(n < 0 ? 0 : n), ow = n - r * p.g.OWP;
    left = left < p.g.OW - ow ? left : p.g.OW - ow;
  }
  return left < 0 ? 0 : (left > 4 ? 4 : left);
}

// ---------------------------------------------------------------------------------------------
// Fused epilogue + predicated store of 4 consecutive output columns of one row.  `ccol` is
// col_offset(n) and `nvalid` is group_valid(n), computed by the caller once for all its rows.
// ---------------------------------------------------------------------------------------------
template <typename TO, int MAPPER, bool DYN = true>
__device__ __forceinline__ void store4(const GemmParams& p, TO* __restrict__ C, const TO* __restrict__ R,
                                       const TO* __restrict__ bias, const float (&col_bias)[4], int m, int n,
                                       long long ccol, int nvalid, const float (&acc)[4]) {
  if (m >= p.M || nvalid <= 0) return;
  const bool remap = (MAPPER == MAP_NCHW) || (DYN && p.out_map != 0);
  const long long crow = row_offset<MAPPER, DYN>(p, m, p.ldc);
  const long long rrow = remap ? crow : (long long)m * p.ldr;
  const long long off = crow + ccol, roff = rrow + ccol;
  // four consecutive elements as one access; the address need only be element aligned
  struct __attribute__((packed, aligned(sizeof(TO)))) Quad {
    TO e[4];
  };
  float v[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = p.alpha * acc[e];
  const bool whole = p.vec_store && nvalid == 4;
  if (p.bias_axis == 2) {
    const float b = to_f32(bias[m]);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += b;
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += col_bias[e];  // zeros unless the bias is per column
  }
  if (R != nullptr) {
    if (whole) {
      TO r[4];
      *reinterpret_cast<Quad*>(r) = *reinterpret_cast<const Quad*>(R + roff);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += to_f32(r[e]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (e < nvalid) {
          long long ro = roff + e;  // plain and NCHW: the group is contiguous
          if (MAPPER == MAP_PLAIN && remap) ro = rrow + col_offset<MAPPER, DYN>(p, n + e);
          v[e] += to_f32(R[ro]);
        }
      }
    }
  }
  if (p.relu) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = v[e] < 0.0f ? 0.0f : v[e];
  }
  TO o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) o[e] = from_f32<TO>(v[e]);
  if (whole) {
    // streaming stores: the output is not read again by this kernel, and lines that do not linger
    // dirty in L2 shorten the write-back at the end of the kernel
    if (p.vec_store == 2) {  // 4-element aligned address
      if constexpr (sizeof(TO) == 2)
        __builtin_nontemporal_store(*reinterpret_cast<const u32x2*>(o), reinterpret_cast<u32x2*>(C + off));
      else
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(o), reinterpret_cast<u32x4*>(C + off));
    } else {
      *reinterpret_cast<Quad*>(C + off) = *reinterpret_cast<const Quad*>(o);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (e < nvalid) {
        long long oo = off + e;
        if (MAPPER == MAP_PLAIN && remap) oo = crow + col_offset<MAPPER, DYN>(p, n + e);
        C[oo] = o[e];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Pieces shared by the kernels.
// ---------------------------------------------------------------------------------------------
struct BlockCoords {
  int batch;    // batch entry whose A and B are used
  int cbatch;   // index of the output matrix (batch entry, or batch * k_slices + slice for K-parallel partial sums)
  int m0, n0;   // tile origin
  int k_begin;  // K range of this workgroup
  int k_len;
};

// Step 1, block-level task mapping.  Workgroups are handed to the 8 accelerator dies (XCDs)
// round-robin; they are renumbered so that each die, which has a private L2, works on one
// contiguous run of tiles of the grouped traversal.
template <int BM, int BN>
__device__ __forceinline__ BlockCoords block_coords(const GemmParams& p) {
  const int total = p.total_blocks;
  const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
  const int per = total / 8, extra = total % 8;
  const int logical = xcd * per + (xcd < extra ? xcd : extra) + slot;
  const int tiles = p.tiles_m * p.tiles_n;
  const int zb = logical / tiles;
  const tmap::Task tile = tmap::GroupedSpatial{p.tiles_m, p.tiles_n, p.group}.task(logical - zb * tiles);
  BlockCoords bc;
  bc.cbatch = zb;
  bc.m0 = tile.i * BM;
  bc.n0 = tile.j * BN;
  if (p.k_slices > 1) {
    bc.batch = zb / p.k_slices;
    bc.k_begin = (zb - bc.batch * p.k_slices) * p.k_slice_len;
    const int left = p.K - bc.k_begin;
    bc.k_len = left < p.k_slice_len ? left : p.k_slice_len;
  } else {
    bc.batch = zb;
    bc.k_begin = 0;
    bc.k_len = p.K;
  }
  return bc;
}

template <class Cfg, class OpA, class OpB>
__device__ __forceinline__ void setup_operands(const GemmParams& p, const BlockCoords& bc, OpA& opa, OpB& opb) {
  using T = typename Cfg::T;
  const T* A = reinterpret_cast<const T*>(p.A) + (long long)bc.batch * p.strideA;
  const T* B = reinterpret_cast<const T*>(p.B) + (long long)bc.batch * p.strideB;
  opa.src = (Cfg::LA == L_KC) ? A + (long long)bc.m0 * p.lda + bc.k_begin : A + (long long)bc.k_begin * p.lda + bc.m0;
  opa.ld = p.lda;
  opa.rows_left = p.M - bc.m0;
  opa.K = bc.k_len;
  opa.kofs = bc.k_begin;
  opa.r0 = bc.m0;
  if constexpr (Cfg::MODE_B == LD_IM2COL)
    opb.src = B;  // the gather addresses the whole input tensor
  else
    opb.src = (Cfg::LB == L_KC) ? B + (long long)bc.n0 * p.ldb + bc.k_begin : B + (long long)bc.k_begin * p.ldb + bc.n0;
  opb.ld = p.ldb;
  opb.rows_left = p.N - bc.n0;
  opb.K = bc.k_len;
  opb.kofs = bc.k_begin;
  opb.r0 = bc.n0;
}

// Per-column bias of the 4 columns a lane owns in the epilogue, fetched before the main loop so that
// the latency disappears behind it.
template <class Cfg>
__device__ __forceinline__ void load_col_bias(const GemmParams& p, int n_wave0, int lane, float (&col_bias)[4]) {
  using TO = typename Cfg::TO;
#pragma unroll
  for (int e = 0; e < 4; ++e) col_bias[e] = 0.0f;
  if (p.bias_axis == 1) {
    const TO* bptr = reinterpret_cast<const TO*>(p.bias);
    const int n = n_wave0 + (lane % (Cfg::WTN / 4)) * 4;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (n + e < p.N) col_bias[e] = to_f32(bptr[n + e]);
  }
}

// Step 5: fused epilogue + predicated store.  The MFMAs are issued with their operands swapped, so
// an accumulator tile holds C transposed and each lane owns 4 consecutive columns of MI different
// rows.  Storing that directly would scatter 8-byte pieces over as many cache lines, so each wave
// transposes its accumulators through a private LDS region, MI rows at a time: written as they lie
// in registers, read back so that consecutive lanes hold consecutive columns of one row, and stored
// as whole 128-byte lines.  No workgroup barrier is involved: the region is private to the wave and
// a wave's LDS operations complete in order (the fences are wave-scope, LDS-only).
// Must be entered after a workgroup barrier that ends all use of the staging buffers.
template <class Cfg, class Acc, bool DYN = true>
__device__ __forceinline__ void epilogue(const GemmParams& p, const BlockCoords& bc, int wave, int lane, int wm0, int wn0,
                                         Acc (&acc)[Cfg::FM][Cfg::FN], const float (&col_bias)[4], unsigned char* smem) {
  using TO = typename Cfg::TO;
  constexpr int MI = Cfg::MI, FM = Cfg::FM, FN = Cfg::FN, WTN = Cfg::WTN;
  TO* C = reinterpret_cast<TO*>(p.C) + (long long)bc.cbatch * p.strideC;
  const TO* R = p.residual ? reinterpret_cast<const TO*>(p.residual) + (long long)bc.batch * p.strideR : nullptr;
  const TO* bias = reinterpret_cast<const TO*>(p.bias);
  constexpr int GROUPS = (MI == 32) ? 4 : 1;  // groups of 4 consecutive columns per accumulator tile
  constexpr int ROW_BYTES = WTN * 4 + 16;     // +16: consecutive rows start 4 banks apart
  constexpr int LANES_PER_ROW = WTN / 4;
  constexpr int SLOTS = MI * LANES_PER_ROW;   // 16-byte pieces per pass
  constexpr int READS = (SLOTS + 63) / 64;
  static_assert(64 % LANES_PER_ROW == 0, "a lane must keep the same 4 columns in every read-back step");
  unsigned char* region = smem + wave * (MI * ROW_BYTES);
  const int my_n = bc.n0 + wn0 + (lane % LANES_PER_ROW) * 4;  // the same 4 columns in every read-back step
  const long long my_ccol = col_offset<Cfg::MAPPER, DYN>(p, my_n);
  const int my_valid = group_valid<Cfg::MAPPER>(p, my_n);
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int gq = 0; gq < GROUPS; ++gq) {
        const int nl = j * MI + ((MI == 32) ? 8 * gq + 4 * (lane / 32) : 4 * (lane / 16));
        const f32x4 v = {acc[i][j][4 * gq + 0], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
        *reinterpret_cast<f32x4*>(region + (lane % MI) * ROW_BYTES + nl * 4) = v;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
#pragma unroll
    for (int t = 0; t < READS; ++t) {
      const int idx = t * 64 + lane;
      const int row = idx / LANES_PER_ROW, c4 = idx % LANES_PER_ROW;
      if (SLOTS % 64 == 0 || idx < SLOTS) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(region + row * ROW_BYTES + c4 * 16);
        const float vv[4] = {v[0], v[1], v[2], v[3]};
        store4<TO, Cfg::MAPPER, DYN>(p, C, R, bias, col_bias, bc.m0 + wm0 + i * MI + row, my_n, my_ccol, my_valid, vv);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
  }
}

// ---------------------------------------------------------------------------------------------
// The kernel, general schedule: two LDS stages, next tile staged through registers (the double
// buffering of Section 3.1), fragments double-buffered in registers so that LDS reads of k step
// ks+1 run under the MFMAs of k step ks.  Handles every load mode and every edge.
// ---------------------------------------------------------------------------------------------
template <class Cfg>
__global__ void __launch_bounds__(Cfg::NT) gemm_kernel(const GemmParams p) {
  using T = typename Cfg::T;
  using Acc = typename AccT<Cfg::MI>::type;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, MI = Cfg::MI, NT = Cfg::NT;
  constexpr int FM = Cfg::FM, FN = Cfg::FN, KS = Cfg::KS;
  using OpA = Operand<T, BM, BK, Cfg::LA, Cfg::MODE_A, NT, MI>;
  using OpB = Operand<T, BN, BK, Cfg::LB, Cfg::MODE_B, NT, MI>;

  __shared__ __attribute__((aligned(16))) unsigned char smem[Cfg::LDS_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid % 64;
  const int wave = tid / 64;

  const BlockCoords bc = block_coords<BM, BN>(p);  // step 1
  OpA opa;
  OpB opb;
  setup_operands<Cfg>(p, bc, opa, opb);

  // step 4 (set-up): wave-level task mapping spatial(WAVES_M, WAVES_N) o repeat(FM, FN)
  const tmap::Task wt = tmap::Spatial<Cfg::WAVES_M, Cfg::WAVES_N>::task(wave, 0);
  const int wm0 = wt.i * Cfg::WTM, wn0 = wt.j * Cfg::WTN;

  Acc acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < (int)(sizeof(Acc) / 4); ++r) acc[i][j][r] = 0.0f;

  float col_bias[4];
  load_col_bias<Cfg>(p, bc.n0 + wn0, lane, col_bias);

  // ---- steps 2 + 3: double-buffered main loop --------------------------------------------------
  const int KT = (bc.k_len + BK - 1) / BK;
  const int KT_full = bc.k_len / BK;  // tiles that lie entirely inside the K range
  u32x4 ra[OpA::NL], rb[OpB::NL];
  opa.init(tid, p.g);
  opb.init(tid, p.g);

  auto fetch = [&](int kt) {  // global -> registers
    if (kt < KT_full) {
      opa.load_full(ra, tid, kt * BK, p.g);
      opb.load_full(rb, tid, kt * BK, p.g);
    } else {
      opa.load_edge(ra, tid, kt * BK, p.g);
      opb.load_edge(rb, tid, kt * BK, p.g);
    }
  };
  auto commit = [&](unsigned char* stage) {  // registers -> LDS
    opa.store(ra, tid, stage);
    opb.store(rb, tid, stage + Cfg::A_BYTES);
  };
  typename OpA::Frag fa[2][FM];
  typename OpB::Frag fb[2][FN];
  auto load_frags = [&](int buf, const unsigned char* stage, int ks) {
#pragma unroll
    for (int i = 0; i < FM; ++i) fa[buf][i] = opa.fragment(stage, lane, wm0, i, ks);
#pragma unroll
    for (int j = 0; j < FN; ++j) fb[buf][j] = opb.fragment(stage + Cfg::A_BYTES, lane, wn0, j, ks);
  };
  auto mfmas = [&](int buf) {
    // operands swapped on purpose: the accumulator tile then holds C transposed (see epilogue)
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j) acc[i][j] = mfma_op(fb[buf][j], fa[buf][i], acc[i][j]);
  };

  // One iteration of the K loop.  `next`: 1 = tile kt+1 lies entirely inside K (predicate-free loads),
  // 2 = it is the last, partial tile, 0 = there is none.
  //   top        global loads of tile kt+1 -> registers
  //   ks < KS-1  LDS reads of k step ks+1, MFMAs of k step ks; during k step KS-2 the registers of
  //              tile kt+1 are written to the other LDS buffer
  //   barrier    every wave has written its share of tile kt+1 and has read all of tile kt
  //   ks = KS-1  LDS reads of k step 0 of tile kt+1, MFMAs of the last k step of tile kt
  // On entry frag[0] holds k step 0 of tile kt.  (With an odd number of k steps the fragment
  // buffers cannot alternate across tiles; that case runs the plain load-then-multiply order.)
  auto iteration = [&](int kt, auto next) {
    unsigned char* cur = smem + (kt & 1) * Cfg::STAGE_BYTES;
    unsigned char* nxt = smem + ((kt + 1) & 1) * Cfg::STAGE_BYTES;
    if constexpr (next.value == 1) {
      opa.load_full(ra, tid, (kt + 1) * BK, p.g);
      opb.load_full(rb, tid, (kt + 1) * BK, p.g);
    } else if constexpr (next.value == 2) {
      opa.load_edge(ra, tid, (kt + 1) * BK, p.g);
      opb.load_edge(rb, tid, (kt + 1) * BK, p.g);
    }
    // keep the global loads where they are written: issued before the MFMAs, so that their latency
    // overlaps the contraction instead of being paid right before the LDS stores
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (KS % 2 == 0) {
#pragma unroll
      for (int ks = 0; ks + 1 < KS; ++ks) {
        load_frags((ks + 1) & 1, cur, ks + 1);
        if constexpr (next.value != 0) {
          if (ks == KS - 2) commit(nxt);
        }
        mfmas(ks & 1);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (next.value != 0) {
        __syncthreads();
        load_frags(0, nxt, 0);
      }
      mfmas((KS - 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
    } else {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        load_frags(0, cur, ks);
        mfmas(0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (next.value != 0) {
        commit(nxt);
        __syncthreads();
      }
    }
  };

  if (KT > 0) {
    fetch(0);
    commit(smem);
    __syncthreads();
    if constexpr (KS % 2 == 0) load_frags(0, smem, 0);
    int kt = 0;
    for (; kt + 1 < KT_full; ++kt) iteration(kt, std::integral_constant<int, 1>{});
    if (kt + 1 < KT) {
      iteration(kt, std::integral_constant<int, 2>{});
      ++kt;
    }
    iteration(kt, std::integral_constant<int, 0>{});
    __syncthreads();  // the epilogue reuses the LDS
  }

  epilogue<Cfg>(p, bc, wave, lane, wm0, wn0, acc, col_bias, smem);
}

// ---------------------------------------------------------------------------------------------
// The kernel, large-tile schedule: 8 waves (2 per SIMD), vector mode only.
//
// K is consumed in stages of BK; LDS holds a ring of 4 stages.  Stage s+3 is requested with direct
// global -> LDS loads while stage s is being multiplied, so a load has two full stages to land.
// The two waves of a SIMD run half a stage apart: in every phase one of them issues nothing but
// MFMAs (at raised priority) while the other issues the LDS reads of its next fragments and the
// global loads -- the LDS pipe and the matrix cores are busy at the same time instead of taking
// turns.  Phases are separated by bare s_barrier instructions; what must be complete before a
// barrier is waited for explicitly:
//   * the wave's own LDS reads of stage s (its buffer is overwritten by loads issued right after
//     the barrier by the other wave group),
//   * the wave's own direct loads of stage s+1 (read by the other wave group right after).
// The second wave group enters the loop one barrier late and leaves it one barrier early.
// A last partial stage (K not a multiple of BK) is staged through registers with zero fill after the
// ring has drained.
// ---------------------------------------------------------------------------------------------
template <class Cfg>
__global__ void __launch_bounds__(Cfg::NT) gemm_kernel_pingpong(const GemmParams p) {
  using T = typename Cfg::T;
  using Acc = typename AccT<Cfg::MI>::type;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, MI = Cfg::MI, NT = Cfg::NT;
  constexpr int FM = Cfg::FM, FN = Cfg::FN, KS = Cfg::KS;
  static_assert(Cfg::NWAVES == 8 && !Cfg::IS_F32 && Cfg::MODE_A == LD_VEC && Cfg::MODE_B == LD_VEC && Cfg::STAGES == 4,
                "ping-pong schedule: 8 waves, 16-bit vector mode, 4 LDS stages");
  using OpA = Operand<T, BM, BK, Cfg::LA, LD_VEC, NT, MI>;
  using OpB = Operand<T, BN, BK, Cfg::LB, LD_VEC, NT, MI>;
  constexpr int LOADS = OpA::NL + OpB::NL;  // direct loads per thread per stage

  __shared__ __attribute__((aligned(16))) unsigned char smem[Cfg::LDS_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid % 64;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int grp = wave / 4;  // waves w and w+4 share a SIMD

  const BlockCoords bc = block_coords<BM, BN>(p);
  OpA opa;
  OpB opb;
  setup_operands<Cfg>(p, bc, opa, opb);
  const tmap::Task wt = tmap::Spatial<Cfg::WAVES_M, Cfg::WAVES_N>::task(wave, 0);
  const int wm0 = wt.i * Cfg::WTM, wn0 = wt.j * Cfg::WTN;

  Acc acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < (int)(sizeof(Acc) / 4); ++r) acc[i][j][r] = 0.0f;

  float col_bias[4];
  load_col_bias<Cfg>(p, bc.n0 + wn0, lane, col_bias);
  __builtin_amdgcn_s_waitcnt(0);  // nothing outstanding before the hand-counted loads begin

  typename OpA::Frag fa[KS][FM];
  typename OpB::Frag fb[KS][FN];
  auto load_frags = [&](const unsigned char* stage) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int i = 0; i < FM; ++i) fa[ks][i] = opa.fragment(stage, lane, wm0, i, ks);
#pragma unroll
      for (int j = 0; j < FN; ++j) fb[ks][j] = opb.fragment(stage + Cfg::A_BYTES, lane, wn0, j, ks);
    }
  };
  auto mfmas = [&]() {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma_op(fb[ks][j], fa[ks][i], acc[i][j]);
  };
  auto phase_barrier = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  const unsigned smem_lds = (unsigned)(size_t)(__attribute__((address_space(3))) void*)smem;
  auto request = [&](int s) {  // direct loads of stage s into ring slot s % 4
    const unsigned slot = smem_lds + (unsigned)((s & 3) * Cfg::STAGE_BYTES);
    opa.load_direct(slot, wave, s * BK);
    opb.load_direct(slot + Cfg::A_BYTES, wave, s * BK);
  };
  // wait until at most `younger` stages of this wave's direct loads are still in flight, and all LDS reads are back
  auto wait_stage = [&](int younger) {
    if (younger >= 2)
      __builtin_amdgcn_s_waitcnt(0x0070 | ((2 * LOADS) & 15) | (((2 * LOADS) >> 4) << 14));
    else if (younger == 1)
      __builtin_amdgcn_s_waitcnt(0x0070 | (LOADS & 15) | ((LOADS >> 4) << 14));
    else
      __builtin_amdgcn_s_waitcnt(0x0070);
  };

  const int S = bc.k_len / BK;  // full stages
  if (S > 0) {
    opa.init_direct(tid);
    opb.init_direct(tid);
    const int pre = S < 3 ? S : 3;
    for (int s = 0; s < pre; ++s) request(s);
    wait_stage(pre - 1);
    phase_barrier();
    if (grp == 1) phase_barrier();
    for (int s = 0; s < S; ++s) {
      // ---- memory phase
      load_frags(smem + (s & 3) * Cfg::STAGE_BYTES);
      if (s + 3 < S) request(s + 3);
      wait_stage((s + 2 < S) + (s + 3 < S));
      phase_barrier();
      // ---- compute phase
      __builtin_amdgcn_s_setprio(1);
      mfmas();
      __builtin_amdgcn_s_setprio(0);
      phase_barrier();
    }
    if (grp == 0) phase_barrier();
  }
  if (S * BK < bc.k_len) {  // the partial last stage, through registers with zero fill
    u32x4 ra[OpA::NL], rb[OpB::NL];
    opa.init(tid, p.g);
    opb.init(tid, p.g);
    opa.load_edge(ra, tid, S * BK, p.g);
    opb.load_edge(rb, tid, S * BK, p.g);
    __syncthreads();
    opa.store(ra, tid, smem);
    opb.store(rb, tid, smem + Cfg::A_BYTES);
    __syncthreads();
    load_frags(smem);
    mfmas();
  }
  __syncthreads();  // the epilogue reuses the LDS

  epilogue<Cfg, Acc, false>(p, bc, wave, lane, wm0, wn0, acc, col_bias, smem);
}

// ---------------------------------------------------------------------------------------------
// Parallel reduction on K, second pass (Sections 5.2 and 6.3.4: the matmul optimisation that lets
// batch-1 convolutions fill the GPU): sums the fp32 partial results of the k_slices workgroups of
// every output element and applies the fused epilogue.  p.A points at the workspace
// [batch][k_slices][M][N]; p.C, bias, residual and the index map are those of the real output.
// One thread per group of 4 consecutive columns.
// ---------------------------------------------------------------------------------------------
template <typename TO, int MAPPER>
__global__ void __launch_bounds__(256) splitk_reduce_kernel(const GemmParams p) {
  const int groups_per_row = (p.N + 3) / 4;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long long)p.M * groups_per_row) return;
  const int m = (int)(idx / groups_per_row);
  const int n = (int)(idx - (long long)m * groups_per_row) * 4;
  const int batch = blockIdx.y;
  const float* ws = reinterpret_cast<const float*>(p.A) + ((long long)batch * p.k_slices) * p.M * p.N + (long long)m * p.N + n;
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  const bool vec = (p.N % 4 == 0);
  const long long slice = (long long)p.M * p.N;
  // Eight slices are requested together (the loads do not depend on one another; out-of-range slices
  // re-read the last one) and then added in ascending order, so the result does not depend on the
  // unrolling while the memory latency is paid once per eight slices instead of once per slice.
  constexpr int U = 8;
  for (int z0 = 0; z0 < p.k_slices; z0 += U) {
    float v[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int z = z0 + u < p.k_slices ? z0 + u : p.k_slices - 1;
      const float* src = ws + z * slice;
      if (vec) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(src);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[u][e] = t[e];
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[u][e] = src[n + e < p.N ? e : 0];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (z0 + u < p.k_slices) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += v[u][e];
      }
    }
  }
  float col_bias[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  const TO* bias = reinterpret_cast<const TO*>(p.bias);
  if (p.bias_axis == 1) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (n + e < p.N) col_bias[e] = to_f32(bias[n + e]);
  }
  TO* C = reinterpret_cast<TO*>(p.C) + (long long)batch * p.strideC;
  const TO* R = p.residual ? reinterpret_cast<const TO*>(p.residual) + (long long)batch * p.strideR : nullptr;
  store4<TO, MAPPER>(p, C, R, bias, col_bias, m, n, col_offset<MAPPER>(p, n), group_valid<MAPPER>(p, n), acc);
}

}  // namespace hidet
