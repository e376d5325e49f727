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

struct ConvGeom {
  int IC, H, W, KH, KW, sh, sw, ph, pw, OH, OW;
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
  int vec_store;  // 1: groups of 4 consecutive output columns may use one vector access
  int tiles_m, tiles_n, group;
  int total_blocks;
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
// ---------------------------------------------------------------------------------------------
template <int CPR>
__device__ __forceinline__ constexpr int swz_kc(int row) {
  if constexpr (CPR >= 16) return row & 15;
  if constexpr (CPR == 8) return (row & 7) ^ ((row >> 3) & 1);
  if constexpr (CPR == 4) return ((row >> 1) & 3) ^ ((row >> 3) & 1);
  return 0;
}
template <int CPR>
__device__ __forceinline__ constexpr int swz_mc(int k) {
  if constexpr (CPR >= 16) {
    const int t = k & 3;
    return t == 0 ? 0 : (t == 1 ? 6 : (t == 2 ? 10 : 12));
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
          int MODE_A_, int MODE_B_, int MAPPER_>
struct GemmConfig {
  using T = T_;
  using TO = TO_;
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, MI = MI_;
  static constexpr int LA = LA_, LB = LB_, MODE_A = MODE_A_, MODE_B = MODE_B_, MAPPER = MAPPER_;
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
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
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
  int K;
  int r0;            // global row/column of the panel origin (needed by the img2col gather)

  // ---- global -> registers ------------------------------------------------------------------
  __device__ __forceinline__ u32x4 gather(int sr, int sc, int k0, const ConvGeom& g) const {
    // element-by-element, zero-filled: any alignment, any edge
    T tmp[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) tmp[e] = (T)0.0f;
    if constexpr (MODE == LD_IM2COL) {
      // stored row sr = k index (ic, kh, kw), columns sc.. = output positions p (n, oh, ow)
      const int k = k0 + sr;
      if (k < K) {
        const int khw = g.KH * g.KW;
        const int ic = k / khw, rem = k - ic * khw;
        const int kh = rem / g.KW, kw = rem - kh * g.KW;
        const int ohw = g.OH * g.OW;
        int p = r0 + sc;
        int n = p / ohw;
        int q = p - n * ohw;
        int oh = q / g.OW, ow = q - oh * g.OW;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          if (sc + e < rows_left) {
            const int ih = oh * g.sh + kh - g.ph, iw = ow * g.sw + kw - g.pw;
            if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W)
              tmp[e] = src[(((long long)n * g.IC + ic) * g.H + ih) * g.W + iw];
          }
          if (++ow == g.OW) {
            ow = 0;
            if (++oh == g.OH) {
              oh = 0;
              ++n;
            }
          }
        }
      }
    } else if constexpr (LAYOUT == L_KC) {
      if (sr < rows_left) {
        const T* ptr = src + (long long)sr * ld + (k0 + sc);
#pragma unroll
        for (int e = 0; e < VEC; ++e)
          if (k0 + sc + e < K) tmp[e] = ptr[e];
      }
    } else {
      if (k0 + sr < K) {
        const T* ptr = src + (long long)(k0 + sr) * ld + sc;
#pragma unroll
        for (int e = 0; e < VEC; ++e)
          if (sc + e < rows_left) tmp[e] = ptr[e];
      }
    }
    return __builtin_bit_cast(u32x4, tmp);
  }

  __device__ __forceinline__ void load(u32x4 (&regs)[NL], int tid, int k0, const ConvGeom& g) const {
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const tmap::Task t = LoadMap::task(tid, q);
      const int sr = t.i, sc = t.j * VEC;  // stored row, first stored column of the chunk
      if constexpr (MODE == LD_VEC) {
        bool full;
        const T* ptr;
        if constexpr (LAYOUT == L_KC) {
          full = (sr < rows_left) && (k0 + sc + VEC <= K);
          ptr = src + (long long)sr * ld + (k0 + sc);
        } else {
          full = (k0 + sr < K) && (sc + VEC <= rows_left);
          ptr = src + (long long)(k0 + sr) * ld + sc;
        }
        if (full)
          regs[q] = *reinterpret_cast<const u32x4*>(ptr);
        else
          regs[q] = gather(sr, sc, k0, g);
      } else {
        regs[q] = gather(sr, sc, k0, g);
      }
    }
  }

  // ---- registers -> LDS ---------------------------------------------------------------------
  __device__ __forceinline__ void store(const u32x4 (&regs)[NL], int tid, unsigned char* tile) const {
#pragma unroll
    for (int q = 0; q < NL; ++q) {
      const tmap::Task t = LoadMap::task(tid, q);
      if constexpr (!IS_F32) {
        const int swz = (LAYOUT == L_KC) ? swz_kc<CPR>(t.i) : swz_mc<CPR>(t.i);
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
      const u32x4 v = *reinterpret_cast<const u32x4*>(tile + (r * CPR + (c ^ swz_kc<CPR>(r))) * 16);
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
        const unsigned char* addr = tile + (kk * CPR + ((col / 8) ^ swz_mc<CPR>(kk))) * 16 + (col % 8) * 2;
        const i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) i16x4*)(const_cast<unsigned char*>(addr)));
        h[i] = __builtin_bit_cast(u32x2, v);
      }
      const u32x4 v = {h[0][0], h[0][1], h[1][0], h[1][1]};
      return __builtin_bit_cast(Frag, v);
    }
  }
};

// ---------------------------------------------------------------------------------------------
// Fused epilogue + predicated store of 4 consecutive output columns of one row.
// ---------------------------------------------------------------------------------------------
template <typename TO, int MAPPER>
__device__ __forceinline__ void store4(const GemmParams& p, TO* __restrict__ C, const TO* __restrict__ R,
                                       const TO* __restrict__ bias, int m, int n, const float (&acc)[4]) {
  if (m >= p.M || n >= p.N) return;
  long long off, roff;
  if constexpr (MAPPER == MAP_PLAIN) {
    off = (long long)m * p.ldc + n;
    roff = (long long)m * p.ldr + n;
  } else {
    const long long img = n / p.out_inner;
    off = img * p.out_outer + (long long)m * p.out_inner + (n - img * p.out_inner);
    roff = off;
  }
  float v[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = p.alpha * acc[e];
  const bool whole = p.vec_store && (n + 3 < p.N);
  if (p.bias_axis == 2) {
    const float b = to_f32(bias[m]);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += b;
  } else if (p.bias_axis == 1) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (n + e < p.N) v[e] += to_f32(bias[n + e]);
  }
  if (R != nullptr) {
    if (whole) {
      TO r[4];
      if constexpr (sizeof(TO) == 2)
        *reinterpret_cast<u32x2*>(r) = *reinterpret_cast<const u32x2*>(R + roff);
      else
        *reinterpret_cast<u32x4*>(r) = *reinterpret_cast<const u32x4*>(R + roff);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += to_f32(r[e]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (n + e < p.N) {
          long long ro = roff + e;
          if constexpr (MAPPER == MAP_NCHW) {
            const long long img = (n + e) / p.out_inner;
            ro = img * p.out_outer + (long long)m * p.out_inner + ((n + e) - img * p.out_inner);
          }
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
    if constexpr (sizeof(TO) == 2)
      *reinterpret_cast<u32x2*>(C + off) = *reinterpret_cast<const u32x2*>(o);
    else
      *reinterpret_cast<u32x4*>(C + off) = *reinterpret_cast<const u32x4*>(o);
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (n + e < p.N) {
        long long oo = off + e;
        if constexpr (MAPPER == MAP_NCHW) {
          const long long img = (n + e) / p.out_inner;
          oo = img * p.out_outer + (long long)m * p.out_inner + ((n + e) - img * p.out_inner);
        }
        C[oo] = o[e];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// The kernel.
// ---------------------------------------------------------------------------------------------
template <class Cfg>
__global__ void __launch_bounds__(Cfg::NT) gemm_kernel(const GemmParams p) {
  using T = typename Cfg::T;
  using TO = typename Cfg::TO;
  using Acc = typename AccT<Cfg::MI>::type;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, MI = Cfg::MI, NT = Cfg::NT;
  constexpr int FM = Cfg::FM, FN = Cfg::FN, KS = Cfg::KS;
  using OpA = Operand<T, BM, BK, Cfg::LA, Cfg::MODE_A, NT, MI>;
  using OpB = Operand<T, BN, BK, Cfg::LB, Cfg::MODE_B, NT, MI>;

  __shared__ __attribute__((aligned(16))) unsigned char smem[Cfg::LDS_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid % 64;
  const int wave = tid / 64;

  // ---- step 1: block-level task mapping ------------------------------------------------------
  // Workgroups are handed to the 8 accelerator dies (XCDs) round-robin; renumber them so that each
  // die, which has a private L2, works on one contiguous run of tiles of the grouped traversal.
  const int total = p.total_blocks;
  const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
  const int per = total / 8, extra = total % 8;
  const int logical = xcd * per + (xcd < extra ? xcd : extra) + slot;
  const int tiles = p.tiles_m * p.tiles_n;
  const int batch = logical / tiles;
  const tmap::Task tile = tmap::GroupedSpatial{p.tiles_m, p.tiles_n, p.group}.task(logical - batch * tiles);
  const int m0 = tile.i * BM, n0 = tile.j * BN;

  OpA opa;
  OpB opb;
  {
    const T* A = reinterpret_cast<const T*>(p.A) + (long long)batch * p.strideA;
    const T* B = reinterpret_cast<const T*>(p.B) + (long long)batch * p.strideB;
    opa.src = (Cfg::LA == L_KC) ? A + (long long)m0 * p.lda : A + m0;
    opa.ld = p.lda;
    opa.rows_left = p.M - m0;
    opa.K = p.K;
    opa.r0 = m0;
    if constexpr (Cfg::MODE_B == LD_IM2COL)
      opb.src = B;  // the gather addresses the whole input tensor
    else
      opb.src = (Cfg::LB == L_KC) ? B + (long long)n0 * p.ldb : B + n0;
    opb.ld = p.ldb;
    opb.rows_left = p.N - n0;
    opb.K = p.K;
    opb.r0 = n0;
  }

  // ---- step 4 (set-up): wave-level task mapping spatial(WAVES_M, WAVES_N) o repeat(FM, FN) ------
  const tmap::Task wt = tmap::Spatial<Cfg::WAVES_M, Cfg::WAVES_N>::task(wave, 0);
  const int wm0 = wt.i * Cfg::WTM, wn0 = wt.j * Cfg::WTN;

  Acc acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int r = 0; r < (int)(sizeof(Acc) / 4); ++r) acc[i][j][r] = 0.0f;

  const int KT = (p.K + BK - 1) / BK;
  u32x4 ra[OpA::NL], rb[OpB::NL];

  // ---- steps 2 + 3: double-buffered main loop --------------------------------------------------
  if (KT > 0) {
    opa.load(ra, tid, 0, p.g);
    opb.load(rb, tid, 0, p.g);
    opa.store(ra, tid, smem);
    opb.store(rb, tid, smem + Cfg::A_BYTES);
    __syncthreads();
  }
  for (int kt = 0; kt < KT; ++kt) {
    unsigned char* cur = smem + (kt & 1) * Cfg::STAGE_BYTES;
    unsigned char* nxt = smem + ((kt + 1) & 1) * Cfg::STAGE_BYTES;
    const bool more = kt + 1 < KT;
    if (more) {  // next tile: global -> registers, in flight during the MFMAs below
      opa.load(ra, tid, (kt + 1) * BK, p.g);
      opb.load(rb, tid, (kt + 1) * BK, p.g);
    }
    const unsigned char* ta = cur;
    const unsigned char* tb = cur + Cfg::A_BYTES;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      typename OpA::Frag fa[FM];
      typename OpB::Frag fb[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) fa[i] = opa.fragment(ta, lane, wm0, i, ks);
#pragma unroll
      for (int j = 0; j < FN; ++j) fb[j] = opb.fragment(tb, lane, wn0, j, ks);
      // operands swapped on purpose: the accumulator tile then holds C transposed, so that each
      // lane owns 4 consecutive columns of one row of C and can store them with one access
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma_op(fb[j], fa[i], acc[i][j]);
    }
    if (more) {  // registers -> the other LDS buffer
      opa.store(ra, tid, nxt);
      opb.store(rb, tid, nxt + Cfg::A_BYTES);
    }
    __syncthreads();
  }

  // ---- step 5: fused epilogue + predicated store -----------------------------------------------
  TO* C = reinterpret_cast<TO*>(p.C) + (long long)batch * p.strideC;
  const TO* R = p.residual ? reinterpret_cast<const TO*>(p.residual) + (long long)batch * p.strideR : nullptr;
  const TO* bias = reinterpret_cast<const TO*>(p.bias);
  constexpr int GROUPS = (MI == 32) ? 4 : 1;  // groups of 4 consecutive columns per accumulator tile
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int gq = 0; gq < GROUPS; ++gq) {
      const int n = n0 + wn0 + j * MI + ((MI == 32) ? 8 * gq + 4 * (lane / 32) : 4 * (lane / 16));
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int m = m0 + wm0 + i * MI + lane % MI;
        const float v[4] = {acc[i][j][4 * gq + 0], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]};
        store4<TO, Cfg::MAPPER>(p, C, R, bias, m, n, v);
      }
    }
}

}  // namespace hidet
