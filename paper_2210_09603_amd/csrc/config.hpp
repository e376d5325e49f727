// Tile configurations (one entry of the hardware-centric schedule space as compile-time constants) and the
// cooperative-load task mappings of an operand tile.
#pragma once

#include "taskmap.hpp"
#include "types.hpp"

namespace hidet {

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
  // SCHED_KSPLIT: sixteen wavefronts, 16 / (WAVES_M x WAVES_N) groups of WAVES_M x WAVES_N that share every K tile,
  // each multiplying its share of the k steps; their partial sums meet in LDS before the epilogue
  static constexpr int NWAVES_MN = WAVES_M * WAVES_N;
  static constexpr int WAVES_K = (SCHED == SCHED_KSPLIT) ? 16 / NWAVES_MN : 1;
  static constexpr int NWAVES = NWAVES_MN * WAVES_K;
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
  static constexpr int EPI_BYTES = NWAVES_MN * MI * (WTN * 4 + 16);
  // partial accumulators of the wave groups 1 .. WAVES_K-1, behind the epilogue regions
  static constexpr int RED_BYTES = (WAVES_K - 1) * NWAVES_MN * 64 * (FM * FN * MI * MI / 64) * 4;
  // img2col gather: table of the 16-byte masks that keep elements [lo, hi) of a chunk, behind the stages
  static constexpr bool GATHER_B = MODE_B == LD_IM2COL || MODE_B == LD_IM2COL_TAP;
  static constexpr int MASK_BYTES = GATHER_B ? (VEC + 1) * (VEC + 1) * 16 : 0;
  static constexpr int MAIN_BYTES = STAGES * STAGE_BYTES + MASK_BYTES;
  static constexpr int LDS_BYTES = MAIN_BYTES > EPI_BYTES + RED_BYTES ? MAIN_BYTES : EPI_BYTES + RED_BYTES;
  static constexpr int NL_A = BM * BK / VEC / NT;  // chunks per thread per tile
  static constexpr int NL_B = BN * BK / VEC / NT;
  static_assert(BM % (WAVES_M * MI) == 0 && BN % (WAVES_N * MI) == 0, "wave tiles must be whole MFMA tiles");
  static_assert(BK % KSTEP == 0, "BK must be a multiple of the MFMA k extent");
  static_assert(KS % WAVES_K == 0, "the k steps of a tile must split evenly over the wave groups");
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

}  // namespace hidet
