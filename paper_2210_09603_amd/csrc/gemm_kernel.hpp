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

#include "epilogue.hpp"

namespace hidet {

// ---------------------------------------------------------------------------------------------
// The kernel, general schedule: two LDS stages, next tile staged through registers (the double
// buffering of Section 3.1), fragments double-buffered in registers so that LDS reads of k step
// ks+1 run under the MFMAs of k step ks.  Handles every load mode and every edge.  Two orders of
// the same steps: SCHED_SIMPLE issues the loads of the next tile at the top of an iteration,
// SCHED_AHEAD one iteration earlier.
// ---------------------------------------------------------------------------------------------
template <class Cfg>
__global__ void __launch_bounds__(Cfg::NT) gemm_kernel(const GemmParams p) {
  using T = typename Cfg::T;
  using Acc = typename AccT<Cfg::MI>::type;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, MI = Cfg::MI, NT = Cfg::NT;
  constexpr int FM = Cfg::FM, FN = Cfg::FN;
  // k steps of a tile that this wavefront multiplies.  An fp32 MFMA covers only 2 or 4 values of k with one float per
  // lane and operand, so fp32 fragments are read (and multiplied) G MFMAs at a time: a k step of the loop below is
  // then G matrix-core k extents, and one LDS round trip feeds G times the matrix-core work.
  constexpr int KS_MFMA = Cfg::KS / Cfg::WAVES_K;
  // (Wave tiles of four or more MFMA tiles have enough matrix-core work per k extent to cover the round trip.)
  constexpr int G = (!Cfg::IS_F32 || FM * FN > 2) ? 1 : (KS_MFMA % 4 == 0) ? 4 : (KS_MFMA % 2 == 0) ? 2 : 1;
  constexpr int KS = KS_MFMA / G;
  using OpA = Operand<T, BM, BK, Cfg::LA, Cfg::MODE_A, NT, MI>;
  using OpB = Operand<T, BN, BK, Cfg::LB, Cfg::MODE_B, NT, MI>;

  __shared__ __attribute__((aligned(16))) unsigned char smem[Cfg::LDS_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid % 64;
  const int wave = tid / 64;
  const int kg = wave / Cfg::NWAVES_MN;   // wave group along K (always 0 unless SCHED_KSPLIT)
  const int wsp = wave % Cfg::NWAVES_MN;  // position in the spatial(WAVES_M, WAVES_N) mapping
  const int ks0 = kg * KS;                // first k step of every tile that this wavefront multiplies

  const BlockCoords bc = block_coords<BM, BN>(p);  // step 1
  OpA opa;
  OpB opb;
  setup_operands<Cfg>(p, bc, opa, opb);

  // step 4 (set-up): wave-level task mapping spatial(WAVES_M, WAVES_N) o repeat(FM, FN)
  const tmap::Task wt = tmap::Spatial<Cfg::WAVES_M, Cfg::WAVES_N>::task(wsp, 0);
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
  if constexpr (Cfg::GATHER_B) {
    opb.fill_masks(tid, smem + Cfg::STAGES * Cfg::STAGE_BYTES);
    __syncthreads();
  }

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
    opa.store(ra, tid, stage, p.relu_a != 0);
    opb.store(rb, tid, stage + Cfg::A_BYTES, p.relu_b != 0);
  };
  typename OpA::Frag fa[2][G][FM];
  typename OpB::Frag fb[2][G][FN];
  auto load_frags = [&](int buf, const unsigned char* stage, int ks) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int i = 0; i < FM; ++i) fa[buf][g][i] = opa.fragment(stage, lane, wm0, i, (ks0 + ks) * G + g);
#pragma unroll
      for (int j = 0; j < FN; ++j) fb[buf][g][j] = opb.fragment(stage + Cfg::A_BYTES, lane, wn0, j, (ks0 + ks) * G + g);
    }
  };
  auto mfmas = [&](int buf) {
    // operands swapped on purpose: the accumulator tile then holds C transposed (see epilogue)
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) acc[i][j] = mfma_op(fb[buf][g][j], fa[buf][g][i], acc[i][j]);
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

  // The same iteration with the loads one step further ahead (SCHED_AHEAD).  On entry the global loads of tile
  // kt+1 (if there is one) are already in flight towards the staging registers: they were issued during the
  // previous iteration, right after tile kt had been written to LDS and the registers were free again, and so
  // have a whole iteration to arrive instead of the first k steps of one.  The staging registers stay occupied
  // all the time, which is why this is a schedule of its own: it pays where an iteration is short (small tiles,
  // latency-bound problems) and costs occupancy where the tile is large.
  // `has_next`: there is a tile kt+1.  `ahead`: 1 = tile kt+2 lies entirely inside K (predicate-free loads),
  // 2 = decide at run time whether there is a tile kt+2 and whether it is the partial one, 0 = there is none.
  auto iteration_ahead = [&](int kt, auto has_next, auto ahead) {
    unsigned char* cur = smem + (kt & 1) * Cfg::STAGE_BYTES;
    unsigned char* nxt = smem + ((kt + 1) & 1) * Cfg::STAGE_BYTES;
    auto stage_next = [&]() {
      commit(nxt);
      if constexpr (ahead.value == 1) {
        opa.load_full(ra, tid, (kt + 2) * BK, p.g);
        opb.load_full(rb, tid, (kt + 2) * BK, p.g);
      } else if constexpr (ahead.value == 2) {
        if (kt + 2 < KT) fetch(kt + 2);
      }
    };
    if constexpr (KS % 2 == 0) {
#pragma unroll
      for (int ks = 0; ks + 1 < KS; ++ks) {
        load_frags((ks + 1) & 1, cur, ks + 1);
        if constexpr (has_next.value != 0) {
          if (ks == KS - 2) stage_next();
        }
        mfmas(ks & 1);
        __builtin_amdgcn_sched_barrier(0);
      }
      if constexpr (has_next.value != 0) {
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
      if constexpr (has_next.value != 0) {
        stage_next();
        __syncthreads();
      }
    }
  };

  if (KT > 0) {
    using std::integral_constant;
    fetch(0);
    commit(smem);
    if constexpr (Cfg::SCHED == SCHED_AHEAD || Cfg::SCHED == SCHED_KSPLIT) {
      if (KT > 1) fetch(1);
    }
    __syncthreads();
    if constexpr (KS % 2 == 0) load_frags(0, smem, 0);
    int kt = 0;
    if constexpr (Cfg::SCHED == SCHED_AHEAD || Cfg::SCHED == SCHED_KSPLIT) {
      for (; kt + 2 < KT_full; ++kt) iteration_ahead(kt, integral_constant<int, 1>{}, integral_constant<int, 1>{});
      for (; kt + 1 < KT; ++kt) iteration_ahead(kt, integral_constant<int, 1>{}, integral_constant<int, 2>{});
      iteration_ahead(kt, integral_constant<int, 0>{}, integral_constant<int, 0>{});
    } else {
      for (; kt + 1 < KT_full; ++kt) iteration(kt, integral_constant<int, 1>{});
      if (kt + 1 < KT) {
        iteration(kt, integral_constant<int, 2>{});
        ++kt;
      }
      iteration(kt, integral_constant<int, 0>{});
    }
    __syncthreads();  // the epilogue reuses the LDS
  }

  if (!reduce_wave_groups<Cfg>(acc, smem, kg, wsp, lane)) return;  // (no workgroup barrier follows)
  epilogue<Cfg>(p, bc, wsp, lane, wm0, wn0, acc, col_bias, smem);
}

// ---------------------------------------------------------------------------------------------
// The kernel, large-tile schedule: 8 waves (2 per SIMD), plain 16-bit operands.
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
// Operands whose rows are only element aligned (odd leading dimensions, offset pointers -- the sizes on
// which input-centric schedule spaces have no schedule, Section 3.3) run the same schedule: the direct
// loads take any element-aligned address.  A direct load cannot be predicated, so there the LAST stage,
// whole or partial, always goes through registers: no 16-byte chunk of a direct load then touches the
// last row of a row-major operand, where reading past the last column would leave the allocation
// (on every other row it reads the beginning of the next one, into columns that are never stored).
// ---------------------------------------------------------------------------------------------
// SLOTS = 2 is the same kernel for a K range of at most two stages: nothing is ever requested into a slot that was
// used before, two slots of LDS are enough, and two such workgroups fit on a compute unit where the registers allow
// (the output write of one then overlaps the loads and the matrix-core work of the other).
template <class Cfg, int SLOTS = 4>
__global__ void __launch_bounds__(Cfg::NT) gemm_kernel_pingpong(const GemmParams p) {
  using T = typename Cfg::T;
  using Acc = typename AccT<Cfg::MI>::type;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, MI = Cfg::MI, NT = Cfg::NT;
  constexpr int FM = Cfg::FM, FN = Cfg::FN, KS = Cfg::KS;
  static_assert(Cfg::NWAVES == 8 && !Cfg::IS_F32 && Cfg::MODE_A == Cfg::MODE_B &&
                    (Cfg::MODE_A == LD_VEC || Cfg::MODE_A == LD_ELEM) && Cfg::STAGES == 4,
                "ping-pong schedule: 8 waves, 16-bit types, plain operands, 4 LDS stages");
  constexpr bool ELEM = Cfg::MODE_A == LD_ELEM;  // rows only element aligned
  using OpA = Operand<T, BM, BK, Cfg::LA, Cfg::MODE_A, NT, MI>;
  using OpB = Operand<T, BN, BK, Cfg::LB, Cfg::MODE_B, NT, MI>;
  constexpr int LOADS = OpA::NL + OpB::NL;  // direct loads per thread per stage

  static_assert(SLOTS == 4 || SLOTS == 2, "ring of four stages, or two stages without reuse");
  constexpr int RING_BYTES = SLOTS * Cfg::STAGE_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char smem[RING_BYTES > Cfg::EPI_BYTES ? RING_BYTES : Cfg::EPI_BYTES];

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
    const unsigned slot = smem_lds + (unsigned)((s & (SLOTS - 1)) * Cfg::STAGE_BYTES);
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

  // stages loaded directly: the full ones; all but the last one for element-aligned operands
  const int S = ELEM ? (bc.k_len > 0 ? (bc.k_len - 1) / BK : 0) : bc.k_len / BK;
  if (S > 0) {
    opa.init_direct(tid, ELEM);
    opb.init_direct(tid, ELEM);
    const int pre = S < 3 ? S : 3;
    for (int s = 0; s < pre; ++s) request(s);
    wait_stage(pre - 1);
    phase_barrier();
    if (grp == 1) phase_barrier();
    for (int s = 0; s < S; ++s) {
      // ---- memory phase
      load_frags(smem + (s & (SLOTS - 1)) * Cfg::STAGE_BYTES);
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
  if (S * BK < bc.k_len) {  // the last stage (partial, or any for element-aligned operands), through registers with zero fill
    u32x4 ra[OpA::NL], rb[OpB::NL];
    opa.init(tid, p.g);
    opb.init(tid, p.g);
    opa.load_edge(ra, tid, S * BK, p.g);
    opb.load_edge(rb, tid, S * BK, p.g);
    __syncthreads();
    opa.store(ra, tid, smem, p.relu_a != 0);
    opb.store(rb, tid, smem + Cfg::A_BYTES, p.relu_b != 0);
    __syncthreads();
    load_frags(smem);
    mfmas();
  }
  __syncthreads();  // the epilogue reuses the LDS

  epilogue<Cfg, Acc, false>(p, bc, wave, lane, wm0, wn0, acc, col_bias, smem);
}

// ---------------------------------------------------------------------------------------------
// The large-tile schedule with its stages staged through registers, for what a direct global -> LDS load
// cannot do: an input prologue applied to the operand as it is loaded, and the head-split output map
// (compiled out of the kernel above).  A stage is
// requested (16-byte loads at element alignment) during the memory phase of one iteration, written
// into its ring slot during the memory phase of the next, and multiplied one iteration after that.
// Phases, barriers and the half-stage offset between the two wavefronts of a SIMD are those of
// gemm_kernel_pingpong; the waits are the compiler's (no hand-counted loads), except that a wave's LDS
// writes and fragment reads must be complete before the barrier that ends its memory phase.
// ---------------------------------------------------------------------------------------------
template <class Cfg>
__global__ void __launch_bounds__(Cfg::NT) gemm_kernel_pingpong_regs(const GemmParams p) {
  using T = typename Cfg::T;
  using Acc = typename AccT<Cfg::MI>::type;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, MI = Cfg::MI, NT = Cfg::NT;
  constexpr int FM = Cfg::FM, FN = Cfg::FN, KS = Cfg::KS;
  static_assert(Cfg::NWAVES == 8 && !Cfg::IS_F32 && Cfg::MODE_A == LD_ELEM && Cfg::MODE_B == LD_ELEM && Cfg::STAGES == 4,
                "ping-pong schedule through registers: 8 waves, 16-bit element mode, 4 LDS stages");
  using OpA = Operand<T, BM, BK, Cfg::LA, LD_ELEM, NT, MI>;
  using OpB = Operand<T, BN, BK, Cfg::LB, LD_ELEM, NT, MI>;

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
  // all of this wave's LDS operations are complete (global loads may stay in flight)
  auto lds_done = [&]() { __builtin_amdgcn_s_waitcnt(0xc07f); };

  u32x4 ra[OpA::NL], rb[OpB::NL];
  opa.init(tid, p.g);
  opb.init(tid, p.g);
  auto request = [&](int s) {  // global -> registers
    opa.load_full(ra, tid, s * BK, p.g);
    opb.load_full(rb, tid, s * BK, p.g);
  };
  auto deposit = [&](int s) {  // registers -> ring slot s % 4
    unsigned char* slot = smem + (s & 3) * Cfg::STAGE_BYTES;
    opa.store(ra, tid, slot, p.relu_a != 0);
    opb.store(rb, tid, slot + Cfg::A_BYTES, p.relu_b != 0);
  };

  const int S = bc.k_len / BK;  // full stages
  if (S > 0) {
    request(0);
    deposit(0);
    if (S > 1) {
      request(1);
      deposit(1);
    }
    if (S > 2) request(2);
    lds_done();
    phase_barrier();
    if (grp == 1) phase_barrier();
    for (int s = 0; s < S; ++s) {
      // ---- memory phase: stage s+1 (requested one iteration ago) into its slot, fragments of stage s, request s+2
      if (s >= 1 && s + 1 < S) deposit(s + 1);
      load_frags(smem + (s & 3) * Cfg::STAGE_BYTES);
      if (s >= 1 && s + 2 < S) request(s + 2);
      lds_done();
      phase_barrier();
      // ---- compute phase
      __builtin_amdgcn_s_setprio(1);
      mfmas();
      __builtin_amdgcn_s_setprio(0);
      phase_barrier();
    }
    if (grp == 0) phase_barrier();
  }
  if (S * BK < bc.k_len) {  // the partial last stage, zero filled
    opa.load_edge(ra, tid, S * BK, p.g);
    opb.load_edge(rb, tid, S * BK, p.g);
    __syncthreads();
    opa.store(ra, tid, smem, p.relu_a != 0);
    opb.store(rb, tid, smem + Cfg::A_BYTES, p.relu_b != 0);
    __syncthreads();
    load_frags(smem);
    mfmas();
  }
  __syncthreads();  // the epilogue reuses the LDS

  epilogue<Cfg>(p, bc, wave, lane, wm0, wn0, acc, col_bias, smem);
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
