// Table of compiled kernels: [tile configuration][input type][variant] -> launcher.
#pragma once

#include <hip/hip_runtime.h>

#include "gemm_kernel.hpp"

namespace hidet {

using LaunchFn = hipError_t (*)(const GemmParams&, hipStream_t);

constexpr int kMaxConfigs = 64;
constexpr int kNumTypes = 3;     // index = hidet_dtype_t of the inputs: 0 f32, 1 f16, 2 bf16 (output has the same type)
constexpr int kNumVariants = 22; // GEMM: transA*4 + transB*2 + mode (0 vector loads, 1 element loads); conv: 8 + mode;
                                 // +10: the same operand forms writing raw fp32 partial sums to a plain [M][N]
                                 // workspace (first pass of the parallel reduction on K);
                                 // 20, 21: convolution with repacked (tap-major) weights, and its partial-sum form

struct ConfigRow {
  int index, bm, bn, bk, waves_m, waves_n, mfma, trans_a, sched, is_f32;
};

struct Registry {
  LaunchFn fn[kMaxConfigs][kNumTypes][kNumVariants];
};

inline int gemm_variant(int transA, int transB, int elem_mode) { return (transA ? 4 : 0) + (transB ? 2 : 0) + (elem_mode ? 1 : 0); }
inline int conv_variant(int elem_mode) { return 8 + (elem_mode ? 1 : 0); }
constexpr int kPartialVariants = 10;  // offset of the K-parallel partial-sum kernels
constexpr int kConvTapVariant = 20;   // convolution over the tap-major K order (repacked weights); +1: partial sums

template <class Cfg>
hipError_t launch_kernel(const GemmParams& p, hipStream_t stream) {
  // the element-mode variant of a ring tile also serves what the direct loads cannot do (input prologue, head-split
  // output map), with its stages staged through registers
  if (Cfg::SCHED == SCHED_PINGPONG && Cfg::MODE_A == LD_ELEM && (p.out_map != 0 || p.relu_a != 0 || p.relu_b != 0)) {
    if constexpr (Cfg::SCHED == SCHED_PINGPONG && Cfg::MODE_A == LD_ELEM)
      hipLaunchKernelGGL(gemm_kernel_pingpong_regs<Cfg>, dim3((unsigned)p.total_blocks), dim3(Cfg::NT), 0, stream, p);
  } else if constexpr (Cfg::SCHED == SCHED_PINGPONG) {
    // a K range of at most two stages never reuses a ring slot: the two-slot form leaves LDS for a second workgroup
    const int k_len = p.k_slices > 1 ? p.k_slice_len : p.K;
    if (k_len <= 2 * Cfg::BK)
      hipLaunchKernelGGL((gemm_kernel_pingpong<Cfg, 2>), dim3((unsigned)p.total_blocks), dim3(Cfg::NT), 0, stream, p);
    else
      hipLaunchKernelGGL((gemm_kernel_pingpong<Cfg, 4>), dim3((unsigned)p.total_blocks), dim3(Cfg::NT), 0, stream, p);
  } else
    hipLaunchKernelGGL(gemm_kernel<Cfg>, dim3((unsigned)p.total_blocks), dim3(Cfg::NT), 0, stream, p);
  return hipGetLastError();
}

// Fills the launchers of one (configuration, input type) pair.
template <typename T, int BM, int BN, int BK, int WM, int WN, int MI, int TRANS_A, int SCHED>
void register_config(Registry& r, int index, int type_index) {
  LaunchFn* v = r.fn[index][type_index];
  // the operand forms that the ring schedule does not cover run the general kernel on the same tile
  constexpr int GS = (SCHED == SCHED_PINGPONG) ? SCHED_SIMPLE : SCHED;
  // row-major A: KC;  row-major B: MC;  transposed B: KC;  transposed A: MC
  v[gemm_variant(0, 0, 0)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_VEC, LD_VEC, MAP_PLAIN, SCHED>>;
  v[gemm_variant(0, 0, 1)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_ELEM, LD_ELEM, MAP_PLAIN, SCHED>>;
  v[gemm_variant(0, 1, 0)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_KC, L_KC, LD_VEC, LD_VEC, MAP_PLAIN, SCHED>>;
  v[gemm_variant(0, 1, 1)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_KC, L_KC, LD_ELEM, LD_ELEM, MAP_PLAIN, SCHED>>;
  if constexpr (TRANS_A != 0) {
    v[gemm_variant(1, 0, 0)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_MC, L_MC, LD_VEC, LD_VEC, MAP_PLAIN, SCHED>>;
    v[gemm_variant(1, 0, 1)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_MC, L_MC, LD_ELEM, LD_ELEM, MAP_PLAIN, SCHED>>;
    v[gemm_variant(1, 1, 0)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_MC, L_KC, LD_VEC, LD_VEC, MAP_PLAIN, SCHED>>;
    v[gemm_variant(1, 1, 1)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_MC, L_KC, LD_ELEM, LD_ELEM, MAP_PLAIN, SCHED>>;
  }
  // convolution: weights are a row-major OC x (IC*KH*KW) matrix, B is the img2col gather, C is NCHW
  v[conv_variant(0)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_VEC, LD_IM2COL, MAP_NCHW, GS>>;
  v[conv_variant(1)] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_ELEM, LD_IM2COL, MAP_NCHW, GS>>;
  v[kConvTapVariant] = launch_kernel<GemmConfig<T, T, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_VEC, LD_IM2COL_TAP, MAP_NCHW, GS>>;
  // K-parallel partial sums (fp32 out, plain map): built for the small and medium tiles, which are the ones a
  // problem with few output tiles and a long K wants, and for the ring-schedule tiles (medium-sized problems whose
  // tiles do not fill the device)
  if constexpr (BM * BN <= 128 * 128 || SCHED == SCHED_PINGPONG) {
    LaunchFn* w = v + kPartialVariants;
    w[gemm_variant(0, 0, 0)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_VEC, LD_VEC, MAP_PLAIN, SCHED>>;
    w[gemm_variant(0, 0, 1)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_ELEM, LD_ELEM, MAP_PLAIN, SCHED>>;
    w[gemm_variant(0, 1, 0)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_KC, L_KC, LD_VEC, LD_VEC, MAP_PLAIN, SCHED>>;
    w[gemm_variant(0, 1, 1)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_KC, L_KC, LD_ELEM, LD_ELEM, MAP_PLAIN, SCHED>>;
    if constexpr (TRANS_A != 0) {
      w[gemm_variant(1, 0, 0)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_MC, L_MC, LD_VEC, LD_VEC, MAP_PLAIN, SCHED>>;
      w[gemm_variant(1, 0, 1)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_MC, L_MC, LD_ELEM, LD_ELEM, MAP_PLAIN, SCHED>>;
      w[gemm_variant(1, 1, 0)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_MC, L_KC, LD_VEC, LD_VEC, MAP_PLAIN, SCHED>>;
      w[gemm_variant(1, 1, 1)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_MC, L_KC, LD_ELEM, LD_ELEM, MAP_PLAIN, SCHED>>;
    }
    w[conv_variant(0)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_VEC, LD_IM2COL, MAP_PLAIN, GS>>;
    w[conv_variant(1)] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_ELEM, LD_IM2COL, MAP_PLAIN, GS>>;
    v[kConvTapVariant + 1] = launch_kernel<GemmConfig<T, float, BM, BN, BK, WM, WN, MI, L_KC, L_MC, LD_VEC, LD_IM2COL_TAP, MAP_PLAIN, GS>>;
  }
}

// Second pass of the parallel reduction on K: [output type index][0 plain map, 1 NCHW map].
template <typename TO, int MAPPER>
hipError_t launch_reduce(const GemmParams& p, int batch, hipStream_t stream) {
  const long long groups = (long long)p.M * ((p.N + 3) / 4);
  hipLaunchKernelGGL((splitk_reduce_kernel<TO, MAPPER>), dim3((unsigned)((groups + 255) / 256), (unsigned)batch), dim3(256), 0,
                     stream, p);
  return hipGetLastError();
}

}  // namespace hidet
