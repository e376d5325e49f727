// Matrix-core ceiling probe: what the MFMA units of this GPU sustain, at the clock the power
// management grants for the given operand values, when nothing else (LDS, memory, barriers)
// stands in the way.  The benchmark reports it next to the GEMM throughput: on this chip the
// sustained clock under dense MFMA load depends strongly on the entropy of the operand bits.
#include <hip/hip_runtime.h>

#include "../../include/hidet_mi355x.h"
#include "gemm_kernel.hpp"

using namespace hidet;

namespace {

constexpr int kProbeBlocks = 256, kProbeThreads = 512;  // 2 wavefronts per SIMD on every compute unit

template <typename T, int MI>
__global__ void __launch_bounds__(kProbeThreads) mfma_probe_kernel(const T* sample, int sample_elems, int iters,
                                                                   float* sink, long long* clocks) {
  using Frag = typename FragT<T>::type;
  using Acc = typename AccT<MI>::type;
  constexpr int NACC = (MI == 32) ? 8 : 16;  // enough independent accumulators to keep the pipe full
  constexpr int FE = (int)(sizeof(Frag) / sizeof(T));
  Frag a, b;
  T ta[FE], tb[FE];
  for (int e = 0; e < FE; ++e) {
    ta[e] = sample[(threadIdx.x * FE + e + blockIdx.x * 37) % sample_elems];
    tb[e] = sample[(threadIdx.x * FE + e + 1234 + blockIdx.x * 91) % sample_elems];
  }
  a = __builtin_bit_cast(Frag, ta);
  b = __builtin_bit_cast(Frag, tb);
  Acc acc[NACC];
  for (int i = 0; i < NACC; ++i)
    for (int r = 0; r < (int)(sizeof(Acc) / 4); ++r) acc[i][r] = 0.0f;
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = mfma_op(a, b, acc[i]);
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.0f;
  for (int i = 0; i < NACC; ++i)
    for (int r = 0; r < (int)(sizeof(Acc) / 4); ++r) s += acc[i][r];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    clocks[0] = c1 - c0;  // shader clocks
    clocks[1] = w1 - w0;  // constant 100 MHz counter
  }
}

__global__ void empty_kernel() {}

template <typename T, int MI>
hidet_status_t run_probe(const void* sample, long long sample_bytes, void* scratch, hipStream_t stream, float* tflops,
                         float* sclk_mhz) {
  constexpr int NACC = (MI == 32) ? 8 : 16;
  const int iters = (MI == 32) ? 6000 : 6000;
  float* sink = reinterpret_cast<float*>(scratch);
  long long* clocks = reinterpret_cast<long long*>(sink + kProbeBlocks * kProbeThreads);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return HIDET_ERR_LAUNCH;
  float best_ms = 0.0f;
  for (int rep = 0; rep < 3; ++rep) {  // the first launch also ramps the clocks
    (void)hipEventRecord(e0, stream);
    hipLaunchKernelGGL((mfma_probe_kernel<T, MI>), dim3(kProbeBlocks), dim3(kProbeThreads), 0, stream,
                       reinterpret_cast<const T*>(sample), (int)(sample_bytes / (long long)sizeof(T)), iters, sink, clocks);
    (void)hipEventRecord(e1, stream);
    if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess) {
      (void)hipEventDestroy(e0);
      (void)hipEventDestroy(e1);
      return HIDET_ERR_LAUNCH;
    }
    (void)hipEventElapsedTime(&best_ms, e0, e1);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  long long h[2] = {0, 0};
  if (hipMemcpy(h, clocks, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return HIDET_ERR_LAUNCH;
  const double k_extent = sizeof(T) == 4 ? (64.0 / MI) : (512.0 / MI);
  const double flop_per_mfma = 2.0 * MI * MI * k_extent;
  const double total = (double)kProbeBlocks * (kProbeThreads / 64) * (double)iters * NACC * flop_per_mfma;
  if (tflops) *tflops = (float)(total / (best_ms * 1e-3) / 1e12);
  if (sclk_mhz) *sclk_mhz = h[1] > 0 ? (float)((double)h[0] / ((double)h[1] / 100.0)) : 0.0f;
  return HIDET_OK;
}

}  // namespace

extern "C" hidet_status_t hidet_probe_mfma_peak(int32_t dtype, int32_t mfma, const void* sample, int64_t sample_bytes,
                                                void* scratch, int64_t scratch_bytes, void* stream, float* tflops,
                                                float* sclk_mhz) {
  if (!sample || !scratch || sample_bytes < 4096 || (mfma != 16 && mfma != 32)) return HIDET_ERR_INVALID_ARG;
  if (scratch_bytes < hidet_probe_scratch_bytes()) return HIDET_ERR_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(scratch) % 8 != 0 || reinterpret_cast<uintptr_t>(sample) % 4 != 0) return HIDET_ERR_ALIGNMENT;
  hipStream_t s = (hipStream_t)stream;
  switch (dtype) {
    case HIDET_F16:
      return mfma == 32 ? run_probe<f16, 32>(sample, sample_bytes, scratch, s, tflops, sclk_mhz)
                        : run_probe<f16, 16>(sample, sample_bytes, scratch, s, tflops, sclk_mhz);
    case HIDET_BF16:
      return mfma == 32 ? run_probe<bf16, 32>(sample, sample_bytes, scratch, s, tflops, sclk_mhz)
                        : run_probe<bf16, 16>(sample, sample_bytes, scratch, s, tflops, sclk_mhz);
    case HIDET_F32:
      return mfma == 32 ? run_probe<float, 32>(sample, sample_bytes, scratch, s, tflops, sclk_mhz)
                        : run_probe<float, 16>(sample, sample_bytes, scratch, s, tflops, sclk_mhz);
    default:
      return HIDET_ERR_INVALID_ARG;
  }
}

extern "C" int64_t hidet_probe_scratch_bytes(void) { return (int64_t)kProbeBlocks * kProbeThreads * 4 + 64; }

// Launch floor: `iters` launches of a kernel that does nothing, back to back on `stream`, between two events.
extern "C" hidet_status_t hidet_probe_launch_floor(void* stream, int32_t iters, float* us_per_launch) {
  if (iters <= 0 || !us_per_launch) return HIDET_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return HIDET_ERR_LAUNCH;
  for (int i = 0; i < 10; ++i) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, s);
  (void)hipEventRecord(e0, s);
  for (int i = 0; i < iters; ++i) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, s);
  (void)hipEventRecord(e1, s);
  float ms = 0.0f;
  const bool ok = hipGetLastError() == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
                  hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok) return HIDET_ERR_LAUNCH;
  *us_per_launch = ms * 1000.0f / (float)iters;
  return HIDET_OK;
}

// Streaming rates of plain kernels (measurement aid): what this part sustains when a kernel does nothing but read,
// write or copy memory that no cache holds -- the ceiling to hold the memory-bound products against, which the
// datasheet's 8 TB/s is not.  The buffer is walked in pieces of 128 MiB, launch after launch, so that with a buffer of
// 1 GiB every launch finds its piece in HBM only (the Infinity Cache holds 256 MB).
namespace {
typedef unsigned int stream_u32x4 __attribute__((ext_vector_type(4)));
constexpr long long kPiece = 128LL << 20;

__global__ void __launch_bounds__(256) stream_read_kernel(const stream_u32x4* src, long long n, unsigned* sink) {
  stream_u32x4 acc = {0u, 0u, 0u, 0u};
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
    acc ^= __builtin_nontemporal_load(src + i);
  // (never true for the probe's fill pattern; keeps the loads alive)
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) sink[0] = 1u;
}
__global__ void __launch_bounds__(256) stream_write_kernel(stream_u32x4* dst, long long n) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
    __builtin_nontemporal_store(stream_u32x4{1u, 2u, 3u, (unsigned)i}, dst + i);
}
__global__ void __launch_bounds__(256) stream_copy_kernel(const stream_u32x4* src, stream_u32x4* dst, long long n) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256)
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}
}  // namespace

extern "C" hidet_status_t hidet_probe_stream_bandwidth(void* buffer, int64_t bytes, int32_t mode, void* stream,
                                                       float* gbytes_per_s) {
  if (!buffer || !gbytes_per_s || mode < 0 || mode > 2) return HIDET_ERR_INVALID_ARG;
  const long long pieces = bytes / kPiece;
  if (pieces < 2) return HIDET_ERR_INVALID_ARG;  // a copy needs a source and a destination piece
  if (reinterpret_cast<uintptr_t>(buffer) % 16 != 0) return HIDET_ERR_ALIGNMENT;
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return HIDET_ERR_LAUNCH;
  unsigned char* base = static_cast<unsigned char*>(buffer);
  const long long n = kPiece / 16;
  const int grid = 8192, warm = 8, timed = 40;
  // (the read kernel's sink is the first word of another piece)
  auto launch = [&](int it) {
    unsigned char* a = base + (it % pieces) * kPiece;
    unsigned char* b = base + ((it + pieces / 2) % pieces) * kPiece;
    if (mode == 0)
      hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, s, (const stream_u32x4*)a, n, (unsigned*)b);
    else if (mode == 1)
      hipLaunchKernelGGL(stream_write_kernel, dim3(grid), dim3(256), 0, s, (stream_u32x4*)a, n);
    else
      hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(256), 0, s, (const stream_u32x4*)a, (stream_u32x4*)b, n);
  };
  for (int i = 0; i < warm; ++i) launch(i);
  (void)hipEventRecord(e0, s);
  for (int i = 0; i < timed; ++i) launch(warm + i);
  (void)hipEventRecord(e1, s);
  float ms = 0.0f;
  const bool ok = hipGetLastError() == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
                  hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok || ms <= 0.0f) return HIDET_ERR_LAUNCH;
  const double moved = (mode == 2 ? 2.0 : 1.0) * (double)kPiece * timed;
  *gbytes_per_s = (float)(moved / (ms * 1e-3) * 1e-9);
  return HIDET_OK;
}
