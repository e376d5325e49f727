// Reduction schedule template (the second of the two templates the Hidet paper schedules by hand:
// reductions such as a sum along one axis; end of Section 5) and the row softmax built from it.
//
// Both operations are memory bound: a row is read once and (softmax) written once.  The schedule is a
// task mapping in the sense of Section 5.1 over the [rows, 16-byte chunks] grid of the input:
//
//   short rows   workgroup = 4 wavefronts; wavefront = spatial(64 / L, L) over (rows, chunks) composed
//                with repeat(1, R): L lanes share one row, lane c of the group owns chunks c, c + L, ...
//                The whole row sits in registers, so max, exp and sum need one pass over memory;
//                lanes combine with xor butterflies (L is a power of two).
//   long rows    workgroup = spatial(1, 256) over chunks, repeat over the row; one row per workgroup;
//                a running (max, sum) pair per thread, merged through LDS; softmax re-reads the row
//                (from L2 when it fits) to write the result.
//
// Arithmetic is fp32 whatever the storage type.
#include <hip/hip_runtime.h>

#include "../../include/hidet_mi355x.h"
#include "gemm_kernel.hpp"

using namespace hidet;

namespace {

struct RowParams {
  const void* x;
  void* y;
  long long ldx, ldy;
  long long rows;
  int cols;
  int op;       // reduce: hidet_reduce_op_t
  int vec_in;   // rows of x allow 16-byte loads
  int vec_out;  // softmax: rows of y allow 16-byte stores
  int out_f32;  // reduce: y is fp32 whatever T is
};

constexpr float kNegInf = -__builtin_huge_valf();

template <typename T>
struct Chunk {
  static constexpr int VEC = 16 / (int)sizeof(T);
};

// One 16-byte chunk of a row -> VEC floats; elements at or beyond `cols` read as `fill`.
template <typename T>
__device__ __forceinline__ void load_chunk(const T* row, int col0, int cols, bool vec_ok, float fill, float* v) {
  constexpr int VEC = Chunk<T>::VEC;
  if (col0 + VEC <= cols && vec_ok) {
    T t[VEC];
    *reinterpret_cast<u32x4*>(t) = *reinterpret_cast<const u32x4*>(row + col0);
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] = to_f32(t[e]);
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const bool ok = col0 + e < cols;
      const T t = row[ok ? col0 + e : 0];  // cols > 0 whenever a chunk is loaded
      v[e] = ok ? to_f32(t) : fill;
    }
  }
}

template <typename T>
__device__ __forceinline__ void store_chunk(T* row, int col0, int cols, bool vec_ok, const float* v) {
  constexpr int VEC = Chunk<T>::VEC;
  T t[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) t[e] = from_f32<T>(v[e]);
  if (col0 + VEC <= cols && vec_ok) {
    *reinterpret_cast<u32x4*>(row + col0) = *reinterpret_cast<const u32x4*>(t);
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e)
      if (col0 + e < cols) row[col0 + e] = t[e];
  }
}

template <int L>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int o = L / 2; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
template <int L>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = L / 2; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ void write_scalar(const RowParams& p, long long row, float v, int dtype_tag) {
  if (p.out_f32)
    reinterpret_cast<float*>(p.y)[row] = v;
  else if (dtype_tag == 1)
    reinterpret_cast<f16*>(p.y)[row] = from_f32<f16>(v);
  else if (dtype_tag == 2)
    reinterpret_cast<bf16*>(p.y)[row] = from_f32<bf16>(v);
  else
    reinterpret_cast<float*>(p.y)[row] = v;
}

template <typename T>
struct Tag {
  static constexpr int value = sizeof(T) == 4 ? 0 : (std::is_same<T, f16>::value ? 1 : 2);
};

// ---- short rows: the row lives in the registers of L lanes ------------------------------------------
template <typename T, int L, int R, bool SOFTMAX>
__global__ void __launch_bounds__(256) rows_in_registers_kernel(const RowParams p) {
  constexpr int VEC = Chunk<T>::VEC;
  constexpr int G = 64 / L;  // rows per wavefront
  const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  const int sub = lane % L;
  const bool is_max = SOFTMAX || p.op == HIDET_REDUCE_MAX;
  const float fill = is_max ? kNegInf : 0.0f;
  const long long stride = (long long)gridDim.x * 4 * G;
  for (long long row = ((long long)blockIdx.x * 4 + wave) * G + lane / L; row < p.rows; row += stride) {
    const T* xr = reinterpret_cast<const T*>(p.x) + row * p.ldx;
    float v[R][VEC];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int col0 = (r * L + sub) * VEC;
      if (col0 < p.cols) {
        load_chunk<T>(xr, col0, p.cols, p.vec_in != 0, fill, v[r]);
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[r][e] = fill;
      }
    }
    float m = fill;
    if (is_max) {
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < VEC; ++e) m = fmaxf(m, v[r][e]);
      m = group_max<L>(m);
    }
    if constexpr (SOFTMAX) {
      float s = 0.0f;
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          v[r][e] = __expf(v[r][e] - m);  // padding: exp(-inf) = 0
          s += v[r][e];
        }
      s = group_sum<L>(s);
      const float inv = 1.0f / s;
      T* yr = reinterpret_cast<T*>(p.y) + row * p.ldy;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int col0 = (r * L + sub) * VEC;
        if (col0 < p.cols) {
#pragma unroll
          for (int e = 0; e < VEC; ++e) v[r][e] *= inv;
          store_chunk<T>(yr, col0, p.cols, p.vec_out != 0, v[r]);
        }
      }
    } else {
      float out = m;
      if (!is_max) {
        float s = 0.0f;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int e = 0; e < VEC; ++e) s += v[r][e];
        s = group_sum<L>(s);
        out = p.op == HIDET_REDUCE_MEAN ? s / (float)p.cols : s;
      }
      if (sub == 0) write_scalar(p, row, out, Tag<T>::value);
    }
  }
}

// ---- long rows: one workgroup per row, streamed ------------------------------------------------------
// Merge of two (max, sum-of-exp-relative-to-max) pairs; pairs with max = -inf carry sum 0.
__device__ __forceinline__ void merge(float& m, float& s, float m2, float s2) {
  const float mm = fmaxf(m, m2);
  const float a = (m == kNegInf) ? 0.0f : s * __expf(m - mm);
  const float b = (m2 == kNegInf) ? 0.0f : s2 * __expf(m2 - mm);
  m = mm;
  s = a + b;
}

template <typename T, bool SOFTMAX>
__global__ void __launch_bounds__(256) long_rows_kernel(const RowParams p) {
  constexpr int VEC = Chunk<T>::VEC;
  __shared__ float red_m[4], red_s[4];
  const int tid = threadIdx.x, lane = tid % 64, wave = tid / 64;
  const bool is_max = SOFTMAX || p.op == HIDET_REDUCE_MAX;
  const float fill = is_max ? kNegInf : 0.0f;
  const int chunks = (p.cols + VEC - 1) / VEC;
  for (long long row = blockIdx.x; row < p.rows; row += gridDim.x) {
    const T* xr = reinterpret_cast<const T*>(p.x) + row * p.ldx;
    float m = fill, s = 0.0f;
    for (int c = tid; c < chunks; c += 256) {
      float v[VEC];
      load_chunk<T>(xr, c * VEC, p.cols, p.vec_in != 0, fill, v);
      if (is_max) {
        float cm = v[0];
#pragma unroll
        for (int e = 1; e < VEC; ++e) cm = fmaxf(cm, v[e]);
        if constexpr (SOFTMAX) {
          if (cm != kNegInf) {
            float cs = 0.0f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) cs += __expf(v[e] - cm);
            merge(m, s, cm, cs);
          }
        } else {
          m = fmaxf(m, cm);
        }
      } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) s += v[e];
      }
    }
    // wavefront, then workgroup
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
      const float m2 = __shfl_xor(m, o, 64), s2 = __shfl_xor(s, o, 64);
      if constexpr (SOFTMAX)
        merge(m, s, m2, s2);
      else {
        m = fmaxf(m, m2);
        s += s2;
      }
    }
    __syncthreads();  // the previous row's readers are done with red_*
    if (lane == 0) {
      red_m[wave] = m;
      red_s[wave] = s;
    }
    __syncthreads();
    m = red_m[0];
    s = red_s[0];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      if constexpr (SOFTMAX)
        merge(m, s, red_m[w], red_s[w]);
      else {
        m = fmaxf(m, red_m[w]);
        s += red_s[w];
      }
    }
    if constexpr (SOFTMAX) {
      const float inv = 1.0f / s;
      T* yr = reinterpret_cast<T*>(p.y) + row * p.ldy;
      for (int c = tid; c < chunks; c += 256) {
        float v[VEC];
        load_chunk<T>(xr, c * VEC, p.cols, p.vec_in != 0, kNegInf, v);
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = __expf(v[e] - m) * inv;
        store_chunk<T>(yr, c * VEC, p.cols, p.vec_out != 0, v);
      }
    } else if (tid == 0) {
      const float out = is_max ? m : (p.op == HIDET_REDUCE_MEAN ? s / (float)p.cols : s);
      write_scalar(p, row, out, Tag<T>::value);
    }
  }
}

// ---- host side ------------------------------------------------------------------------------------------
constexpr int kMaxBlocks = 256 * 8;  // 8 workgroups of 4 wavefronts fill a compute unit

template <typename T, int L, int R, bool SOFTMAX>
hipError_t launch_short(const RowParams& p, hipStream_t stream) {
  constexpr int G = 64 / L;
  long long blocks = (p.rows + 4 * G - 1) / (4 * G);
  if (blocks > kMaxBlocks) blocks = kMaxBlocks;
  hipLaunchKernelGGL((rows_in_registers_kernel<T, L, R, SOFTMAX>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

template <typename T, bool SOFTMAX>
hipError_t dispatch(const RowParams& p, hipStream_t stream) {
  constexpr int VEC = Chunk<T>::VEC;
  const int chunks = (p.cols + VEC - 1) / VEC;
  if (chunks <= 8) return launch_short<T, 8, 1, SOFTMAX>(p, stream);
  if (chunks <= 16) return launch_short<T, 16, 1, SOFTMAX>(p, stream);
  if (chunks <= 32) return launch_short<T, 32, 1, SOFTMAX>(p, stream);
  if (chunks <= 64) return launch_short<T, 64, 1, SOFTMAX>(p, stream);
  if (chunks <= 128) return launch_short<T, 64, 2, SOFTMAX>(p, stream);
  if (chunks <= 256) return launch_short<T, 64, 4, SOFTMAX>(p, stream);
  if (chunks <= 512) return launch_short<T, 64, 8, SOFTMAX>(p, stream);
  if (chunks <= 1024) return launch_short<T, 64, 16, SOFTMAX>(p, stream);
  long long blocks = p.rows < kMaxBlocks ? p.rows : kMaxBlocks;
  hipLaunchKernelGGL((long_rows_kernel<T, SOFTMAX>), dim3((unsigned)blocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}

template <bool SOFTMAX>
hipError_t dispatch_dtype(int dtype, const RowParams& p, hipStream_t stream) {
  switch (dtype) {
    case HIDET_F32: return dispatch<float, SOFTMAX>(p, stream);
    case HIDET_F16: return dispatch<f16, SOFTMAX>(p, stream);
    default: return dispatch<bf16, SOFTMAX>(p, stream);
  }
}

bool aligned_to(const void* ptr, size_t a) { return (reinterpret_cast<uintptr_t>(ptr) % a) == 0; }
int elem_bytes(int dtype) { return dtype == HIDET_F32 ? 4 : 2; }

}  // namespace

// rows * ld elements must be addressable (below 2^47), so that the 64-bit row offsets cannot overflow
static bool span_ok(long long rows, long long ld) {
  constexpr long long lim = 1LL << 47;
  return ld <= lim && (rows <= 1 || ld <= lim / rows);
}

extern "C" {

hidet_status_t hidet_reduce_rows(int32_t in, int32_t out, int32_t op, int64_t rows, int64_t cols, const void* x,
                                 int64_t ldx, void* y, void* stream) {
  if (in < 0 || in > 2 || out < 0 || out > 2 || op < 0 || op > 2) return HIDET_ERR_INVALID_ARG;
  if (out != in && out != HIDET_F32) return HIDET_ERR_UNSUPPORTED;
  if (rows < 0 || cols < 0) return HIDET_ERR_INVALID_ARG;
  if (cols > 0x7fffffffLL - 64) return HIDET_ERR_UNSUPPORTED;
  if (rows == 0) return HIDET_OK;
  if (!y || (cols > 0 && !x) || ldx < cols) return HIDET_ERR_INVALID_ARG;
  if (!span_ok(rows, ldx)) return HIDET_ERR_UNSUPPORTED;
  if (!aligned_to(x, (size_t)elem_bytes(in)) || !aligned_to(y, (size_t)elem_bytes(out))) return HIDET_ERR_ALIGNMENT;
  RowParams p;
  p.x = x;
  p.y = y;
  p.ldx = ldx;
  p.ldy = 0;
  p.rows = rows;
  p.cols = (int)cols;
  p.op = op;
  p.vec_in = (aligned_to(x, 16) && ldx % (16 / elem_bytes(in)) == 0) ? 1 : 0;
  p.vec_out = 0;
  p.out_f32 = out == HIDET_F32 ? 1 : 0;
  return dispatch_dtype<false>(in, p, (hipStream_t)stream) == hipSuccess ? HIDET_OK : HIDET_ERR_LAUNCH;
}

hidet_status_t hidet_softmax_rows(int32_t dtype, int64_t rows, int64_t cols, const void* x, int64_t ldx, void* y,
                                  int64_t ldy, void* stream) {
  if (dtype < 0 || dtype > 2) return HIDET_ERR_INVALID_ARG;
  if (rows < 0 || cols < 0) return HIDET_ERR_INVALID_ARG;
  if (cols > 0x7fffffffLL - 64) return HIDET_ERR_UNSUPPORTED;
  if (rows == 0 || cols == 0) return HIDET_OK;
  if (!x || !y || ldx < cols || ldy < cols) return HIDET_ERR_INVALID_ARG;
  if (!span_ok(rows, ldx) || !span_ok(rows, ldy)) return HIDET_ERR_UNSUPPORTED;
  const size_t es = (size_t)elem_bytes(dtype);
  if (!aligned_to(x, es) || !aligned_to(y, es)) return HIDET_ERR_ALIGNMENT;
  RowParams p;
  p.x = x;
  p.y = y;
  p.ldx = ldx;
  p.ldy = ldy;
  p.rows = rows;
  p.cols = (int)cols;
  p.op = HIDET_REDUCE_MAX;
  p.vec_in = (aligned_to(x, 16) && ldx % (16 / (int)es) == 0) ? 1 : 0;
  p.vec_out = (aligned_to(y, 16) && ldy % (16 / (int)es) == 0) ? 1 : 0;
  p.out_f32 = 0;
  return dispatch_dtype<true>(dtype, p, (hipStream_t)stream) == hipSuccess ? HIDET_OK : HIDET_ERR_LAUNCH;
}

}  // extern "C"
