// Output index maps, the fused epilogue with its predicated store, the block-level task mapping and the pieces
// shared by the kernels.
#pragma once

#include "operand.hpp"

namespace hidet {

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
// Four 16-bit outputs as one 8-byte store.  The L2s are private to a die and write back what is dirty when the kernel
// ends; a kernel that ends by writing 32 MB spends 4-5 us there after its last instruction.  `through`: the store
// writes through the L2 (device scope), so nothing is left for that write-back -- measured 2 % (4096^3) to 9 %
// (4096 x 4096 x 256) faster.  The host asks for it only when the output's rows lie at least 4 KB apart, which is
// where it was measured to gain with the output in the Infinity Cache and out of it (2048 and 4096 columns).  With
// the 1 KB rows of 512 x 512 attention scores a 100 MB output that misses the Infinity Cache took 28 % longer when
// written through (also with tiles that span whole rows); there the store is a streaming one.
template <typename TO>
__device__ __forceinline__ void store_group(TO* dst, const TO (&o)[4], bool through) {
  static_assert(sizeof(TO) == 2, "8-byte group");
  unsigned long long bits;
  __builtin_memcpy(&bits, o, 8);
  if (through)
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else
    __builtin_nontemporal_store(bits, reinterpret_cast<unsigned long long*>(dst));
}

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
    // the output is not read again by this kernel: streamed, or written through the die's L2 (see store_group)
    if (p.vec_store >= 2) {  // 4-element aligned address
      if constexpr (sizeof(TO) == 2)
        store_group(C + off, o, p.vec_store == 3);
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
  opa.span = (Cfg::LA == L_KC) ? (long long)(opa.rows_left - 1) * p.lda + (p.K - bc.k_begin)
                               : (long long)(p.K - bc.k_begin - 1) * p.lda + opa.rows_left;
  if constexpr (Cfg::GATHER_B)
    opb.src = B;  // the gather addresses the whole input tensor
  else
    opb.src = (Cfg::LB == L_KC) ? B + (long long)bc.n0 * p.ldb + bc.k_begin : B + (long long)bc.k_begin * p.ldb + bc.n0;
  opb.ld = p.ldb;
  opb.rows_left = p.N - bc.n0;
  opb.K = bc.k_len;
  opb.kofs = bc.k_begin;
  opb.r0 = bc.n0;
  opb.span = (Cfg::LB == L_KC) ? (long long)(opb.rows_left - 1) * p.ldb + (p.K - bc.k_begin)
                               : (long long)(p.K - bc.k_begin - 1) * p.ldb + opb.rows_left;
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

// Wave groups along K (a tile configuration with WAVES_K > 1): every group holds partial sums of the same
// BM x BN tile.  They meet in LDS behind the epilogue regions; group 0 adds them in group order (so the result
// does not depend on timing) and is the only one to go on to the epilogue.  Contains one workgroup barrier and
// must be entered after a barrier that ends all use of the staging buffers.  Returns false for the wavefronts
// that are done.
template <class Cfg, class Acc>
__device__ __forceinline__ bool reduce_wave_groups(Acc (&acc)[Cfg::FM][Cfg::FN], unsigned char* smem, int kg, int wsp, int lane) {
  if constexpr (Cfg::WAVES_K > 1) {
    constexpr int FM = Cfg::FM, FN = Cfg::FN, ACC = (int)(sizeof(Acc) / 4), PER_WAVE = 64 * FM * FN * ACC;
    float* red = reinterpret_cast<float*>(smem + Cfg::EPI_BYTES);
    if (kg > 0) {
      float* mine = red + ((kg - 1) * Cfg::NWAVES_MN + wsp) * PER_WAVE + lane;
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int r = 0; r < ACC; ++r) mine[((i * FN + j) * ACC + r) * 64] = acc[i][j][r];
    }
    __syncthreads();
    if (kg > 0) return false;
#pragma unroll
    for (int g2 = 1; g2 < Cfg::WAVES_K; ++g2) {
      const float* theirs = red + ((g2 - 1) * Cfg::NWAVES_MN + wsp) * PER_WAVE + lane;
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
          for (int r = 0; r < ACC; ++r) acc[i][j][r] += theirs[((i * FN + j) * ACC + r) * 64];
    }
  }
  return true;
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
  // A tile that lies wholly inside a row-major, 8-byte-aligned 16-bit output, without residual or per-row bias (the
  // same for the whole workgroup), skips the per-group predicates of store4.
  bool lean = false;
  if constexpr (Cfg::MAPPER == MAP_PLAIN && sizeof(TO) == 2)
    lean = p.vec_store >= 2 && (!DYN || p.out_map == 0) && p.residual == nullptr && p.bias_axis != 2 &&
           bc.m0 + Cfg::BM <= p.M && bc.n0 + Cfg::BN <= p.N;
  const float alpha = p.alpha;
  const bool relu = p.relu != 0, through = p.vec_store == 3;
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
        if constexpr (Cfg::MAPPER == MAP_PLAIN && sizeof(TO) == 2) {
          if (lean) {
            TO o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float x = alpha * v[e] + col_bias[e];
              if (relu) x = x < 0.0f ? 0.0f : x;
              o[e] = from_f32<TO>(x);
            }
            store_group(C + (long long)(bc.m0 + wm0 + i * MI + row) * p.ldc + my_n, o, through);
            continue;
          }
        }
        const float vv[4] = {v[0], v[1], v[2], v[3]};
        store4<TO, Cfg::MAPPER, DYN>(p, C, R, bias, col_bias, bc.m0 + wm0 + i * MI + row, my_n, my_ccol, my_valid, vv);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
  }
}

}  // namespace hidet
