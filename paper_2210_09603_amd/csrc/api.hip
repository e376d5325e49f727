// C ABI of the library (see include/hidet_mi355x.h): argument validation, choice of the tile
// configuration, the tuner that enumerates the hardware-centric schedule space, and the launch.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/hidet_mi355x.h"
#include "registry.hpp"

using namespace hidet;

// ------------------------------------------------------------------------------------------------
// Table of contents of the schedule space + the launchers registered by the instance objects.
// ------------------------------------------------------------------------------------------------
#define HIDET_ALL
static const ConfigRow kConfigs[] = {
#define X16(idx, BM, BN, BK, WM, WN, MI, TA, SC) {idx, BM, BN, BK, WM, WN, MI, TA, SC, 0},
#define X32(idx, BM, BN, BK, WM, WN, MI, TA, SC) {idx, BM, BN, BK, WM, WN, MI, TA, SC, 1},
#include "configs.def"
#undef X16
#undef X32
};
static const int kNumConfigs = (int)(sizeof(kConfigs) / sizeof(kConfigs[0]));

// weak: a development build may leave some (configuration, type) objects out; their table slots stay empty
#define X16(idx, BM, BN, BK, WM, WN, MI, TA, SC)                                  \
  extern "C" void hidet_register_##idx##_1(Registry*) __attribute__((weak));    \
  extern "C" void hidet_register_##idx##_2(Registry*) __attribute__((weak));
#define X32(idx, BM, BN, BK, WM, WN, MI, TA, SC) extern "C" void hidet_register_##idx##_0(Registry*) __attribute__((weak));
#include "configs.def"
#undef X16
#undef X32

static const Registry& registry() {
  static Registry* r = [] {
    Registry* reg = new Registry();
    std::memset(reg, 0, sizeof(Registry));
#define X16(idx, BM, BN, BK, WM, WN, MI, TA, SC)                \
  if (hidet_register_##idx##_1) hidet_register_##idx##_1(reg); \
  if (hidet_register_##idx##_2) hidet_register_##idx##_2(reg);
#define X32(idx, BM, BN, BK, WM, WN, MI, TA, SC) \
  if (hidet_register_##idx##_0) hidet_register_##idx##_0(reg);
#include "configs.def"
#undef X16
#undef X32
    return reg;
  }();
  return *r;
}
#undef HIDET_ALL

static_assert(sizeof(kConfigs) / sizeof(kConfigs[0]) <= kMaxConfigs, "raise kMaxConfigs");

// ------------------------------------------------------------------------------------------------
// Problem description shared by GEMM, batched GEMM and conv.
// ------------------------------------------------------------------------------------------------
namespace {

struct Problem {
  int op = 0;  // 0 gemm (batched), 1 conv
  int dtype = 0;      // input type
  int wide_out = 0;   // 1: 16-bit inputs, fp32 output (and fp32 bias / residual)
  int transA = 0, transB = 0;
  long long batch = 1;
  int elem_mode = 0;  // 1: some operand is not 16-byte aligned -> element loads
  int packed = 0;     // convolution only: 1 = weights repacked to the tap-major K order (kh, kw, ic)
  GemmParams p{};
  // conv-only key fields
  long long Nb = 0, OC = 0;
};

int elem_size(int dtype) { return dtype == HIDET_F32 ? 4 : 2; }
bool aligned(const void* ptr, size_t a) { return (reinterpret_cast<uintptr_t>(ptr) % a) == 0; }
constexpr long long kIntMax = 2147483647LL;
// Largest extent of a GEMM dimension (and of the input tensor of a convolution, in elements): the kernels keep
// such indices in 32 bits and step past them by at most one tile (or one gather window) before comparing.
constexpr long long kMaxDim = kIntMax - 65536;
constexpr long long kMaxVecLd = 4LL << 20;  // in-tile element offsets (row * ld + col, row < 256) stay below 2^31
// An operand spans (rows - 1) * ld + cols elements per batch entry and batch * stride over the batch; both are
// kept below 2^47 (no allocation is larger), so that neither the checks here nor the 64-bit offsets of the kernels
// can overflow.
constexpr long long kMaxExtent = 1LL << 47;
bool extent_ok(long long rows, long long ld, long long batch, long long stride) {
  if (ld > kMaxExtent || stride > kMaxExtent) return false;
  if (rows > 1 && ld > kMaxExtent / rows) return false;
  if (batch > 1 && stride > kMaxExtent / batch) return false;
  return true;
}
// a * b, saturating at 2^62 (a, b >= 0)
long long sat_mul(long long a, long long b) {
  constexpr long long lim = 1LL << 62;
  if (a == 0 || b == 0) return 0;
  return a > lim / b ? lim : a * b;
}

// GEMM: the output has the input type, or is fp32 for 16-bit inputs.  Convolution: same type only.
hidet_status_t check_dtypes(int in, int out, bool conv) {
  if (in < 0 || in > 2 || out < 0 || out > 2) return HIDET_ERR_INVALID_ARG;
  if (in != out && (conv || out != HIDET_F32)) return HIDET_ERR_UNSUPPORTED;
  return HIDET_OK;
}

hidet_status_t check_epilogue(const hidet_epilogue_t* epi, int dtype, bool conv) {
  if (!epi) return HIDET_OK;
  if (epi->struct_size != sizeof(hidet_epilogue_t)) return HIDET_ERR_INVALID_ARG;
  if (epi->bias_axis < 0 || epi->bias_axis > 2 || epi->act < 0 || epi->act > 1) return HIDET_ERR_INVALID_ARG;
  if (epi->bias_axis != HIDET_BIAS_NONE && !epi->bias) return HIDET_ERR_INVALID_ARG;
  if (conv && epi->bias_axis == HIDET_BIAS_PER_COL) return HIDET_ERR_INVALID_ARG;
  if (epi->out_map < 0 || epi->out_map > 1 || epi->prologue < 0 || epi->prologue > 1) return HIDET_ERR_INVALID_ARG;
  if (conv && epi->out_map != HIDET_MAP_PLAIN) return HIDET_ERR_INVALID_ARG;
  const size_t es = (size_t)elem_size(dtype);
  if (epi->bias_axis != HIDET_BIAS_NONE && !aligned(epi->bias, es)) return HIDET_ERR_ALIGNMENT;
  if (epi->residual && !aligned(epi->residual, es)) return HIDET_ERR_ALIGNMENT;
  if (!(epi->alpha == epi->alpha)) return HIDET_ERR_INVALID_ARG;  // NaN scale
  return HIDET_OK;
}

void fill_epilogue(GemmParams& p, const hidet_epilogue_t* epi) {
  p.alpha = 1.0f;
  p.bias = nullptr;
  p.bias_axis = 0;
  p.residual = nullptr;
  p.ldr = 0;
  p.strideR = 0;
  p.relu = 0;
  p.relu_a = p.relu_b = 0;
  p.out_map = 0;
  p.map_seq = p.map_d = p.map_heads = 1;
  p.d_seq = p.d_hd = make_fastdiv(1);
  if (epi) {
    p.alpha = epi->alpha;
    p.bias_axis = epi->bias_axis;
    p.bias = epi->bias_axis ? epi->bias : nullptr;
    p.residual = epi->residual;
    p.ldr = epi->ld_residual;
    p.strideR = epi->batch_stride_residual;
    p.relu = epi->act == HIDET_ACT_RELU;
    p.relu_a = epi->prologue == HIDET_PROLOGUE_RELU;  // the activation operand of a GEMM (make_conv_problem moves it to x)
  }
}

hidet_status_t make_gemm_problem(Problem& pr, int in, int out, int transA, int transB, long long batch, long long M,
                                 long long N, long long K, const void* A, long long lda, long long strideA,
                                 const void* B, long long ldb, long long strideB, void* C, long long ldc,
                                 long long strideC, const hidet_epilogue_t* epi) {
  hidet_status_t st = check_dtypes(in, out, false);
  if (st != HIDET_OK) return st;
  if (batch < 0 || M < 0 || N < 0 || K < 0) return HIDET_ERR_INVALID_ARG;
  if (M > kMaxDim || N > kMaxDim || K > kMaxDim || batch > kIntMax) return HIDET_ERR_UNSUPPORTED;
  const bool empty = (batch == 0 || M == 0 || N == 0);
  st = check_epilogue(epi, out, false);
  if (st != HIDET_OK) return st;
  if (!empty) {
    if (!C) return HIDET_ERR_INVALID_ARG;
    if (K > 0 && (!A || !B)) return HIDET_ERR_INVALID_ARG;
    if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return HIDET_ERR_INVALID_ARG;
    if (strideA < 0 || strideB < 0 || strideC < 0) return HIDET_ERR_INVALID_ARG;
    if (!extent_ok(transA ? K : M, lda, batch, strideA) || !extent_ok(transB ? N : K, ldb, batch, strideB) ||
        !extent_ok(M, ldc, batch, strideC))
      return HIDET_ERR_UNSUPPORTED;
    if (batch > 1 && strideC < (M - 1) * ldc + N) return HIDET_ERR_INVALID_ARG;
    const bool head_split = epi && epi->out_map == HIDET_MAP_HEAD_SPLIT;
    if (head_split) {
      if (batch != 1) return HIDET_ERR_UNSUPPORTED;
      if (epi->map_seq <= 0 || epi->map_head_dim <= 0 || M % epi->map_seq != 0 || N % epi->map_head_dim != 0)
        return HIDET_ERR_INVALID_ARG;
    }
    if (epi && epi->residual && !head_split) {
      if (epi->ld_residual < N) return HIDET_ERR_INVALID_ARG;
      if (epi->batch_stride_residual < 0) return HIDET_ERR_INVALID_ARG;
      if (!extent_ok(M, epi->ld_residual, batch, epi->batch_stride_residual)) return HIDET_ERR_UNSUPPORTED;
    }
    const size_t es = (size_t)elem_size(in);
    if (!aligned(A, es) || !aligned(B, es) || !aligned(C, (size_t)elem_size(out))) return HIDET_ERR_ALIGNMENT;
  }
  pr.op = 0;
  pr.dtype = in;
  pr.wide_out = (in != out) ? 1 : 0;
  pr.transA = transA ? 1 : 0;
  pr.transB = transB ? 1 : 0;
  pr.batch = batch;
  GemmParams& p = pr.p;
  p.A = A;
  p.B = B;
  p.C = C;
  p.M = (int)M;
  p.N = (int)N;
  p.K = (int)K;
  p.lda = lda;
  p.ldb = ldb;
  p.ldc = ldc;
  p.strideA = strideA;
  p.strideB = strideB;
  p.strideC = strideC;
  fill_epilogue(p, epi);
  const int vec = 16 / elem_size(in);
  // vector loads need 16-byte aligned rows, no chunk straddling a matrix edge, and 32-bit in-tile offsets
  const long long a_contig = transA ? M : K, b_contig = transB ? K : N;
  const bool a_vec = aligned(A, 16) && lda % vec == 0 && strideA % vec == 0 && a_contig % vec == 0 && lda <= kMaxVecLd;
  const bool b_vec = aligned(B, 16) && ldb % vec == 0 && strideB % vec == 0 && b_contig % vec == 0 && ldb <= kMaxVecLd;
  pr.elem_mode = (a_vec && b_vec) ? 0 : 1;
  const size_t va = 4 * (size_t)elem_size(out);
  bool vs = aligned(C, va) && ldc % 4 == 0 && strideC % 4 == 0;
  if (p.residual) vs = vs && aligned(p.residual, va) && p.ldr % 4 == 0 && p.strideR % 4 == 0;
  bool contiguous4 = true;  // row-major: four consecutive columns of a row are always adjacent
  if (!empty && epi && epi->out_map == HIDET_MAP_HEAD_SPLIT) {
    p.out_map = 1;
    p.map_seq = (int)epi->map_seq;
    p.map_d = (int)epi->map_head_dim;
    p.map_heads = (int)(N / epi->map_head_dim);
    p.d_seq = make_fastdiv(epi->map_seq);
    p.d_hd = make_fastdiv(epi->map_head_dim);
    contiguous4 = epi->map_head_dim % 4 == 0;
    vs = contiguous4 && aligned(C, va) && (!p.residual || aligned(p.residual, va));
  }
  p.vec_store = vs ? 2 : (contiguous4 ? 1 : 0);
  // rows at least 4 KB apart: write the output through the L2 (see store_group)
  if (vs && p.out_map == 0 && elem_size(out) == 2 && p.ldc * 2 >= 4096) p.vec_store = 3;
  p.out_inner = 1;
  p.out_outer = 0;
  std::memset(&p.g, 0, sizeof(p.g));
  p.g.d_khw = p.g.d_kw = p.g.d_owp = p.g.d_oh = p.g.d_ic = make_fastdiv(1);
  return HIDET_OK;
}

hidet_status_t make_conv_problem(Problem& pr, int in, int out, long long Nb, long long IC, long long H, long long W,
                                 long long OC, long long KH, long long KW, long long sh, long long sw, long long ph,
                                 long long pw, const void* x, const void* w, void* y, const hidet_epilogue_t* epi) {
  hidet_status_t st = check_dtypes(in, out, true);
  if (st != HIDET_OK) return st;
  if (Nb < 0 || IC < 0 || H < 0 || W < 0 || OC < 0 || KH <= 0 || KW <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0)
    return HIDET_ERR_INVALID_ARG;
  st = check_epilogue(epi, out, true);
  if (st != HIDET_OK) return st;
  // every factor is bounded before a product is formed (the products below then stay under 2^62)
  if (Nb > kMaxDim || IC > kMaxDim || OC > kMaxDim || H > 32767 || W > 32767 || KH > 32767 || KW > 32767 ||
      ph > 32767 || pw > 32767 || sh > 32767 || sw > 32767 || Nb * IC > kMaxDim)
    return HIDET_ERR_UNSUPPORTED;
  const long long OH = (H + 2 * ph - KH) >= 0 ? (H + 2 * ph - KH) / sh + 1 : 0;
  const long long OW = (W + 2 * pw - KW) >= 0 ? (W + 2 * pw - KW) / sw + 1 : 0;
  // GEMM columns enumerate output positions with every output row padded to a multiple of 8 (see ConvGeom)
  const long long OWP = (OW + 7) / 8 * 8;
  const long long M = OC, N = Nb * OH * OWP, K = IC * KH * KW;
  // the gather keeps input rows and columns (padding included) in signed 16-bit fields and element
  // offsets in 32 bits
  if (M > kMaxDim || N > kMaxDim || K > kMaxDim || Nb * IC * H * W > kMaxDim || H + 2 * ph > 32767 ||
      W + 2 * pw > 32767)
    return HIDET_ERR_UNSUPPORTED;
  const bool empty = (M == 0 || N == 0);
  if (!empty) {
    if (!y) return HIDET_ERR_INVALID_ARG;
    if (K > 0 && (!x || !w)) return HIDET_ERR_INVALID_ARG;
    const size_t es = (size_t)elem_size(in);
    if (!aligned(x, es) || !aligned(w, es) || !aligned(y, es)) return HIDET_ERR_ALIGNMENT;
  }
  pr.op = 1;
  pr.packed = 0;
  pr.dtype = in;
  pr.wide_out = 0;
  pr.transA = 0;
  pr.transB = 0;
  pr.batch = 1;
  pr.Nb = Nb;
  pr.OC = OC;
  GemmParams& p = pr.p;
  p.A = w;
  p.B = x;
  p.C = y;
  p.M = (int)M;
  p.N = (int)N;
  p.K = (int)K;
  p.lda = K;
  p.ldb = 0;
  p.ldc = 0;
  p.strideA = p.strideB = p.strideC = 0;
  fill_epilogue(p, epi);
  p.relu_b = p.relu_a;  // the activation operand of the convolution is x, the B operand of the implicit GEMM
  p.relu_a = 0;
  p.ldr = 0;
  p.strideR = 0;
  p.g = ConvGeom{(int)IC, (int)H, (int)W, (int)KH, (int)KW, (int)sh, (int)sw, (int)ph, (int)pw, (int)OH, (int)OW,
                 (int)OWP, (int)(Nb * IC * H * W), make_fastdiv(KH * KW), make_fastdiv(KW),
                 make_fastdiv(OWP > 0 ? OWP : 1), make_fastdiv(OH > 0 ? OH : 1), (int)(H * W),
                 make_fastdiv(IC > 0 ? IC : 1)};
  p.out_inner = OH * OW;
  p.out_outer = OC * OH * OW;
  const int vec = 16 / elem_size(in);
  pr.elem_mode = (aligned(w, 16) && K % vec == 0 && K <= kMaxVecLd) ? 0 : 1;
  const size_t va = 4 * (size_t)elem_size(out);
  // a group of four positions never leaves its (padded) output row, so it is always contiguous in y;
  // it is aligned to four elements when every output row is
  bool vs = aligned(y, va) && OW % 4 == 0;
  if (p.residual) vs = vs && aligned(p.residual, va);
  p.vec_store = vs ? 2 : 1;
  return HIDET_OK;
}

LaunchFn find_launcher(const Problem& pr, int config) {
  if (config < 0 || config >= kNumConfigs) return nullptr;
  // The ring schedule is built without the run-time output map; a head-split problem takes the same tile's
  // element-mode variant, whose launcher then picks the through-registers form of the schedule.
  // repacked weights: the K axis is (kh, kw, ic) and a K tile must lie within one filter tap
  if (pr.packed) return pr.p.g.IC % kConfigs[config].bk == 0 ? registry().fn[config][pr.dtype][kConvTapVariant] : nullptr;
  // The ring schedule is also built without the input prologue (its direct loads bypass the registers): such a
  // problem takes the through-registers form likewise.
  const int elem = ((pr.p.out_map != 0 || pr.p.relu_a != 0 || pr.p.relu_b != 0) && kConfigs[config].sched == 1) ? 1 : pr.elem_mode;
  const int variant = pr.op == 1 ? conv_variant(elem) : gemm_variant(pr.transA, pr.transB, elem);
  // fp32 output from 16-bit inputs: the kernels that the K-parallel form uses for its partial sums are ordinary
  // kernels with an fp32 output type
  return registry().fn[config][pr.dtype][(pr.wide_out ? kPartialVariants : 0) + variant];
}

// The fp32-output kernel of a configuration: writes the partial sums of the K-parallel form.
LaunchFn find_partial_launcher(const Problem& pr, int config) {
  if (config < 0 || config >= kNumConfigs) return nullptr;
  if (pr.packed)
    return pr.p.g.IC % kConfigs[config].bk == 0 ? registry().fn[config][pr.dtype][kConvTapVariant + 1] : nullptr;
  const int elem = ((pr.p.relu_a != 0 || pr.p.relu_b != 0) && kConfigs[config].sched == 1) ? 1 : pr.elem_mode;  // as in find_launcher
  const int variant = pr.op == 1 ? conv_variant(elem) : gemm_variant(pr.transA, pr.transB, elem);
  return registry().fn[config][pr.dtype][kPartialVariants + variant];
}

// Untuned choice: the largest tile that still gives (nearly) every compute unit a workgroup, else the largest
// that gives a quarter of them one, else the tile with the most workgroups.  Outputs large enough to be bound by
// throughput rather than by one workgroup's latency chain (at least 384 tiles of 64x64) ask for about two
// workgroups per compute unit instead, so that one workgroup's loads and output write overlap another's
// arithmetic -- except from the ring schedule on four or more stages of K, which overlaps them inside the
// workgroup and needs just over half a round of workgroups.  Between tiles of one size the ring schedule, the
// 16x16 matrix-core shape and (small tiles) the loads-ahead order are preferred (they measure faster wherever
// both apply); the tiles that split K over wave groups take part only when K spans at least one of their K tiles
// and the output is small.  With slices > 1 only tiles that have a K-parallel form take part.
int default_config(const Problem& pr, int slices = 1) {
  const long long M = pr.p.M, N = pr.p.N;
  // (measured: equal to the two-stage tiles of their size at K = 1024, ahead beyond; the gather of the convolution
  // moves that point to about 512)
  const bool long_k = pr.p.K >= (pr.op == 1 ? 512 : 1024);
  auto rank = [long_k](const ConfigRow& r) {
    const int ahead = (r.sched == 2 && r.bm * r.bn <= 64 * 64) ? 1 : 0;  // measured faster on small tiles only
    const int ksplit = (r.sched == 3 && long_k) ? 2 : 0;  // where they take part at all, they win on a long K
    return (long long)r.bm * r.bn * 8 + (r.sched == 1 ? 4 : 0) + (r.mfma == 16 ? 2 : 0) + ahead + ksplit;
  };
  const bool throughput = sat_mul(((M + 63) / 64) * ((N + 63) / 64), pr.batch) >= 384;
  int best = -1, fewer = -1, most = -1;
  long long most_blocks = -1, best_key = -(1LL << 62), fewer_key = -(1LL << 62);
  for (int c = 0; c < kNumConfigs; ++c) {
    if (!find_launcher(pr, c)) continue;
    if (slices > 1 && !find_partial_launcher(pr, c)) continue;
    const ConfigRow& r = kConfigs[c];
    // the wave groups along K need at least one whole K tile to share, and are meant for latency-bound problems
    if (r.sched == 3 && (pr.p.K < r.bk || throughput)) continue;
    const long long blocks =
        sat_mul(((M + r.bm - 1) / r.bm) * ((N + r.bn - 1) / r.bn), pr.batch * (slices > 1 ? slices : 1));
    // the ring schedule runs GEMMs only: by direct-to-LDS loads (at any element alignment), with its stages
    // staged through registers when an input prologue has to touch the values
    const bool ring_any = r.sched == 1 && pr.op == 0 && pr.p.out_map == 0;
    const bool ring = ring_any && pr.p.relu_a == 0 && pr.p.relu_b == 0;
    // A ring tile keeps one workgroup per compute unit busy on its own (from four stages of K on).  With 129..191
    // of them the tile of half the size would need a second, mostly empty round of workgroups, so the larger one is
    // still the better choice; from 128 down the smaller tile fits into one round and wins.
    const long long area = (long long)r.bm * r.bn;
    const bool self_overlapping = ring_any && pr.p.K >= 128;
    const long long enough = !throughput ? 192 : !self_overlapping ? 400 : 129;

    // useful outputs per workgroup, discounted by the share of the tile that is padding, decide; then the smaller
    // tile, then the schedule preferences
    const long long useful = (M * N) / (((M + r.bm - 1) / r.bm) * ((N + r.bn - 1) / r.bn));
    long long key = (useful * useful / area) * (1LL << 23) - area * 64 + (rank(r) & 63);
    // a K of at most two stages runs the two-slot ring: two workgroups of a 256x128 tile share a compute unit and
    // outrun one of a 256x256 tile
    if (ring && pr.p.K <= 2 * r.bk && area == 256 * 128) key += (useful * useful / area) * (3LL << 22);
    if (blocks >= enough && key > best_key) {
      best = c;
      best_key = key;
    }
    // second choice when no tile gives that many workgroups: the same order among the tiles that still give 64
    if (blocks >= 64 && key > fewer_key) {
      fewer = c;
      fewer_key = key;
    }
    // last resort (not even 64 workgroups): the most workgroups; between equals the smaller tile, then the deeper K
    // tile that K still fills (one workgroup's latency chain is all there is to shorten), then the preferences
    auto beats = [&](const ConfigRow& a, const ConfigRow& b) {
      if (a.bm * a.bn != b.bm * b.bn) return a.bm * a.bn < b.bm * b.bn;
      const int ka = a.bk <= pr.p.K ? a.bk : 0, kb = b.bk <= pr.p.K ? b.bk : 0;
      if (ka != kb) return ka > kb;
      return rank(a) > rank(b);
    };
    if (blocks > most_blocks || (blocks == most_blocks && beats(r, kConfigs[most]))) {
      most_blocks = blocks;
      most = c;
    }
  }
  return best >= 0 ? best : (fewer >= 0 ? fewer : most);
}

// ---- static scratch of the allocation-free K-parallel entry point --------------------------------------
// One array per GPU, part of the code object, held until the process ends.  In host code the array's name is only
// a handle: the device address is asked for once per device (with that device current) and kept.
constexpr long long kScratchBytes = 32LL << 20;
constexpr int kMaxDevices = 64;
__device__ __attribute__((aligned(256))) unsigned char g_scratch[kScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {};

// ---- tuned-config cache ---------------------------------------------------------------------------
std::mutex g_mutex;

hidet_status_t scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HIDET_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_scratch)) != hipSuccess || !ptr) return HIDET_ERR_LAUNCH;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return HIDET_OK;
}
struct Tuned {
  int config;
  int slices;
  int route = 0;  // convolutions only: 1 = the remembered choice is for the batched-GEMM form of a 1x1 convolution
};
std::map<std::string, Tuned> g_cache;
std::vector<float> g_last_times;

std::string problem_key(const Problem& pr, bool with_workspace = false) {
  char buf[256];
  const GemmParams& p = pr.p;
  const int epi_kind = p.bias_axis | (p.residual ? 4 : 0) | (p.relu ? 8 : 0) | (p.alpha != 1.0f ? 16 : 0) |
                       (p.out_map ? 32 : 0) | (pr.wide_out ? 64 : 0) | ((p.relu_a || p.relu_b) ? 128 : 0);
  if (pr.op == 0)
    std::snprintf(buf, sizeof(buf), "gemm:t%d:%d%d:b%lld:%dx%dx%d:e%d:m%d", pr.dtype, pr.transA, pr.transB, pr.batch, p.M,
                  p.N, p.K, epi_kind, pr.elem_mode);
  else
    std::snprintf(buf, sizeof(buf), "conv:t%d:n%lld:c%d:%dx%d:o%lld:k%dx%d:s%dx%d:p%dx%d:e%d:m%d%s", pr.dtype, pr.Nb, p.g.IC,
                  p.g.H, p.g.W, pr.OC, p.g.KH, p.g.KW, p.g.sh, p.g.sw, p.g.ph, p.g.pw, epi_kind, pr.elem_mode,
                  pr.packed ? ":pk" : "");
  return std::string(buf) + (with_workspace ? ":ws" : "");
}

struct SplitK {  // how the caller wants K parallelised
  int slices = 1;            // requested number of K slices (<= 1: none); < 0 with a workspace: take the tuned value
  void* workspace = nullptr;
  long long workspace_bytes = 0;
  bool fixed = false;  // the workspace is the library's static scratch array: too small is HIDET_ERR_SCRATCH
};

template <int MAPPER>
hipError_t reduce_dispatch(int dtype, const GemmParams& p, int batch, hipStream_t stream) {
  switch (dtype) {
    case HIDET_F32: return launch_reduce<float, MAPPER>(p, batch, stream);
    case HIDET_F16: return launch_reduce<f16, MAPPER>(p, batch, stream);
    default: return launch_reduce<bf16, MAPPER>(p, batch, stream);
  }
}

thread_local long long g_kernel_launches = 0;  // GEMM / convolution kernels this thread has launched so far

// The part of a GEMM (rows or columns, a multiple of 256) that the 256x256 ring tile should take when the rest is
// better served by a smaller tile; none if both extents are 0.  With T tiles of 256x256, T / 256 whole rounds keep
// every compute unit busy; a thin last round leaves most of the device idle for 0.6 of a tile's time (measured: it
// runs at a higher clock than a full round).  At most 64 left-over tiles make at most 256 tiles of 128x128, one
// round that takes 0.3 to 0.45 of that time; more of them would need the 128x256 tile (0.6: no gain) or a second
// round.  Measured, 4352^3: 196 -> 154 us; 7168^3: 643 -> 602 us.  The cut is made along M or along N, whichever
// leaves fewer tiles over.
struct RoundCut {
  long long rows = 0, cols = 0;  // at most one is non-zero: extent of the head along M or along N
};
RoundCut cut_for_whole_rounds(const Problem& pr, int config, int slices) {
  RoundCut cut;
  const ConfigRow& r = kConfigs[config];
  const GemmParams& p = pr.p;
  if (pr.op != 0 || pr.batch != 1 || slices > 1 || p.out_map != 0) return cut;
  if (r.sched != 1 || r.bm != 256 || r.bn != 256) return cut;
  const long long tm = (p.M + 255) / 256, tn = (p.N + 255) / 256, tiles = tm * tn;
  const long long whole = tiles / 256;
  if (whole < 1 || tiles % 256 == 0) return cut;
  // tile rows (columns) that fit into the whole rounds, and the 256x256 tiles left over
  const long long head_rows = whole * 256 / tn, head_cols = whole * 256 / tm;
  const long long rest_rows = head_rows >= 1 && head_rows < tm ? (tm - head_rows) * tn : -1;
  const long long rest_cols = head_cols >= 1 && head_cols < tn ? (tn - head_cols) * tm : -1;
  // (at most 64: one round of 128x128 tiles)
  const bool rows_ok = rest_rows >= 0 && rest_rows <= 64, cols_ok = rest_cols >= 0 && rest_cols <= 64;
  if (rows_ok && (!cols_ok || rest_rows <= rest_cols))
    cut.rows = head_rows * 256;
  else if (cols_ok)
    cut.cols = head_cols * 256;
  return cut;
}

hidet_status_t launch(const Problem& pr_in, int config, const SplitK& sk, hipStream_t stream) {
  Problem pr = pr_in;
  GemmParams& p = pr.p;
  if (pr.batch == 0 || p.M == 0 || p.N == 0) return HIDET_OK;
  int slices = sk.slices;
  if (config < 0) {
    {
      std::lock_guard<std::mutex> lock(g_mutex);
      auto it = g_cache.find(problem_key(pr, sk.workspace != nullptr));
      if (it != g_cache.end()) {
        config = it->second.config;
        if (slices < 0) slices = it->second.slices;
      }
    }
    if (slices < 0) slices = 1;
    // (a remembered configuration that has no K-parallel form cannot serve an explicit slice count)
    if (config < 0 || !find_launcher(pr, config) || (slices > 1 && !find_partial_launcher(pr, config)))
      config = default_config(pr, slices);
    // A GEMM for which the caller named no configuration (size-based or remembered choice), on the 256x256 ring
    // tile, whose tiles fill whole rounds of the 256 compute units plus a thin last round (at most a quarter full):
    // the tile rows (or columns) that make up the whole rounds run as they are, the remaining ones run as a problem
    // of their own, for which the size-based choice takes a smaller tile that fills the device.  Two launches on
    // the same stream, no partial sums: every output element is still computed by one workgroup over all of K.
    const RoundCut cut = config >= 0 ? cut_for_whole_rounds(pr, config, slices) : RoundCut();
    if (cut.rows > 0 || cut.cols > 0) {
      Problem head = pr, tail = pr;
      const long long es_in = elem_size(pr.dtype), es_out = pr.wide_out ? 4 : es_in;
      if (cut.rows > 0) {
        const long long rows = cut.rows;
        head.p.M = (int)rows;
        tail.p.M = p.M - (int)rows;
        tail.p.A = static_cast<const char*>(p.A) + (pr.transA ? rows : rows * p.lda) * es_in;
        tail.p.C = static_cast<char*>(p.C) + rows * p.ldc * es_out;
        if (p.residual) tail.p.residual = static_cast<const char*>(p.residual) + rows * p.ldr * es_out;
        if (p.bias && p.bias_axis == 2) tail.p.bias = static_cast<const char*>(p.bias) + rows * es_out;
      } else {
        const long long cols = cut.cols;
        head.p.N = (int)cols;
        tail.p.N = p.N - (int)cols;
        tail.p.B = static_cast<const char*>(p.B) + (pr.transB ? cols * p.ldb : cols) * es_in;
        tail.p.C = static_cast<char*>(p.C) + cols * es_out;
        if (p.residual) tail.p.residual = static_cast<const char*>(p.residual) + cols * es_out;
        if (p.bias && p.bias_axis == 1) tail.p.bias = static_cast<const char*>(p.bias) + cols * es_out;
      }
      // the rest's configuration is settled before anything is launched: a call that fails has written nothing
      const int tail_config = default_config(tail, 1);
      if (tail_config >= 0 && find_launcher(tail, tail_config) && find_launcher(head, config)) {
        const hidet_status_t st = launch(head, config, sk, stream);
        return st != HIDET_OK ? st : launch(tail, tail_config, sk, stream);
      }
    }
  }
  if (slices < 0) slices = 1;
  LaunchFn fn = find_launcher(pr, config);
  if (!fn) return HIDET_ERR_NO_CONFIG;
  const ConfigRow& r = kConfigs[config];
  p.tiles_m = (p.M + r.bm - 1) / r.bm;
  p.tiles_n = (p.N + r.bn - 1) / r.bn;
  // grouped traversal: each run of 32 consecutive workgroups (one die's share of a 256-tile wave)
  // should cover a near-square patch of tiles
  p.group = p.tiles_m >= 4 ? 4 : p.tiles_m;
  p.k_slices = 1;
  p.k_slice_len = p.K;
  long long len = p.K, actual = 1;
  if (slices > 1 && p.K > 0) {
    len = (p.K + slices - 1) / slices;
    len = (len + r.bk - 1) / r.bk * r.bk;  // whole K tiles per slice keeps every slice 16-byte aligned
    actual = (p.K + len - 1) / len;
  }
  if (actual <= 1) {
    const long long total = sat_mul((long long)p.tiles_m * p.tiles_n, pr.batch);
    if (total > kIntMax) return HIDET_ERR_UNSUPPORTED;
    p.total_blocks = (int)total;
    if (fn(p, stream) != hipSuccess) return HIDET_ERR_LAUNCH;
    ++g_kernel_launches;
    return HIDET_OK;
  }
  // ---- parallel reduction on K: partial sums into the workspace, then reduce + epilogue
  LaunchFn pfn = find_partial_launcher(pr, config);
  if (!pfn) return HIDET_ERR_NO_CONFIG;
  if (pr.batch > 65535) return HIDET_ERR_UNSUPPORTED;
  const long long total = sat_mul((long long)p.tiles_m * p.tiles_n, pr.batch * actual);
  if (total > kIntMax) return HIDET_ERR_UNSUPPORTED;
  const long long need = sat_mul(sat_mul(4LL * pr.batch * actual, p.M), p.N);
  if (sk.fixed && sk.workspace_bytes < need) return HIDET_ERR_SCRATCH;
  if (!sk.workspace || sk.workspace_bytes < need) return HIDET_ERR_INVALID_ARG;
  if (!aligned(sk.workspace, 16)) return HIDET_ERR_ALIGNMENT;
  GemmParams q = p;
  q.C = sk.workspace;
  q.ldc = p.N;
  q.strideC = (long long)p.M * p.N;
  q.alpha = 1.0f;
  q.bias = nullptr;
  q.bias_axis = 0;
  q.residual = nullptr;
  q.relu = 0;
  q.out_map = 0;
  q.vec_store = (p.N % 4 == 0) ? 2 : 1;
  q.k_slices = (int)actual;
  q.k_slice_len = (int)len;
  q.total_blocks = (int)total;
  q.out_inner = 1;
  q.out_outer = 0;
  if (pfn(q, stream) != hipSuccess) return HIDET_ERR_LAUNCH;
  ++g_kernel_launches;
  GemmParams rp = p;
  rp.A = sk.workspace;
  rp.k_slices = (int)actual;
  const int out_type = pr.wide_out ? (int)HIDET_F32 : pr.dtype;
  const hipError_t e = pr.op == 1 ? reduce_dispatch<MAP_NCHW>(out_type, rp, (int)pr.batch, stream)
                                  : reduce_dispatch<MAP_PLAIN>(out_type, rp, (int)pr.batch, stream);
  if (e == hipSuccess) ++g_kernel_launches;
  return e == hipSuccess ? HIDET_OK : HIDET_ERR_LAUNCH;
}

const int kSliceChoices[] = {1, 2, 3, 4, 6, 8, 12, 16};

// Enumerates the schedule space (x the K-slice choices when a workspace is given) on the caller's fused problem.
hidet_status_t tune(const Problem& pr, const SplitK& sk, hipStream_t stream, int iters, int32_t* best_config,
                    int32_t* best_slices, float* best_us) {
  if (iters <= 0) iters = 10;
  std::vector<float> times(kNumConfigs, -1.0f);
  int best = -1, best_sl = 1;
  float best_t = 0.0f;
  if (!(pr.batch == 0 || pr.p.M == 0 || pr.p.N == 0)) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return HIDET_ERR_LAUNCH;
    for (int c = 0; c < kNumConfigs; ++c) {
      if (!find_launcher(pr, c)) continue;
      for (int sl : kSliceChoices) {
        if (sl > 1 && !sk.workspace) break;
        SplitK one = sk;
        one.slices = sl;
        hidet_status_t st = launch(pr, c, one, stream);  // warm-up, also loads the code object
        if (st != HIDET_OK) continue;
        (void)hipEventRecord(e0, stream);
        for (int i = 0; i < iters; ++i) launch(pr, c, one, stream);
        (void)hipEventRecord(e1, stream);
        if (hipEventSynchronize(e1) != hipSuccess) {
          (void)hipEventDestroy(e0);
          (void)hipEventDestroy(e1);
          return HIDET_ERR_LAUNCH;
        }
        float ms = 0.0f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        const float us = ms * 1000.0f / (float)iters;
        if (times[c] < 0.0f || us < times[c]) times[c] = us;
        if (best < 0 || us < best_t) {
          best = c;
          best_sl = sl;
          best_t = us;
        }
      }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (best < 0) return HIDET_ERR_NO_CONFIG;
    // leave the winner's output in the buffer
    SplitK win = sk;
    win.slices = best_sl;
    launch(pr, best, win, stream);
    (void)hipStreamSynchronize(stream);
  }
  {
    std::lock_guard<std::mutex> lock(g_mutex);
    if (best >= 0) g_cache[problem_key(pr, sk.workspace != nullptr)] = Tuned{best, best_sl, 0};
    g_last_times = times;
  }
  if (best_config) *best_config = best;
  if (best_slices) *best_slices = best_sl;
  if (best_us) *best_us = best_t;
  return HIDET_OK;
}

// No C++ exception crosses the C boundary: the cache and the tuner allocate host memory (strings, a map, a
// vector), and a failed allocation is reported as a failed launch.
template <class F>
hidet_status_t guarded(F f) noexcept {
  try {
    return f();
  } catch (...) {
    return HIDET_ERR_LAUNCH;
  }
}

// ---- convolution calls ------------------------------------------------------------------------------------------
// A 1x1 convolution with unit stride and no padding needs no gather: image b of x is an IC x (H*W) row-major
// matrix as it stands, so y[b] = w . x[b] is a batched GEMM with the weights shared across the batch (and the
// aligned direct-to-LDS loads of the ring schedule apply).  Such a call carries both descriptions of the problem.
struct ConvCall {
  Problem conv, gemm;
  bool pointwise = false;
};

hidet_status_t make_conv_call(ConvCall& cc, int in, int out, long long Nb, long long IC, long long H, long long W,
                              long long OC, long long KH, long long KW, long long sh, long long sw, long long ph,
                              long long pw, const void* x, const void* w, void* y, const hidet_epilogue_t* epi) {
  const hidet_status_t st = make_conv_problem(cc.conv, in, out, Nb, IC, H, W, OC, KH, KW, sh, sw, ph, pw, x, w, y, epi);
  if (st != HIDET_OK) return st;
  cc.pointwise = false;
  if (KH == 1 && KW == 1 && sh == 1 && sw == 1 && ph == 0 && pw == 0) {
    hidet_epilogue_t e;
    const hidet_epilogue_t* ep = nullptr;
    if (epi) {  // the residual is a dense tensor of y's shape
      e = *epi;
      e.ld_residual = H * W;
      e.batch_stride_residual = OC * H * W;
      ep = &e;
    }
    cc.pointwise = make_gemm_problem(cc.gemm, in, out, 0, 0, Nb, OC, H * W, IC, w, IC, 0, x, H * W, IC * H * W, y, H * W,
                                     OC * H * W, ep) == HIDET_OK;
    // the activation operand is x here too: the B operand of this GEMM
    cc.gemm.p.relu_b = cc.gemm.p.relu_a;
    cc.gemm.p.relu_a = 0;
  }
  return HIDET_OK;
}

// An explicit configuration always runs the gather form; config < 0 runs what the tuner remembered for this
// convolution, else (1x1 convolutions) the batched-GEMM form with its size-based default.
hidet_status_t launch_conv(const ConvCall& cc, int config, const SplitK& sk, hipStream_t stream) {
  if (config >= 0 || !cc.pointwise) return launch(cc.conv, config, sk, stream);
  Tuned t{-1, 1, 0};
  {
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_cache.find(problem_key(cc.conv, sk.workspace != nullptr));
    if (it != g_cache.end()) t = it->second;
  }
  if (t.config < 0) return launch(cc.gemm, -1, sk, stream);
  SplitK one = sk;
  if (one.slices < 0) one.slices = t.slices;
  return launch(t.route == 1 ? cc.gemm : cc.conv, t.config, one, stream);
}

// Tunes the gather form and, for a 1x1 convolution, the batched-GEMM form; the faster one is remembered under
// the convolution's key.
hidet_status_t tune_conv(const ConvCall& cc, const SplitK& sk, hipStream_t stream, int iters, int32_t* best_config,
                         int32_t* best_slices, float* best_us) {
  int32_t c0 = -1, s0 = 1;
  float t0 = 0.0f;
  hidet_status_t st = tune(cc.conv, sk, stream, iters, &c0, &s0, &t0);
  if (st != HIDET_OK) return st;
  if (cc.pointwise) {
    std::vector<float> times0;
    {
      std::lock_guard<std::mutex> lock(g_mutex);
      times0 = g_last_times;
    }
    int32_t c1 = -1, s1 = 1;
    float t1 = 0.0f;
    st = tune(cc.gemm, sk, stream, iters, &c1, &s1, &t1);
    if (st != HIDET_OK) return st;
    std::lock_guard<std::mutex> lock(g_mutex);
    for (size_t i = 0; i < g_last_times.size() && i < times0.size(); ++i)
      if (times0[i] >= 0.0f && (g_last_times[i] < 0.0f || times0[i] < g_last_times[i])) g_last_times[i] = times0[i];
    if (c1 >= 0 && (c0 < 0 || t1 < t0)) {
      g_cache[problem_key(cc.conv, sk.workspace != nullptr)] = Tuned{c1, s1, 1};
      c0 = c1;
      s0 = s1;
      t0 = t1;
    }
  }
  if (best_config) *best_config = c0;
  if (best_slices) *best_slices = s0;
  if (best_us) *best_us = t0;
  return HIDET_OK;
}

// ---- convolution with repacked weights ----------------------------------------------------------------------------
// OIHW -> O(HW)I: w_packed[oc][kh][kw][ic] = w[oc][ic][kh][kw].  With the K axis of the implicit GEMM ordered
// (kh, kw, ic) a K tile lies within one filter tap, which makes the padding mask and the spatial offset of the img2col
// gather the same for all of a thread's chunks of the tile (Operand::request_tile).
template <typename U>
__global__ void __launch_bounds__(256) pack_weights_kernel(const U* __restrict__ w, U* __restrict__ wp, long long total,
                                                          int IC, int KHW, FastDiv d_ic) {
  const long long o = (long long)blockIdx.x * 256 + threadIdx.x;
  if (o >= total) return;
  // o = (oc * KHW + t) * IC + ic; rows of KHW * IC elements stay below 2^31 (checked on the host)
  const long long row = o / ((long long)KHW * IC);
  const int in_row = (int)(o - row * ((long long)KHW * IC));
  const int t = d_ic.div(in_row), ic = in_row - t * IC;
  wp[o] = w[row * ((long long)KHW * IC) + (long long)ic * KHW + t];
}

// The packed form: a ConvCall whose gather problem is marked `packed`.  Needs IC % 8 == 0 (16-byte rows of the
// repacked weights), strides of at most 2 and an input of at least two chunks.
hidet_status_t make_packed_conv_call(ConvCall& cc, int in, int out, long long Nb, long long IC, long long H, long long W,
                                     long long OC, long long KH, long long KW, long long sh, long long sw, long long ph,
                                     long long pw, const void* x, const void* w_packed, void* y,
                                     const hidet_epilogue_t* epi) {
  const hidet_status_t st = make_conv_problem(cc.conv, in, out, Nb, IC, H, W, OC, KH, KW, sh, sw, ph, pw, x, w_packed, y, epi);
  if (st != HIDET_OK) return st;
  const int vec = 16 / elem_size(in);
  if (IC % vec != 0 || sw > 2 || Nb * IC * H * W < 4 * vec || cc.conv.elem_mode != 0) return HIDET_ERR_UNSUPPORTED;
  cc.conv.packed = 1;
  cc.pointwise = false;
  return HIDET_OK;
}

// ---- task-mapping instances exposed to tests ----------------------------------------------------------
struct TaskMapEntry {
  const char* expr;
  int workers, shape0, shape1, tasks;
  tmap::Task (*task)(int, int);
};
template <class M>
TaskMapEntry tm_entry(const char* expr) {
  return TaskMapEntry{expr, M::workers, M::shape0, M::shape1, M::tasks, [](int w, int q) { return M::task(w, q); }};
}
using namespace hidet::tmap;
const TaskMapEntry kTaskMaps[] = {
    // the paper's worked examples
    tm_entry<Compose<Repeat<4, 1>, Spatial<16, 8>>>("repeat(4,1)*spatial(16,8)"),
    tm_entry<Chain<Spatial<4, 2>, Repeat<2, 2>, Spatial<4, 8>, Repeat<4, 4>>>(
        "spatial(4,2)*repeat(2,2)*spatial(4,8)*repeat(4,4)"),
    tm_entry<Compose<Spatial<2, 2>, Repeat<2, 2>>>("spatial(2,2)*repeat(2,2)"),
    tm_entry<Repeat<2, 2>>("repeat(2,2)"),
    tm_entry<Spatial<2, 2>>("spatial(2,2)"),
    tm_entry<Compose<Spatial<1, 3>, Spatial<2, 1>>>("spatial(1,3)*spatial(2,1)"),
    tm_entry<Compose<Compose<Repeat<2, 1>, Spatial<2, 3>>, Repeat<1, 2>>>("repeat(2,1)*spatial(2,3)*repeat(1,2)"),
    tm_entry<Compose<Repeat<2, 1>, Compose<Spatial<2, 3>, Repeat<1, 2>>>>("repeat(2,1)*spatial(2,3)*repeat(1,2)"),
    // the mappings the headline kernel (configuration 19: 256x256x32 tile, 8 waves, 16x16x32 matrix-core tiles) walks:
    // its direct global -> LDS loads (Operand::init_direct) and its wave -> MFMA-tile assignment
    tm_entry<LoadMapRowMajor<256, 4, 512>::Map>("repeat(2,1)*spatial(128,4)"),   // A tile, 256 rows x 4 chunks
    tm_entry<LoadMapRowMajor<32, 32, 512>::Map>("repeat(2,1)*spatial(16,32)"),   // B tile, 32 k-rows x 32 chunks
    tm_entry<Compose<Spatial<2, 4>, Repeat<8, 4>>>("spatial(2,4)*repeat(8,4)"),  // waves -> MFMA tiles
    // the same for the general schedule on a 256x256x64 tile with 32x32x16 tiles (configuration 20)
    tm_entry<LoadMapRowMajor<256, 8, 512>::Map>("repeat(4,1)*spatial(64,8)"),    // A tile, 256 rows x 8 chunks
    tm_entry<LoadMapRowMajor<64, 32, 512>::Map>("repeat(4,1)*spatial(16,32)"),   // B tile, 64 k-rows x 32 chunks
    tm_entry<Compose<Spatial<2, 4>, Repeat<4, 2>>>("spatial(2,4)*repeat(4,2)"),  // waves -> MFMA tiles
    // fp32 A tile of the 128x128x16 configuration: threads walk down the rows first
    tm_entry<LoadMapColMajor<128, 4, 256>::Map>("repeat(2,1)*spatial(2,128)"),
    tm_entry<LoadMapColMajor<256, 4, 128>::Map>("repeat(4,2)*spatial(1,128)"),
};
const int kNumTaskMaps = (int)(sizeof(kTaskMaps) / sizeof(kTaskMaps[0]));

}  // namespace

// ------------------------------------------------------------------------------------------------
// exported functions
// ------------------------------------------------------------------------------------------------
extern "C" {

hidet_status_t hidet_batched_gemm_cfg(int32_t config, int32_t in, int32_t out, int32_t transA, int32_t transB,
                                      int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                      int64_t strideA, const void* B, int64_t ldb, int64_t strideB, void* C,
                                      int64_t ldc, int64_t strideC, const hidet_epilogue_t* epi, void* stream) {
  Problem pr;
  hidet_status_t st = make_gemm_problem(pr, in, out, transA, transB, batch, M, N, K, A, lda, strideA, B, ldb, strideB,
                                        C, ldc, strideC, epi);
  if (st != HIDET_OK) return st;
  if (config >= kNumConfigs) return HIDET_ERR_NO_CONFIG;
  return guarded([&] { return launch(pr, config, SplitK{}, (hipStream_t)stream); });
}

hidet_status_t hidet_gemm_cfg(int32_t config, int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t M,
                              int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
                              int64_t ldc, const hidet_epilogue_t* epi, void* stream) {
  return hidet_batched_gemm_cfg(config, in, out, transA, transB, 1, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, epi,
                                stream);
}

hidet_status_t hidet_gemm(int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t M, int64_t N, int64_t K,
                          const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                          const hidet_epilogue_t* epi, void* stream) {
  return hidet_gemm_cfg(-1, in, out, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, epi, stream);
}

hidet_status_t hidet_batched_gemm(int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t batch, int64_t M,
                                  int64_t N, int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                                  int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                                  const hidet_epilogue_t* epi, void* stream) {
  return hidet_batched_gemm_cfg(-1, in, out, transA, transB, batch, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc,
                                strideC, epi, stream);
}

hidet_status_t hidet_conv2d_implicit_gemm_cfg(int32_t config, int32_t in, int32_t out, int64_t Nb, int64_t IC,
                                              int64_t H, int64_t W, int64_t OC, int64_t KH, int64_t KW,
                                              int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                              const void* x, const void* w, void* y, const hidet_epilogue_t* epi,
                                              void* stream) {
  ConvCall cc;
  hidet_status_t st = make_conv_call(cc, in, out, Nb, IC, H, W, OC, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                                     epi);
  if (st != HIDET_OK) return st;
  if (config >= kNumConfigs) return HIDET_ERR_NO_CONFIG;
  return guarded([&] { return launch_conv(cc, config, SplitK{}, (hipStream_t)stream); });
}

hidet_status_t hidet_conv2d_implicit_gemm(int32_t in, int32_t out, int64_t Nb, int64_t IC, int64_t H, int64_t W,
                                          int64_t OC, int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                          int64_t pad_h, int64_t pad_w, const void* x, const void* w, void* y,
                                          const hidet_epilogue_t* epi, void* stream) {
  return hidet_conv2d_implicit_gemm_cfg(-1, in, out, Nb, IC, H, W, OC, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w,
                                        y, epi, stream);
}

int32_t hidet_config_count(void) { return kNumConfigs; }

hidet_status_t hidet_config_info(int32_t config, hidet_config_info_t* info) {
  if (!info) return HIDET_ERR_INVALID_ARG;
  if (config < 0 || config >= kNumConfigs) return HIDET_ERR_NO_CONFIG;
  const ConfigRow& r = kConfigs[config];
  info->block_m = r.bm;
  info->block_n = r.bn;
  info->block_k = r.bk;
  info->waves_m = r.waves_m;
  info->waves_n = r.waves_n;
  info->mfma = r.mfma;
  info->is_f32 = r.is_f32;
  info->schedule = r.sched;
  info->stages = r.sched == 1 ? 4 : 2;
  info->waves_k = r.sched == 3 ? 16 / (r.waves_m * r.waves_n) : 1;
  const int staging = info->stages * (r.bm + r.bn) * r.bk * (r.is_f32 ? 4 : 2);
  int epilogue = r.waves_m * r.mfma * (r.bn * 4 + 16 * r.waves_n);  // per-wave transposition regions
  if (r.sched == 3) epilogue += (16 / (r.waves_m * r.waves_n) - 1) * r.bm * r.bn * 4;  // partial sums of the wave groups along K
  info->lds_bytes = staging > epilogue ? staging : epilogue;  // (GEMM form; the convolution adds a 1.3 KB mask table)
  return HIDET_OK;
}

hidet_status_t hidet_tune_gemm(int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t batch, int64_t M,
                               int64_t N, int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                               int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                               const hidet_epilogue_t* epi, void* stream, int32_t iters, int32_t* best_config,
                               float* best_us) {
  Problem pr;
  hidet_status_t st = make_gemm_problem(pr, in, out, transA, transB, batch, M, N, K, A, lda, strideA, B, ldb, strideB,
                                        C, ldc, strideC, epi);
  if (st != HIDET_OK) return st;
  return guarded([&] { return tune(pr, SplitK{}, (hipStream_t)stream, iters, best_config, nullptr, best_us); });
}

hidet_status_t hidet_tune_conv2d(int32_t in, int32_t out, int64_t Nb, int64_t IC, int64_t H, int64_t W, int64_t OC,
                                 int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                 int64_t pad_w, const void* x, const void* w, void* y, const hidet_epilogue_t* epi,
                                 void* stream, int32_t iters, int32_t* best_config, float* best_us) {
  ConvCall cc;
  hidet_status_t st = make_conv_call(cc, in, out, Nb, IC, H, W, OC, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                                     epi);
  if (st != HIDET_OK) return st;
  return guarded([&] { return tune_conv(cc, SplitK{}, (hipStream_t)stream, iters, best_config, nullptr, best_us); });
}

// ---- K-parallel ("split-K") forms ------------------------------------------------------------------------------
int64_t hidet_splitk_workspace_bytes(int64_t batch, int64_t M, int64_t N, int32_t k_slices) {
  if (batch < 0 || M < 0 || N < 0 || k_slices < 1) return -1;
  const long long bytes = sat_mul(sat_mul(sat_mul(4LL * k_slices, batch), M), N);
  return bytes >= (1LL << 62) ? -1 : bytes;
}

hidet_status_t hidet_batched_gemm_splitk(int32_t config, int32_t k_slices, int32_t in, int32_t out, int32_t transA,
                                         int32_t transB, int64_t batch, int64_t M, int64_t N, int64_t K, const void* A,
                                         int64_t lda, int64_t strideA, const void* B, int64_t ldb, int64_t strideB,
                                         void* C, int64_t ldc, int64_t strideC, const hidet_epilogue_t* epi,
                                         void* workspace, int64_t workspace_bytes, void* stream) {
  Problem pr;
  hidet_status_t st = make_gemm_problem(pr, in, out, transA, transB, batch, M, N, K, A, lda, strideA, B, ldb, strideB,
                                        C, ldc, strideC, epi);
  if (st != HIDET_OK) return st;
  if (config >= kNumConfigs) return HIDET_ERR_NO_CONFIG;
  if (workspace_bytes < 0 || k_slices > 1024) return HIDET_ERR_INVALID_ARG;
  SplitK sk;
  sk.slices = k_slices <= 0 ? -1 : k_slices;
  sk.workspace = workspace;
  sk.workspace_bytes = workspace_bytes;
  return guarded([&] { return launch(pr, config, sk, (hipStream_t)stream); });
}

hidet_status_t hidet_conv2d_implicit_gemm_splitk(int32_t config, int32_t k_slices, int32_t in, int32_t out, int64_t Nb,
                                                 int64_t IC, int64_t H, int64_t W, int64_t OC, int64_t KH, int64_t KW,
                                                 int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                                 const void* x, const void* w, void* y, const hidet_epilogue_t* epi,
                                                 void* workspace, int64_t workspace_bytes, void* stream) {
  ConvCall cc;
  hidet_status_t st = make_conv_call(cc, in, out, Nb, IC, H, W, OC, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                                     epi);
  if (st != HIDET_OK) return st;
  if (config >= kNumConfigs) return HIDET_ERR_NO_CONFIG;
  if (workspace_bytes < 0 || k_slices > 1024) return HIDET_ERR_INVALID_ARG;
  SplitK sk;
  sk.slices = k_slices <= 0 ? -1 : k_slices;
  sk.workspace = workspace;
  sk.workspace_bytes = workspace_bytes;
  return guarded([&] { return launch_conv(cc, config, sk, (hipStream_t)stream); });
}

hidet_status_t hidet_conv2d_pack_weights(int32_t dtype, int64_t OC, int64_t IC, int64_t KH, int64_t KW, const void* w,
                                         void* w_packed, void* stream) {
  if (dtype < 0 || dtype > 2 || OC < 0 || IC < 0 || KH <= 0 || KW <= 0) return HIDET_ERR_INVALID_ARG;
  if (KH > 32767 || KW > 32767 || IC > kMaxDim || OC > kMaxDim || sat_mul(IC, KH * KW) > kMaxDim) return HIDET_ERR_UNSUPPORTED;
  const long long total = sat_mul(OC, IC * KH * KW);
  if (total == 0) return HIDET_OK;
  if (total > (1LL << 40)) return HIDET_ERR_UNSUPPORTED;
  if (!w || !w_packed) return HIDET_ERR_INVALID_ARG;
  const size_t es = (size_t)elem_size(dtype);
  if (!aligned(w, es) || !aligned(w_packed, es)) return HIDET_ERR_ALIGNMENT;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  if (es == 2)
    hipLaunchKernelGGL(pack_weights_kernel<unsigned short>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const unsigned short*)w, (unsigned short*)w_packed, total, (int)IC, (int)(KH * KW), make_fastdiv(IC));
  else
    hipLaunchKernelGGL(pack_weights_kernel<unsigned int>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const unsigned int*)w, (unsigned int*)w_packed, total, (int)IC, (int)(KH * KW), make_fastdiv(IC));
  return hipGetLastError() == hipSuccess ? HIDET_OK : HIDET_ERR_LAUNCH;
}

hidet_status_t hidet_conv2d_implicit_gemm_packed(int32_t config, int32_t k_slices, int32_t in, int32_t out, int64_t Nb,
                                                 int64_t IC, int64_t H, int64_t W, int64_t OC, int64_t KH, int64_t KW,
                                                 int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                                 const void* x, const void* w_packed, void* y, const hidet_epilogue_t* epi,
                                                 void* workspace, int64_t workspace_bytes, void* stream) {
  ConvCall cc;
  hidet_status_t st = make_packed_conv_call(cc, in, out, Nb, IC, H, W, OC, KH, KW, stride_h, stride_w, pad_h, pad_w, x,
                                            w_packed, y, epi);
  if (st != HIDET_OK) return st;
  if (config >= kNumConfigs) return HIDET_ERR_NO_CONFIG;
  if (workspace_bytes < 0 || k_slices > 1024) return HIDET_ERR_INVALID_ARG;
  SplitK sk;
  sk.slices = k_slices <= 0 ? (workspace ? -1 : 1) : k_slices;
  sk.workspace = workspace;
  sk.workspace_bytes = workspace_bytes;
  return guarded([&] { return launch(cc.conv, config, sk, (hipStream_t)stream); });
}

hidet_status_t hidet_tune_conv2d_packed(int32_t in, int32_t out, int64_t Nb, int64_t IC, int64_t H, int64_t W, int64_t OC,
                                        int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                        int64_t pad_w, const void* x, const void* w_packed, void* y,
                                        const hidet_epilogue_t* epi, void* workspace, int64_t workspace_bytes, void* stream,
                                        int32_t iters, int32_t* best_config, int32_t* best_slices, float* best_us) {
  ConvCall cc;
  hidet_status_t st = make_packed_conv_call(cc, in, out, Nb, IC, H, W, OC, KH, KW, stride_h, stride_w, pad_h, pad_w, x,
                                            w_packed, y, epi);
  if (st != HIDET_OK) return st;
  if (workspace_bytes < 0) return HIDET_ERR_INVALID_ARG;
  SplitK sk;
  sk.workspace = workspace;
  sk.workspace_bytes = workspace ? workspace_bytes : 0;
  return guarded([&] { return tune(cc.conv, sk, (hipStream_t)stream, iters, best_config, best_slices, best_us); });
}

int64_t hidet_conv2d_splitk_workspace_bytes(int64_t Nb, int64_t OC, int64_t OH, int64_t OW, int32_t k_slices) {
  if (Nb < 0 || OC < 0 || OH < 0 || OW < 0 || OW > kIntMax) return -1;
  // GEMM columns of the implicit GEMM: every output row padded to a multiple of 8 positions (see ConvGeom)
  return hidet_splitk_workspace_bytes(1, OC, sat_mul(sat_mul(Nb, OH), (OW + 7) / 8 * 8), k_slices);
}

int64_t hidet_static_scratch_bytes(void) { return kScratchBytes; }

hidet_status_t hidet_batched_gemm_splitk_static(int32_t config, int32_t k_slices, int32_t in, int32_t out,
                                                int32_t transA, int32_t transB, int64_t batch, int64_t M, int64_t N,
                                                int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                                                int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                                                const hidet_epilogue_t* epi, void* stream) {
  Problem pr;
  hidet_status_t st = make_gemm_problem(pr, in, out, transA, transB, batch, M, N, K, A, lda, strideA, B, ldb, strideB,
                                        C, ldc, strideC, epi);
  if (st != HIDET_OK) return st;
  if (config >= kNumConfigs) return HIDET_ERR_NO_CONFIG;
  if (k_slices > 1024) return HIDET_ERR_INVALID_ARG;
  SplitK sk;
  sk.slices = k_slices <= 0 ? -1 : k_slices;
  sk.workspace_bytes = kScratchBytes;
  sk.fixed = true;
  st = scratch_of_current_device(&sk.workspace);
  if (st != HIDET_OK) return st;
  return guarded([&] { return launch(pr, config, sk, (hipStream_t)stream); });
}

hidet_status_t hidet_tune_gemm_splitk(int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t batch, int64_t M,
                                      int64_t N, int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                                      int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                                      const hidet_epilogue_t* epi, void* workspace, int64_t workspace_bytes, void* stream,
                                      int32_t iters, int32_t* best_config, int32_t* best_slices, float* best_us) {
  Problem pr;
  hidet_status_t st = make_gemm_problem(pr, in, out, transA, transB, batch, M, N, K, A, lda, strideA, B, ldb, strideB,
                                        C, ldc, strideC, epi);
  if (st != HIDET_OK) return st;
  if (!workspace || workspace_bytes <= 0) return HIDET_ERR_INVALID_ARG;
  SplitK sk;
  sk.workspace = workspace;
  sk.workspace_bytes = workspace_bytes;
  return guarded([&] { return tune(pr, sk, (hipStream_t)stream, iters, best_config, best_slices, best_us); });
}

hidet_status_t hidet_tune_conv2d_splitk(int32_t in, int32_t out, int64_t Nb, int64_t IC, int64_t H, int64_t W,
                                        int64_t OC, int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                        int64_t pad_h, int64_t pad_w, const void* x, const void* w, void* y,
                                        const hidet_epilogue_t* epi, void* workspace, int64_t workspace_bytes,
                                        void* stream, int32_t iters, int32_t* best_config, int32_t* best_slices,
                                        float* best_us) {
  ConvCall cc;
  hidet_status_t st = make_conv_call(cc, in, out, Nb, IC, H, W, OC, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                                     epi);
  if (st != HIDET_OK) return st;
  if (!workspace || workspace_bytes <= 0) return HIDET_ERR_INVALID_ARG;
  SplitK sk;
  sk.workspace = workspace;
  sk.workspace_bytes = workspace_bytes;
  return guarded([&] { return tune_conv(cc, sk, (hipStream_t)stream, iters, best_config, best_slices, best_us); });
}

int32_t hidet_tune_last_times(float* us_per_config, int32_t capacity) {
  std::lock_guard<std::mutex> lock(g_mutex);
  const int n = (int)g_last_times.size();
  if (us_per_config)
    for (int i = 0; i < n && i < capacity; ++i) us_per_config[i] = g_last_times[i];
  return n;
}

void hidet_tune_clear(void) {
  std::lock_guard<std::mutex> lock(g_mutex);
  g_cache.clear();
}

hidet_status_t hidet_tune_save(const char* path) {
  if (!path) return HIDET_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_mutex);
  FILE* f = std::fopen(path, "w");
  if (!f) return HIDET_ERR_INVALID_ARG;
  for (const auto& kv : g_cache)
    std::fprintf(f, "%s %d %d %d\n", kv.first.c_str(), kv.second.config, kv.second.slices, kv.second.route);
  std::fclose(f);
  return HIDET_OK;
}

hidet_status_t hidet_tune_load(const char* path) {
  if (!path) return HIDET_ERR_INVALID_ARG;
  FILE* f = std::fopen(path, "r");
  if (!f) return HIDET_ERR_INVALID_ARG;
  char line[512], key[256];
  const hidet_status_t st = guarded([&] {
    std::lock_guard<std::mutex> lock(g_mutex);
    while (std::fgets(line, sizeof(line), f)) {
      int cfg = 0, slices = 1, route = 0;  // the route is absent from files written before it existed
      if (std::sscanf(line, "%255s %d %d %d", key, &cfg, &slices, &route) < 3) continue;
      if (cfg >= 0 && cfg < kNumConfigs && slices >= 1 && slices <= 1024 && (route == 0 || route == 1))
        g_cache[std::string(key)] = Tuned{cfg, slices, route};
    }
    return HIDET_OK;
  });
  std::fclose(f);
  return st;
}

int32_t hidet_taskmap_count(void) { return kNumTaskMaps; }

hidet_status_t hidet_taskmap_info(int32_t index, char* expr, int32_t expr_capacity, int32_t* workers, int32_t* shape0,
                                  int32_t* shape1, int32_t* tasks_per_worker) {
  if (index < 0 || index >= kNumTaskMaps) return HIDET_ERR_INVALID_ARG;
  const TaskMapEntry& e = kTaskMaps[index];
  if (expr && expr_capacity > 0) {
    std::strncpy(expr, e.expr, (size_t)expr_capacity - 1);
    expr[expr_capacity - 1] = 0;
  }
  if (workers) *workers = e.workers;
  if (shape0) *shape0 = e.shape0;
  if (shape1) *shape1 = e.shape1;
  if (tasks_per_worker) *tasks_per_worker = e.tasks;
  return HIDET_OK;
}

hidet_status_t hidet_taskmap_tasks(int32_t index, int32_t worker, int32_t* tasks_ij, int32_t capacity_pairs) {
  if (index < 0 || index >= kNumTaskMaps || !tasks_ij) return HIDET_ERR_INVALID_ARG;
  const TaskMapEntry& e = kTaskMaps[index];
  if (worker < 0 || worker >= e.workers || capacity_pairs < e.tasks) return HIDET_ERR_INVALID_ARG;
  for (int q = 0; q < e.tasks; ++q) {
    const tmap::Task t = e.task(worker, q);
    tasks_ij[2 * q] = t.i;
    tasks_ij[2 * q + 1] = t.j;
  }
  return HIDET_OK;
}

hidet_status_t hidet_block_task(int32_t tiles_m, int32_t tiles_n, int32_t group, int32_t w, int32_t* tile_i,
                                int32_t* tile_j) {
  if (tiles_m <= 0 || tiles_n <= 0 || group <= 0 || w < 0 || w >= tiles_m * tiles_n || !tile_i || !tile_j)
    return HIDET_ERR_INVALID_ARG;
  const tmap::Task t = tmap::GroupedSpatial{tiles_m, tiles_n, group}.task(w);
  *tile_i = t.i;
  *tile_j = t.j;
  return HIDET_OK;
}

hidet_status_t hidet_host_div(int64_t divisor, int32_t n, int32_t* quotient) {
  if (divisor <= 0 || divisor > kIntMax || n < 0 || !quotient) return HIDET_ERR_INVALID_ARG;
  *quotient = make_fastdiv(divisor).div(n);
  return HIDET_OK;
}

const char* hidet_status_string(int32_t status) {
  switch (status) {
    case HIDET_OK: return "ok";
    case HIDET_ERR_INVALID_ARG: return "invalid argument";
    case HIDET_ERR_UNSUPPORTED: return "unsupported";
    case HIDET_ERR_ALIGNMENT: return "misaligned pointer";
    case HIDET_ERR_NO_CONFIG: return "no applicable tile configuration";
    case HIDET_ERR_LAUNCH: return "kernel launch failed";
    case HIDET_ERR_SCRATCH: return "partial sums exceed the static scratch array";
    default: return "unknown status";
  }
}

const char* hidet_version(void) { return "hidet-mi355x 0.1 (gfx950)"; }

int64_t hidet_kernel_launch_count(void) { return g_kernel_launches; }

}  // extern "C"
