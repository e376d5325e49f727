/*
 * hidet_mi355x.h -- C ABI of the MI355X (gfx950) fused matrix-multiplication library.
 *
 * The library implements the scheduled matrix-multiplication tensor program of the Hidet paper
 * (tiled over M and N into independent workgroup tasks, K tiled inside each workgroup, cooperative
 * loads to on-chip memory, double buffering, matrix-core contraction; Sections 2.2 and 3.1), reused
 * for convolution through the img2col formulation (Sections 5.2 and 6.3.4) and extended by
 * post-scheduling fusion of elementwise prologue/epilogue operators (Sections 4.2 and 5.2).
 *
 * Conventions shared by every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library allocates no device
 *     memory, launches asynchronously on the HIP stream passed as `stream` (a hipStream_t cast to
 *     void*, NULL = the default stream) and never synchronises, except hidet_tune_* which time
 *     kernels and therefore synchronise the stream.
 *   - Matrices are row-major with explicit leading dimensions counted in elements.
 *   - Products of fp16/bf16 inputs are accumulated in fp32; fp32 inputs are multiplied and
 *     accumulated in fp32.  The output is rounded once (nearest-even) to `out` after the epilogue.
 *   - Sizes are arbitrary: tiles that stick out of the problem are handled by predicated loads and
 *     stores (the hardware-centric schedule space of Section 4.3 does not depend on input sizes).
 *   - On any status other than HIDET_OK nothing has been launched and no output byte was written, unless the
 *     status is HIDET_ERR_LAUNCH (the HIP runtime refused a launch) from a call that launches two kernels: a
 *     K-parallel form, whose first kernel writes the workspace only, or a large GEMM cut in two (see
 *     hidet_kernel_launch_count), whose first kernel writes its rows or columns of C.  No C++ exception leaves the library; a failed host allocation is reported as HIDET_ERR_LAUNCH.
 *     M == 0, N == 0 or batch == 0 is an OK no-op; K == 0 writes C = epilogue(0).
 *   - Thread safety: entry points may be called from several host threads; the tuned-config cache
 *     is guarded by a mutex.
 */
#ifndef HIDET_MI355X_H_
#define HIDET_MI355X_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HIDET_OK = 0,
  HIDET_ERR_INVALID_ARG = 1, /* null pointer, negative size, leading dimension too small, bad enum */
  HIDET_ERR_UNSUPPORTED = 2, /* dtype combination, dilation/groups, index range beyond 2^31 elements */
  HIDET_ERR_ALIGNMENT = 3,   /* pointer not aligned to its element size */
  HIDET_ERR_NO_CONFIG = 4,   /* config index out of range, or config not applicable to this problem */
  HIDET_ERR_LAUNCH = 5,      /* the HIP runtime refused the launch */
  HIDET_ERR_SCRATCH = 6      /* hidet_batched_gemm_splitk_static: the partial sums do not fit the static scratch array */
} hidet_status_t;

typedef enum { HIDET_F32 = 0, HIDET_F16 = 1, HIDET_BF16 = 2 } hidet_dtype_t;
typedef enum { HIDET_BIAS_NONE = 0, HIDET_BIAS_PER_COL = 1 /* length N */, HIDET_BIAS_PER_ROW = 2 /* length M */ } hidet_bias_axis_t;
typedef enum { HIDET_ACT_NONE = 0, HIDET_ACT_RELU = 1 } hidet_act_t;
typedef enum { HIDET_MAP_PLAIN = 0, HIDET_MAP_HEAD_SPLIT = 1 } hidet_out_map_t;
typedef enum { HIDET_PROLOGUE_NONE = 0, HIDET_PROLOGUE_RELU = 1 } hidet_prologue_t;

/*
 * Fused epilogue: the elementwise ("bijective") operators that post-scheduling fusion folds into
 * the store of each output element (Section 4.2; Section 5.2 describes how an epilogue rewrites the
 * value and the indices of every output store).  Applied in fp32, in this order:
 *     v = alpha * acc;  v += bias[j] (per col) or bias[i] (per row);  v += residual[i][j];
 *     v = max(v, 0) if act == HIDET_ACT_RELU;  out = round_to_out_dtype(v)
 * bias and residual have the OUTPUT dtype.  residual has the shape of the output and its own
 * leading dimension; in batched calls it advances by batch_stride_residual elements per batch
 * entry, while bias is shared by all batch entries.  A NULL epilogue pointer means identity
 * (alpha = 1, nothing else).  struct_size must be sizeof(hidet_epilogue_t).
 *
 * out_map rewrites the INDEX of every output store (the other half of what an epilogue may do,
 * Section 5.2).  HIDET_MAP_PLAIN: C[i][j] at C + i*ldc + j.  HIDET_MAP_HEAD_SPLIT fuses the
 * reshape + transpose that follows the projection matmuls of a transformer (the
 * reshape-matmul-transpose sub-graph named in Section 3.2): with i = b*map_seq + s and
 * j = h*map_head_dim + f, element (i, j) is stored at [b][h][s][f] of a dense tensor
 * [M/map_seq][N/map_head_dim][map_seq][map_head_dim]; ldc is ignored, residual (if any) is a dense
 * tensor of that same shape, bias still follows the GEMM index (per column j or per row i).
 * Only for hidet_gemm* and batch == 1 (HIDET_ERR_UNSUPPORTED otherwise); map_seq must divide M and
 * map_head_dim must divide N (HIDET_ERR_INVALID_ARG otherwise).
 *
 * prologue is the other direction of post-scheduling fusion (Section 5.2: a fused prologue replaces every access
 * X[i] of an input of the anchor operator by f(X[i])) and travels in this descriptor because it describes the same
 * fused sub-graph.  HIDET_PROLOGUE_RELU applies f(v) = (v < 0 ? 0 : v) to every element of the ACTIVATION operand as
 * it is loaded -- A of the GEMMs, x of the convolution (a ReLU that precedes the matmul / convolution in the
 * network); the weights (B, w) are not touched, padding stays zero.  With it, tile configurations whose loads
 * bypass the registers run their through-registers form.
 */
typedef struct {
  uint32_t struct_size;
  float alpha;
  const void* bias;
  int32_t bias_axis; /* hidet_bias_axis_t */
  int32_t act;       /* hidet_act_t */
  const void* residual;
  int64_t ld_residual;
  int64_t batch_stride_residual;
  int32_t out_map; /* hidet_out_map_t */
  int32_t prologue; /* hidet_prologue_t: fused prologue of the activation operand, see above */
  int64_t map_seq;
  int64_t map_head_dim;
} hidet_epilogue_t;

/*
 * C[M,N] = epilogue( op(A)[M,K] . op(B)[K,N] )            (matmul definition, Section 2.3)
 * transA == 0: A is stored M x K (lda >= K); transA != 0: A is stored K x M (lda >= M).
 * transB == 0: B is stored K x N (ldb >= N); transB != 0: B is stored N x K (ldb >= K).
 * `in` is the dtype of A and B, `out` the dtype of C, bias and residual.  Supported pairs:
 * (F32,F32), (F16,F16), (BF16,BF16), and (F16,F32), (BF16,F32) -- the fp32 accumulators stored without
 * the final rounding, on the configurations that have a K-parallel form (others return
 * HIDET_ERR_NO_CONFIG); any other pair returns HIDET_ERR_UNSUPPORTED.  The convolution takes same-type
 * pairs only.
 * The tile configuration is the cached tuning winner for this problem if hidet_tune_gemm has
 * seen it, otherwise a size-based default.
 * Limits (HIDET_ERR_UNSUPPORTED beyond them): M, N and K are at most 2^31 - 65537 each; the number of
 * elements of A, B and C may exceed 2^31 (offsets are 64-bit), but what an operand spans -- (rows - 1) * ld
 * + cols elements per batch entry, batch * stride over the batch -- stays below 2^47 elements.
 */
hidet_status_t hidet_gemm(int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t M, int64_t N, int64_t K,
                          const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                          const hidet_epilogue_t* epi, void* stream);

/*
 * `batch` independent GEMMs; entry b uses A + b*strideA, B + b*strideB, C + b*strideC (strides in
 * elements; a stride of 0 shares that operand across the batch, not allowed for C).
 */
hidet_status_t hidet_batched_gemm(int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t batch, int64_t M,
                                  int64_t N, int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                                  int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                                  const hidet_epilogue_t* epi, void* stream);

/*
 * y = epilogue( conv2d(x, w) ): NCHW input x[Nb][IC][H][W], OIHW weights w[OC][IC][KH][KW], NCHW
 * output y[Nb][OC][OH][OW], OH = floor((H + 2*pad_h - KH)/stride_h) + 1 (same for OW), all three
 * tensors dense.  Cross-correlation with zero padding, dilation 1, groups 1.  Computed as an
 * implicit GEMM (Sections 5.2 and 6.3.4): GEMM M = OC, GEMM N = Nb*OH*OW (internally Nb*OH*roundup(OW, 8):
 * output rows are padded so that 8 consecutive columns are 8 consecutive pixels), GEMM K = IC*KH*KW; the
 * img2col gather is the fused prologue of the B operand and the NCHW index map is part of the
 * fused epilogue, so no img2col matrix is ever materialised.  In the epilogue, bias (if any) must
 * be HIDET_BIAS_PER_ROW, i.e. one value per output channel, and residual (if any) is a dense
 * tensor of y's shape (ld_residual and batch_stride_residual are ignored).
 * A 1x1 convolution with unit stride and no padding needs no gather (image b of x already is the IC x H*W
 * row-major matrix of the GEMM): without an explicit configuration it runs as the batched GEMM
 * y[b] = w . x[b], weights shared across the batch, unless hidet_tune_conv2d measured the gather form to be
 * faster for this problem; a call with an explicit configuration always runs the gather form.  The results of
 * the two forms agree to rounding (different summation order).
 * Limits (HIDET_ERR_UNSUPPORTED beyond them): x has at most 2^31 - 65537 elements (y may have more),
 * H + 2*pad_h, W + 2*pad_w, KH, KW, stride_h and stride_w are at most 32767, and OC, Nb*OH*roundup(OW, 8)
 * and IC*KH*KW are at most 2^31 - 65537.
 */
hidet_status_t hidet_conv2d_implicit_gemm(int32_t in, int32_t out, int64_t Nb, int64_t IC, int64_t H, int64_t W,
                                          int64_t OC, int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                          int64_t pad_h, int64_t pad_w, const void* x, const void* w, void* y,
                                          const hidet_epilogue_t* epi, void* stream);

/*
 * Same three operations with an explicit tile configuration (index into the schedule space below);
 * config < 0 behaves like the plain entry points.  HIDET_ERR_NO_CONFIG if the configuration cannot
 * run this problem (wrong dtype class).
 */
hidet_status_t hidet_gemm_cfg(int32_t config, int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t M,
                              int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
                              int64_t ldc, const hidet_epilogue_t* epi, void* stream);
hidet_status_t hidet_batched_gemm_cfg(int32_t config, int32_t in, int32_t out, int32_t transA, int32_t transB,
                                      int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                                      int64_t strideA, const void* B, int64_t ldb, int64_t strideB, void* C,
                                      int64_t ldc, int64_t strideC, const hidet_epilogue_t* epi, void* stream);
hidet_status_t hidet_conv2d_implicit_gemm_cfg(int32_t config, int32_t in, int32_t out, int64_t Nb, int64_t IC,
                                              int64_t H, int64_t W, int64_t OC, int64_t KH, int64_t KW,
                                              int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                              const void* x, const void* w, void* y, const hidet_epilogue_t* epi,
                                              void* stream);

/*
 * Hardware-centric schedule space (Section 4.3): a fixed list of tile configurations chosen from
 * what the hardware offers (LDS capacity, registers, wavefronts per workgroup, matrix-core shapes),
 * independent of problem sizes.  Index range: 0 .. hidet_config_count()-1.
 */
typedef struct {
  int32_t block_m, block_n, block_k; /* workgroup tile */
  int32_t waves_m, waves_n;          /* wavefront grid inside the workgroup: spatial(waves_m, waves_n) */
  int32_t mfma;                      /* matrix-core tile edge: 32 (32x32xk) or 16 (16x16xk) */
  int32_t is_f32;                    /* 1: configuration for fp32 inputs, 0: for fp16/bf16 inputs */
  int32_t schedule;                  /* 0: two LDS stages, next tile staged through registers;
                                        1: ring of four stages filled by direct global -> LDS loads, wavefront ping-pong;
                                        2: as 0 with the loads of the next tile issued one iteration earlier;
                                        3: as 2 with sixteen wavefronts, 16 / (waves_m * waves_n) groups that each
                                           multiply a share of the k steps of every K tile (sums meet in LDS) */
  int32_t stages;                    /* LDS stages of block_k each */
  int32_t lds_bytes;                 /* LDS allocated by the workgroup */
  int32_t waves_k;                   /* wave groups that share every K tile (1 except with schedule 3); the workgroup
                                        has waves_m * waves_n * waves_k wavefronts */
} hidet_config_info_t;
int32_t hidet_config_count(void);
hidet_status_t hidet_config_info(int32_t config, hidet_config_info_t* info);

/*
 * Tuning (Section 5.1.3, template-based scheduling): run every applicable configuration of the
 * schedule space on the caller's fused problem (same arguments as the batched GEMM / the conv),
 * time `iters` launches of each with HIP events on `stream`, remember the fastest under a key made
 * of (operation, dtypes, transposes, sizes, epilogue kind) and report it.  The output buffer is
 * overwritten with valid results.  best_config / best_us may be NULL.  Synchronises `stream`.
 * For a 1x1 convolution with unit stride and no padding both forms (gather, batched GEMM) are enumerated and
 * the faster one is remembered; the reported configuration may then belong to the batched-GEMM form, which
 * only a call without an explicit configuration runs.
 */
hidet_status_t hidet_tune_gemm(int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t batch, int64_t M,
                               int64_t N, int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                               int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                               const hidet_epilogue_t* epi, void* stream, int32_t iters, int32_t* best_config,
                               float* best_us);
hidet_status_t hidet_tune_conv2d(int32_t in, int32_t out, int64_t Nb, int64_t IC, int64_t H, int64_t W, int64_t OC,
                                 int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                 int64_t pad_w, const void* x, const void* w, void* y, const hidet_epilogue_t* epi,
                                 void* stream, int32_t iters, int32_t* best_config, float* best_us);
/*
 * Parallel reduction on the K dimension (Section 5.2 and Section 6.3.4: the matrix-multiplication
 * optimisation that the fused convolutions inherit, so that problems with few output tiles still fill
 * the device).  K is cut into `k_slices` contiguous slices of whole K tiles; the grid grows by that
 * factor; every workgroup accumulates one slice of one output tile and writes its fp32 partial tile
 * into `workspace`; a second kernel sums the slices in ascending order in fp32 and applies the whole
 * fused epilogue (alpha, bias, residual, ReLU) once, on the sum, then rounds to the output dtype.
 * Results therefore differ from the unsliced call only by fp32 summation order.
 *
 *   workspace        DEVICE pointer, 16-byte aligned, caller-owned, at least
 *                    hidet_splitk_workspace_bytes(batch, M, N, k_slices) bytes (for the convolution:
 *                    batch = 1, M = OC, N = Nb*OH*roundup(OW, 8): the implicit GEMM pads every output
 *                    row to a multiple of 8 columns); contents on entry ignored, clobbered on return;
 *                    layout [batch][slice][M][N] fp32.  Calls that share a workspace must be ordered
 *                    on one stream.
 *   k_slices         > 1: requested slice count (the effective count may be smaller when K has fewer
 *                    K tiles; with one effective slice the call runs the unsliced kernel and ignores
 *                    the workspace); 1: unsliced; <= 0: take (config, k_slices) remembered by
 *                    hidet_tune_*_splitk for this problem, else unsliced.
 *   config           as for the *_cfg entry points; configurations whose workgroup tile is at most 128x128
 *                    and the ring-schedule configurations have a sliced form, others return
 *                    HIDET_ERR_NO_CONFIG when k_slices > 1.
 *
 * Errors: HIDET_ERR_INVALID_ARG if the workspace is NULL or too small for the effective slice count,
 * HIDET_ERR_ALIGNMENT if it is misaligned, HIDET_ERR_UNSUPPORTED if batch > 65535 with slicing.
 * hidet_splitk_workspace_bytes returns -1 for negative sizes, k_slices < 1 or a size beyond 2^62 bytes.
 */
int64_t hidet_splitk_workspace_bytes(int64_t batch, int64_t M, int64_t N, int32_t k_slices);
hidet_status_t hidet_batched_gemm_splitk(int32_t config, int32_t k_slices, int32_t in, int32_t out, int32_t transA,
                                         int32_t transB, int64_t batch, int64_t M, int64_t N, int64_t K, const void* A,
                                         int64_t lda, int64_t strideA, const void* B, int64_t ldb, int64_t strideB,
                                         void* C, int64_t ldc, int64_t strideC, const hidet_epilogue_t* epi,
                                         void* workspace, int64_t workspace_bytes, void* stream);
hidet_status_t hidet_conv2d_implicit_gemm_splitk(int32_t config, int32_t k_slices, int32_t in, int32_t out, int64_t Nb,
                                                 int64_t IC, int64_t H, int64_t W, int64_t OC, int64_t KH, int64_t KW,
                                                 int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                                 const void* x, const void* w, void* y, const hidet_epilogue_t* epi,
                                                 void* workspace, int64_t workspace_bytes, void* stream);
/*
 * Convolution with repacked weights.  The img2col prologue (Sections 5.2 and 6.3.4) reads, for every element of the
 * GEMM's K axis, a shifted window of the input; with the weights in OIHW order that axis is (ic, kh, kw) and every
 * 16-byte piece of the gather has its own filter tap, padding mask and offset.  Inference weights are constants, so
 * they can be reordered once, like the folding of batch normalisation into them: hidet_conv2d_pack_weights writes
 * w_packed[oc][kh][kw][ic] = w[oc][ic][kh][kw] (same element count, DEVICE buffers, must not overlap, asynchronous on
 * `stream`), and hidet_conv2d_implicit_gemm_packed computes the same convolution as hidet_conv2d_implicit_gemm from
 * x and w_packed with the K axis ordered (kh, kw, ic): a K tile then lies within one filter tap, and mask and spatial
 * offset are worked out once per tile instead of once per piece.  Results agree with the OIHW form to rounding
 * (another summation order).
 *   config, k_slices, workspace: as for hidet_conv2d_implicit_gemm_splitk; workspace may be NULL (then k_slices > 1 is
 *     HIDET_ERR_INVALID_ARG and k_slices <= 0 means unsliced).  A configuration applies only if its block_k divides IC
 *     (HIDET_ERR_NO_CONFIG otherwise; without an explicit configuration a fitting one is chosen).
 *   Restrictions (HIDET_ERR_UNSUPPORTED): IC must be a multiple of 8 (fp32: 4), stride_w at most 2, w_packed 16-byte
 *     aligned, x at least 32 elements; otherwise the limits of hidet_conv2d_implicit_gemm.
 * hidet_tune_conv2d_packed: as hidet_tune_conv2d_splitk for the packed form (workspace may be NULL: tiles only).
 */
hidet_status_t hidet_conv2d_pack_weights(int32_t dtype, int64_t OC, int64_t IC, int64_t KH, int64_t KW, const void* w,
                                         void* w_packed, void* stream);
hidet_status_t hidet_conv2d_implicit_gemm_packed(int32_t config, int32_t k_slices, int32_t in, int32_t out, int64_t Nb,
                                                 int64_t IC, int64_t H, int64_t W, int64_t OC, int64_t KH, int64_t KW,
                                                 int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                                 const void* x, const void* w_packed, void* y, const hidet_epilogue_t* epi,
                                                 void* workspace, int64_t workspace_bytes, void* stream);
hidet_status_t hidet_tune_conv2d_packed(int32_t in, int32_t out, int64_t Nb, int64_t IC, int64_t H, int64_t W, int64_t OC,
                                        int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                        int64_t pad_w, const void* x, const void* w_packed, void* y,
                                        const hidet_epilogue_t* epi, void* workspace, int64_t workspace_bytes, void* stream,
                                        int32_t iters, int32_t* best_config, int32_t* best_slices, float* best_us);
/*
 * Workspace of the K-parallel convolution (Sections 5.2 and 6.3.4: the convolution is the matrix multiplication
 * with GEMM M = OC and GEMM N = Nb*OH*roundup(OW, 8), the padded-row column order of the img2col prologue):
 * bytes that hidet_conv2d_implicit_gemm_splitk needs for an output y[Nb][OC][OH][OW] cut into k_slices.
 * Returns -1 under the conditions of hidet_splitk_workspace_bytes.
 */
int64_t hidet_conv2d_splitk_workspace_bytes(int64_t Nb, int64_t OC, int64_t OH, int64_t OW, int32_t k_slices);
/*
 * hidet_batched_gemm_splitk for callers that cannot allocate device memory or hold a workspace of their own
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the fp32 partial sums go
 * to a static array that is part of the library's code object -- hidet_static_scratch_bytes() = 32 MiB per GPU,
 * held by every GPU the library runs on until the process ends.  The call allocates and frees no device memory
 * (the array's device address is looked up once per device, on the first call with that device current); same
 * kernels, same arguments, same results bit for bit as hidet_batched_gemm_splitk with a workspace of that size.
 * HIDET_ERR_SCRATCH (nothing launched) if 4 * batch * effective_slices * M * N exceeds the array.  Nothing in the
 * array needs clearing between calls: every partial tile element that the second kernel reads has been written by
 * the first.  All calls on one GPU share the one array: calls whose execution may overlap (different streams,
 * or the same stream from different host threads without ordering) race on it; order them on one stream.
 */
int64_t hidet_static_scratch_bytes(void);
hidet_status_t hidet_batched_gemm_splitk_static(int32_t config, int32_t k_slices, int32_t in, int32_t out,
                                                int32_t transA, int32_t transB, int64_t batch, int64_t M, int64_t N,
                                                int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                                                int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                                                const hidet_epilogue_t* epi, void* stream);
/*
 * Tuning over (configuration x k_slices in {1,2,3,4,6,8,12,16}) with the given workspace; slice
 * counts the workspace cannot hold are skipped.  Otherwise as hidet_tune_gemm / hidet_tune_conv2d;
 * the winner is remembered for the *_splitk entry points (k_slices <= 0, config < 0).
 */
hidet_status_t hidet_tune_gemm_splitk(int32_t in, int32_t out, int32_t transA, int32_t transB, int64_t batch, int64_t M,
                                      int64_t N, int64_t K, const void* A, int64_t lda, int64_t strideA, const void* B,
                                      int64_t ldb, int64_t strideB, void* C, int64_t ldc, int64_t strideC,
                                      const hidet_epilogue_t* epi, void* workspace, int64_t workspace_bytes, void* stream,
                                      int32_t iters, int32_t* best_config, int32_t* best_slices, float* best_us);
hidet_status_t hidet_tune_conv2d_splitk(int32_t in, int32_t out, int64_t Nb, int64_t IC, int64_t H, int64_t W,
                                        int64_t OC, int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                        int64_t pad_h, int64_t pad_w, const void* x, const void* w, void* y,
                                        const hidet_epilogue_t* epi, void* workspace, int64_t workspace_bytes,
                                        void* stream, int32_t iters, int32_t* best_config, int32_t* best_slices,
                                        float* best_us);
/* After a hidet_tune_* call: per-configuration mean microseconds of that run (negative = not applicable). */
int32_t hidet_tune_last_times(float* us_per_config, int32_t capacity);
/* Forget every tuned entry. */
void hidet_tune_clear(void);
/* Persist / restore the tuned-config cache as a text file (host paths): one line `key config k_slices form` per
 * problem (form: 1 = batched-GEMM form of a 1x1 convolution, else 0; a line without it reads as 0; malformed or
 * out-of-range lines are skipped).  Returns HIDET_ERR_INVALID_ARG on I/O errors. */
hidet_status_t hidet_tune_save(const char* path);
hidet_status_t hidet_tune_load(const char* path);

/*
 * Reduction template (end of Section 5: next to matrix multiplication, reductions such as a sum along
 * an axis are the only other hand-written schedule template) and the row softmax built on it, which
 * turns the two attention products (scores = alpha * Q.K^T, context = S.V) into attention.
 * x is a row-major [rows][cols] matrix with leading dimension ldx >= cols (elements), DEVICE memory.
 *
 * hidet_reduce_rows: y[i] = sum_j x[i][j] (HIDET_REDUCE_SUM), max_j (HIDET_REDUCE_MAX) or the mean
 *   (HIDET_REDUCE_MEAN); y has `rows` elements of dtype `out`, which is `in` or HIDET_F32
 *   (HIDET_ERR_UNSUPPORTED otherwise).  Accumulation is fp32.  cols == 0 gives 0, -inf and NaN.
 * hidet_softmax_rows: y[i][j] = exp(x[i][j] - m_i) / sum_j exp(x[i][j] - m_i) with m_i = max_j x[i][j],
 *   evaluated in fp32, y of the same dtype and shape with leading dimension ldy >= cols.  y == x
 *   (with ldy == ldx) is allowed; any other overlap is not.  A row of -inf only yields NaN.
 * Both: rows == 0 (softmax: or cols == 0) is an OK no-op; asynchronous on `stream`; no allocation.
 * Limits (HIDET_ERR_UNSUPPORTED beyond them): cols is at most 2^31 - 65, rows * ld at most 2^47 elements.
 */
typedef enum { HIDET_REDUCE_SUM = 0, HIDET_REDUCE_MAX = 1, HIDET_REDUCE_MEAN = 2 } hidet_reduce_op_t;
hidet_status_t hidet_reduce_rows(int32_t in, int32_t out, int32_t op, int64_t rows, int64_t cols, const void* x,
                                 int64_t ldx, void* y, void* stream);
hidet_status_t hidet_softmax_rows(int32_t dtype, int64_t rows, int64_t cols, const void* x, int64_t ldx, void* y,
                                  int64_t ldy, void* stream);

/*
 * Task mappings (Section 5.1): the compile-time mappings the kernels are built from, plus the
 * paper's worked examples, evaluated on the host so that tests can compare them with the
 * definitions.  `expr` receives a string such as "repeat(4,1)*spatial(16,8)".  hidet_taskmap_tasks
 * writes the worker's task list as (i, j) pairs into `tasks_ij` (2 * tasks int32 values).
 */
int32_t hidet_taskmap_count(void);
hidet_status_t hidet_taskmap_info(int32_t index, char* expr, int32_t expr_capacity, int32_t* workers, int32_t* shape0,
                                  int32_t* shape1, int32_t* tasks_per_worker);
hidet_status_t hidet_taskmap_tasks(int32_t index, int32_t worker, int32_t* tasks_ij, int32_t capacity_pairs);
/* Block-level mapping used at launch: tile (i, j) of workgroup `w` for a tiles_m x tiles_n grid with grouping `group`. */
hidet_status_t hidet_block_task(int32_t tiles_m, int32_t tiles_n, int32_t group, int32_t w, int32_t* tile_i,
                                int32_t* tile_j);
/*
 * Test aid for the index arithmetic of the img2col gather and of the output index maps: the kernels divide
 * by quantities fixed at launch (KH*KW, KW, the padded output-row length, OH, sequence length, head
 * dimension) with one multiply and one shift; this evaluates the very same routine on the host.
 * 0 < divisor < 2^31, 0 <= n < 2^31, else HIDET_ERR_INVALID_ARG.
 */
hidet_status_t hidet_host_div(int64_t divisor, int32_t n, int32_t* quotient);

/*
 * Matrix-core ceiling probe (measurement aid, Section 6 style reporting): every wavefront of the GPU
 * issues independent MFMAs of shape `mfma` (16 or 32) back to back on operands read from `sample`
 * (device pointer, >= 4096 bytes of dtype `dtype`; the sustained clock under dense MFMA load depends
 * on the operand values, so pass a piece of the real input).  Reports the sustained TFLOP/s and the
 * average shader clock.  `scratch` is a device buffer of at least hidet_probe_scratch_bytes() bytes,
 * 8-byte aligned, whose contents are overwritten.  Synchronises `stream`.
 */
hidet_status_t hidet_probe_mfma_peak(int32_t dtype, int32_t mfma, const void* sample, int64_t sample_bytes,
                                     void* scratch, int64_t scratch_bytes, void* stream, float* tflops,
                                     float* sclk_mhz);
int64_t hidet_probe_scratch_bytes(void);
/*
 * Launch floor (measurement aid): mean microseconds per launch of `iters` back-to-back launches of an empty
 * kernel on `stream` -- what any kernel on this machine costs before it does anything; the small workloads
 * are reported next to it.  Synchronises `stream`.  HIDET_ERR_INVALID_ARG for iters <= 0 or a NULL result.
 */
hidet_status_t hidet_probe_launch_floor(void* stream, int32_t iters, float* us_per_launch);
/*
 * Streaming rate of a plain kernel (measurement aid): GB/s that a kernel which only reads (mode 0), only writes
 * (mode 1) or copies (mode 2, bytes read + bytes written) sustains on memory that no cache holds -- the ceiling the
 * memory-bound workloads are reported against beside the datasheet's 8 TB/s.  `buffer`: DEVICE memory of `bytes`
 * bytes, 16-byte aligned, contents overwritten; it is walked in pieces of 128 MiB (48 launches), so 1 GiB or more
 * keeps every piece out of the 256 MB Infinity Cache; at least 256 MiB.  Synchronises `stream`.
 * HIDET_ERR_INVALID_ARG for a NULL pointer, an unknown mode or fewer than two pieces, HIDET_ERR_ALIGNMENT for a
 * misaligned buffer.
 */
hidet_status_t hidet_probe_stream_bandwidth(void* buffer, int64_t bytes, int32_t mode, void* stream,
                                            float* gbytes_per_s);

const char* hidet_status_string(int32_t status);
/* Library version string and the GPU architecture the kernels were compiled for ("gfx950"). */
const char* hidet_version(void);
/*
 * Number of GEMM / convolution kernels the calling thread has launched through this library so far (a call launches
 * one; two when K is sliced -- partial sums, then reduce + epilogue; two when a large GEMM for which the caller
 * named no configuration is cut into the tile rows that fill whole rounds of the compute units and the rest).  Measurement and test aid; never fails.
 */
int64_t hidet_kernel_launch_count(void);

#ifdef __cplusplus
}
#endif
#endif /* HIDET_MI355X_H_ */
