"""Parity of the HIP path against the CPU oracle, element by element (relative Frobenius error)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

from helpers import (TOL, TORCH_DTYPE, applicable_configs, assert_elementwise, bias_axis_code, make_conv_workspace, make_workspace, run_conv_case, run_gemm_case, sliceable_configs,
                     to_f64, to_gpu, within_bound)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ the benchmark configurations
def test_config1_fp32_256():
    (c,) = wl.config1()
    err, _, _ = run_gemm_case(c)
    _say("cfg1 err %.3e" % err)
    assert err <= TOL["f32"]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_config2_transformer_mlp(dtype):
    for c in wl.config2(dtype):
        err, _, _ = run_gemm_case(c)
        _say("%s %s err %.3e" % (c["name"], dtype, err))
        assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_config3_resnet50_convs(dtype):
    for c in wl.config3(dtype):
        err, _, _ = run_conv_case(c)
        _say("%s %s err %.3e" % (c["name"], dtype, err))
        assert err <= TOL[dtype]


@pytest.mark.parametrize("case", range(4))
def test_config4_attention_products(case):
    """All four cases of the benchmark configuration (batch x heads in {12, 192}, seq in {128, 512}), the very
    tensors bench.py's side report times (workloads.config4: seeds 4000 + case), untuned launch configuration;
    every batch entry as a tensor of its own, the whole batch as one, and every element on its own."""
    c = wl.config4("f16")[case]
    batch, seq = c["batch"], c["seq"]
    Q, K, V, S = (to_gpu(c[k], "f16") for k in ("Q", "K", "V", "S"))
    scores = torch.full((batch, seq, seq), float("nan"), dtype=torch.float16, device="cuda")
    hb.hidet_batched_gemm(Q, K, scores, transB=True, epilogue=hb.make_epilogue(alpha=c["alpha"]))
    ctx = torch.full((batch, seq, c["d"]), float("nan"), dtype=torch.float16, device="cuda")
    hb.hidet_batched_gemm(S, V, ctx)
    torch.cuda.synchronize()
    Q64, K64, S64, V64 = (wl.widen(c[k], "f16") for k in ("Q", "K", "S", "V"))
    ref_s = oracle.batched_gemm(Q64, K64, transB=True, alpha=c["alpha"])
    ref_c = oracle.batched_gemm(S64, V64)
    got_s, got_c = to_f64(scores), to_f64(ctx)
    worst = max(max(oracle.rel_frobenius(got_s[b], ref_s[b]) for b in range(batch)), oracle.rel_frobenius(got_s, ref_s),
                max(oracle.rel_frobenius(got_c[b], ref_c[b]) for b in range(batch)), oracle.rel_frobenius(got_c, ref_c))
    _say("cfg4 b%d s%d worst err %.3e" % (batch, seq, worst))
    assert worst <= TOL["f16"]
    nq, nk = np.sqrt((Q64 * Q64).sum(-1)), np.sqrt((K64 * K64).sum(-1))
    assert_elementwise(got_s, ref_s, c["alpha"] * nq[:, :, None] * nk[:, None, :], "f16", c["d"], "cfg4 scores")
    ns, nv = np.sqrt((S64 * S64).sum(-1)), np.sqrt((V64 * V64).sum(-2))
    assert_elementwise(got_c, ref_c, ns[:, :, None] * nv[:, None, :], "f16", seq, "cfg4 context")


# ------------------------------------------------------------------ sizes that are not multiples of anything
ODD = [(1, 1, 1), (1, 17, 5), (17, 1, 33), (31, 33, 7), (127, 129, 65), (257, 63, 130), (64, 64, 64), (200, 300, 72)]


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, False), (True, True)])
def test_odd_shapes(dtype, transA, transB):
    for i, (M, N, K) in enumerate(ODD):
        c = wl.gemm_case(7000 + i, M, N, K, dtype, transA=transA, transB=transB, bias="col", residual=(i % 2 == 0))
        err, _, ref = run_gemm_case(c, relu=(i % 3 == 0), alpha=0.5)
        _say("odd %s tA%d tB%d %dx%dx%d err %.3e" % (dtype, transA, transB, M, N, K, err))
        assert within_bound(err, ref, dtype), (M, N, K)


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_padded_leading_dimensions_keep_vector_loads(dtype):
    # leading dimensions that are multiples of 16 bytes but larger than the rows: the vector path with K and N tails
    c = wl.gemm_case(7100, 150, 203, 77, dtype, bias="row", lda_pad=83 - 77 + 5, ldb_pad=5)
    assert c["lda"] % 8 == 0 and c["ldb"] % 8 == 0
    err, _, _ = run_gemm_case(c, relu=True)
    assert err <= TOL[dtype]


def test_prime_size_2039():
    # the size on which input-centric schedule spaces have no valid schedule (Section 3.3)
    c = wl.gemm_case(7200, 2039, 2039, 2039, "f16", bias="col")
    err, _, _ = run_gemm_case(c, relu=True)
    _say("2039^3 err %.3e" % err)
    assert err <= TOL["f16"]


# ------------------------------------------------------------------ every configuration of the schedule space
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_every_config_on_an_odd_shape(dtype):
    for cfg in applicable_configs(dtype):
        for tB in (False, True):
            c = wl.gemm_case(7300 + cfg, 283, 331, 203, dtype, transB=tB, bias="col", residual=True)
            err, _, _ = run_gemm_case(c, config=cfg, relu=True, alpha=0.75)
            _say("config %d %s tB%d err %.3e" % (cfg, dtype, tB, err))
            assert err <= TOL[dtype], cfg
        # aligned variant (vector loads) of the same configuration
        c = wl.gemm_case(7400 + cfg, 264, 328, 200, dtype, bias="row")
        err, _, _ = run_gemm_case(c, config=cfg)
        assert err <= TOL[dtype], cfg


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_ring_schedules_every_stage_count(dtype):
    """The ring schedules (direct global -> LDS loads, on aligned and on element-aligned operands) fill and drain a
    ring of four stages: K values that give 0, 1, 2, 3, 4, 5 and 9 full stages, each with and without a partial last
    stage, on every ring configuration.  Element-aligned rows come from an odd K (row-major A, transposed B) and,
    with K a whole number of stages, from odd M and N (row-major B, transposed A, the output)."""
    ring = [i for i in applicable_configs(dtype) if hb.hidet_config_info(i)["schedule"] == 1]
    assert ring
    ran_trans_a = 0
    for cfg in ring:
        bk = hb.hidet_config_info(cfg)["block_k"]
        for stages in (0, 1, 2, 3, 4, 5, 9):
            for tail in (0, 8, 13):
                K = stages * bk + tail
                if K == 0:
                    continue
                for odd in ((False, True) if tail % 8 == 0 else (True,)):
                    M, N = (263, 517) if odd else (264, 520)  # odd sizes: element-aligned rows
                    for tA, tB in ((False, False), (False, True), (True, False), (True, True)):
                        if tA and (stages not in (1, 4) or tail == 8):
                            continue  # the transposed-A forms on a few stage counts only
                        c = wl.gemm_case(7450 + cfg, M, N, K, dtype, transA=tA, transB=tB, bias="col")
                        try:
                            err, _, ref = run_gemm_case(c, config=cfg, relu=True)
                        except hb.HidetError as e:
                            assert tA and e.status == 4, (cfg, stages, tail, tA, tB, e)  # tile built without transposed A
                            continue
                        ran_trans_a += int(tA)
                        assert within_bound(err, ref, dtype), (cfg, stages, tail, odd, tA, tB, err)
    assert ran_trans_a > 0
    _say("ring configurations %s: all stage counts pass (%s)" % (ring, dtype))


def test_ring_schedule_on_offset_pointers_and_padded_rows():
    """Element alignment from the pointers alone: operands and output that start one element into their buffers, with
    leading dimensions larger than the rows, on the 256x256 ring tile; K spans whole stages and a tail."""
    cfg = next(i for i in applicable_configs("f16")
               if hb.hidet_config_info(i)["schedule"] == 1 and hb.hidet_config_info(i)["block_m"] == 256
               and hb.hidet_config_info(i)["block_n"] == 256 and hb.hidet_config_info(i)["mfma"] == 16)
    for M, N, K in ((300, 520, 128), (257, 263, 167), (512, 256, 96)):
        c = wl.gemm_case(7470 + K, M, N, K, "f16", bias="col", lda_pad=16, ldb_pad=24)
        bufA = torch.zeros(M * c["lda"] + 1, dtype=torch.float16, device="cuda")
        bufB = torch.zeros(K * c["ldb"] + 1, dtype=torch.float16, device="cuda")
        bufC = torch.full((M * (N + 9) + 1,), float("nan"), dtype=torch.float16, device="cuda")
        A = bufA[1:].view(M, c["lda"])
        B = bufB[1:].view(K, c["ldb"])
        A.copy_(to_gpu(c["A"], "f16"))
        B.copy_(to_gpu(c["B"], "f16"))
        C = bufC[1:].view(M, N + 9)[:, :N]
        bias = to_gpu(c["bias"], "f16")
        hb.hidet_gemm(A[:, :K], B[:, :N], C, epilogue=hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True),
                      config=cfg)
        torch.cuda.synchronize()
        A64, B64 = wl.widen(c["A"], "f16")[:, :K], wl.widen(c["B"], "f16")[:, :N]
        ref = oracle.gemm(A64, B64, bias=wl.widen(c["bias"], "f16"), bias_axis=oracle.BIAS_PER_COL, relu=True)
        got = to_f64(C)
        err = oracle.rel_frobenius(got, ref)
        assert within_bound(err, ref, "f16"), (M, N, K, err)
        # what lies between the rows of the output, and before it, is untouched
        whole = bufC[1:].view(M, N + 9)
        assert torch.isnan(whole[:, N:]).all() and torch.isnan(bufC[0])


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_every_config_conv(dtype):
    for cfg in applicable_configs(dtype):
        c = wl.conv_case(7500 + cfg, 2, 5, 11, 9, 7, 3, 3, 2, 1, dtype, residual=True)
        c.update(relu=True)
        err, _, _ = run_conv_case(c, config=cfg)
        _say("conv config %d %s err %.3e" % (cfg, dtype, err))
        assert err <= TOL[dtype], cfg


# ------------------------------------------------------------------ epilogue flags, all 8 combinations
@pytest.mark.parametrize("flags", range(8))
def test_epilogue_flag_combinations(flags):
    c = wl.gemm_case(7600 + flags, 96, 136, 72, "f16", bias="col" if flags & 1 else None, residual=bool(flags & 2))
    err, got, _ = run_gemm_case(c, relu=bool(flags & 4), alpha=1.0 if flags < 4 else 0.125)
    assert err <= TOL["f16"]
    if flags & 4:
        assert got.min() >= 0.0


def test_identity_epilogue_and_closed_forms():
    # all-ones contraction: every output equals K exactly (fp16 holds 1..2048 exactly)
    for K in (1, 64, 100, 2048):
        A = torch.ones((70, K), dtype=torch.float16, device="cuda")
        B = torch.ones((K, 90), dtype=torch.float16, device="cuda")
        C = torch.zeros((70, 90), dtype=torch.float16, device="cuda")
        hb.hidet_gemm(A, B, C)
        assert torch.all(C == K)
    eye = torch.eye(96, dtype=torch.float32, device="cuda")
    X = torch.randn(96, 96, device="cuda")
    C = torch.zeros_like(X)
    hb.hidet_gemm(X, eye, C)
    assert torch.equal(C, X)


# ------------------------------------------------------------------ convolution prologue variants
CONVS = [
    # Nb, IC, H, W, OC, KH, KW, stride, pad
    (1, 3, 8, 8, 4, 1, 1, 1, 0),
    (1, 8, 14, 14, 16, 3, 3, 1, 1),
    (2, 16, 9, 7, 5, 3, 3, 2, 1),
    (3, 4, 12, 12, 9, 5, 5, 1, 2),
    (1, 256, 28, 28, 32, 3, 3, 2, 1),  # the strided layer of the paper's schedule-space study (fewer output channels)
    (2, 7, 10, 10, 3, 2, 2, 2, 0),
]


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_conv_shapes(dtype):
    for i, (Nb, IC, H, W, OC, KH, KW, s, p) in enumerate(CONVS):
        c = wl.conv_case(7700 + i, Nb, IC, H, W, OC, KH, KW, s, p, dtype, residual=(i % 2 == 1))
        c.update(relu=(i % 2 == 0))
        err, _, _ = run_conv_case(c)
        _say("conv %s %s err %.3e" % (dtype, CONVS[i], err))
        assert err <= TOL[dtype], CONVS[i]


def test_conv_rectangular_stride_and_padding():
    c = wl.conv_case(7800, 2, 6, 13, 10, 8, 3, 2, (2, 1), (0, 1), "f16")
    c.update(relu=True)
    err, _, _ = run_conv_case(c)
    assert err <= TOL["f16"]


def test_case_study_strided_conv_and_larger_batches():
    # the layer of the schedule-space case study (Section 6.3.1): 28x28, 256 channels, 3x3, padding 1, stride 2
    c = wl.conv_case(7700, 1, 256, 28, 28, 256, 3, 3, 2, 1, "f16")
    c.update(relu=True)
    err, _, ref = run_conv_case(c)
    _say("case-study conv err %.3e" % err)
    assert ref.shape == (1, 256, 14, 14) and err <= TOL["f16"]
    err, _, _ = run_conv_case(c, k_slices=4, config=sliceable_configs("f16")[0])
    assert err <= TOL["f16"]
    # batch sizes 4 and 8 (Section 6.3.3) on a bottleneck 3x3 and a 1x1 layer
    for nb in (4, 8):
        for (ic, hw, oc, k, s_, p_) in ((64, 28, 64, 3, 1, 1), (128, 14, 256, 1, 1, 0)):
            c = wl.conv_case(7710 + nb + k, nb, ic, hw, hw, oc, k, k, s_, p_, "f16", residual=True)
            c.update(relu=True)
            err, _, _ = run_conv_case(c)
            _say("batch %d conv k%d err %.3e" % (nb, k, err))
            assert err <= TOL["f16"]


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_conv_gather_windows(dtype):
    """Shapes chosen for the whole-chunk gather: output rows shorter than, equal to and just above one chunk, input
    rows narrower than a chunk, wide padding (pixels left and right of the row), strides 1, 2 and 3, several images
    (the first and the last pixels of the tensor are where a window would leave the allocation)."""
    cases = [  # Nb, IC, H, W, OC, KH, KW, stride, pad
        (1, 3, 7, 7, 5, 3, 3, 1, 1), (2, 4, 9, 9, 6, 3, 3, 1, 1), (1, 2, 8, 8, 4, 1, 1, 1, 0), (3, 2, 5, 3, 4, 3, 3, 1, 1),
        (1, 3, 12, 12, 4, 5, 5, 1, 2), (2, 3, 6, 20, 4, 3, 7, 1, 3), (1, 2, 4, 4, 3, 3, 3, 1, 2), (2, 3, 15, 15, 4, 3, 3, 2, 1),
        (1, 4, 16, 16, 4, 1, 1, 2, 0), (1, 2, 9, 30, 3, 3, 3, 2, 0), (1, 3, 17, 17, 4, 5, 5, 3, 2), (1, 1, 2, 2, 1, 1, 1, 1, 0),
        (1, 1, 1, 9, 2, 1, 3, 1, 1), (2, 2, 3, 17, 3, 3, 3, (1, 2), (1, 0)), (1, 2, 11, 11, 3, 3, 3, (2, 1), (0, 2)),
    ]
    for i, (Nb, IC, H, W, OC, KH, KW, st, pd) in enumerate(cases):
        c = wl.conv_case(7720 + i, Nb, IC, H, W, OC, KH, KW, st, pd, dtype, residual=bool(i % 2))
        c.update(relu=bool(i % 3))
        err, _, ref = run_conv_case(c)
        assert within_bound(err, ref, dtype), (i, err)
        err, _, ref = run_conv_case(c, k_slices=2, config=sliceable_configs(dtype)[i % 3])
        assert within_bound(err, ref, dtype), (i, err)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_pointwise_convolutions_in_both_forms(dtype):
    """A 1x1, stride-1, unpadded convolution runs as a batched GEMM (weights shared over the batch) when no
    configuration is named and through the gather when one is: both against the oracle, unsliced and K-sliced,
    image sizes that allow 16-byte rows and sizes that do not, then once more after tuning has chosen between them."""
    cases = [(2, 64, 16, 24, 96), (3, 40, 7, 7, 72), (1, 33, 14, 14, 50), (4, 128, 28, 28, 64), (2, 17, 5, 9, 3),
             (1, 8, 1, 1, 5), (5, 1, 3, 3, 1)]
    hb.hidet_tune_clear()
    for i, (Nb, IC, H, W, OC) in enumerate(cases):
        c = wl.conv_case(7750 + i, Nb, IC, H, W, OC, 1, 1, 1, 0, dtype, residual=bool(i % 2))
        c.update(relu=bool((i + 1) % 3), alpha=[1.0, 0.5][i % 2])
        _say("pointwise %s case %d: %dx%dx%dx%d -> %d" % (dtype, i, Nb, IC, H, W, OC))
        err_g, got_g, ref = run_conv_case(c)  # batched-GEMM form
        assert within_bound(err_g, ref, dtype), (i, err_g)
        err_c, got_c, _ = run_conv_case(c, config=applicable_configs(dtype)[i % 5])  # gather form
        assert within_bound(err_c, ref, dtype), (i, err_c)
        assert oracle.rel_frobenius(got_g, got_c) <= 2 * TOL[dtype] + 1e-5 or ref.size < 64
        err, _, _ = run_conv_case(c, k_slices=3)
        assert within_bound(err, ref, dtype), (i, err)
        err, _, _ = run_conv_case(c, k_slices=2, config=sliceable_configs(dtype)[i % 3])
        assert within_bound(err, ref, dtype), (i, err)
    # the tuner enumerates both forms and the remembered choice is what an unnamed configuration then runs
    c = wl.conv_case(7760, 4, 128, 28, 28, 64, 1, 1, 1, 0, dtype)
    c.update(relu=True)
    x, w, bias = to_gpu(c["x"], dtype), to_gpu(c["w"], dtype), to_gpu(c["bias"], dtype)
    y = torch.empty((4, 64, 28, 28), dtype=TORCH_DTYPE[dtype], device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
    cfg, us = hb.hidet_tune_conv2d(x, w, y, epilogue=epi, iters=3)
    times = [t for t in hb.hidet_tune_last_times() if t > 0]
    assert cfg in applicable_configs(dtype) and us > 0 and abs(us - min(times)) <= 1e-3 * us
    err, _, ref = run_conv_case(c)
    assert within_bound(err, ref, dtype), err
    ws = make_conv_workspace(y.shape, 16)
    cfg, slices, us = hb.hidet_tune_conv2d_splitk(x, w, y, ws, epilogue=epi, iters=3)
    assert slices >= 1 and us > 0
    y.fill_(float("nan"))
    hb.hidet_conv2d_implicit_gemm_splitk(x, w, y, ws, k_slices=0, epilogue=epi)  # the remembered (form, tile, slices)
    torch.cuda.synchronize()
    err = oracle.rel_frobenius(to_f64(y), ref)
    assert within_bound(err, ref, dtype), err
    hb.hidet_tune_clear()


# ------------------------------------------------------------------ output index map (reshape-matmul-transpose)
@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_head_split_output_map(dtype):
    for seed, (b, seq, heads, d), kw in ((7800, (2, 48, 3, 20), dict(bias="col")),       # d % 4 == 0: vector stores
                                         (7801, (3, 17, 5, 10), dict(residual=True)),    # scalar stores, odd sizes
                                         (7802, (1, 128, 12, 64), dict(bias="col"))):    # a BERT-base projection
        M, N, K = b * seq, heads * d, 72 if seed != 7802 else 768
        c = wl.gemm_case(seed, M, N, K, dtype, **kw)
        A, B = to_gpu(c["A"], dtype), to_gpu(c["B"], dtype)
        bias, res = to_gpu(c["bias"], dtype), to_gpu(c["residual"], dtype)
        if res is not None:  # the residual has the shape of the stored tensor
            res = res.view(b, seq, heads, d).permute(0, 2, 1, 3).contiguous()
        ref = oracle.gemm(wl.widen(c["A"], dtype), wl.widen(c["B"], dtype),
                          bias=None if c["bias"] is None else wl.widen(c["bias"], dtype),
                          residual=None if c["residual"] is None else wl.widen(c["residual"], dtype), relu=True)
        ref = oracle.head_split(ref, seq, d)
        epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, residual=res, relu=True, head_split=(seq, d))
        for cfg in (-1, applicable_configs(dtype)[-1]):
            C = torch.full((b, heads, seq, d), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
            hb.hidet_gemm(A, B, C, epilogue=epi, config=cfg)
            torch.cuda.synchronize()
            err = oracle.rel_frobenius(to_f64(C), ref)
            _say("head split %s %s config %d err %.3e" % (dtype, (b, seq, heads, d), cfg, err))
            assert err <= TOL[dtype]
        # the same map applied by the reduce pass of the K-parallel form
        C = torch.full((b, heads, seq, d), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
        hb.hidet_batched_gemm_splitk(A, B, C.view(M, N), make_workspace(1, M, N, 2), k_slices=2, epilogue=epi,
                                     config=sliceable_configs(dtype)[0])
        torch.cuda.synchronize()
        assert oracle.rel_frobenius(to_f64(C), ref) <= TOL[dtype]


# ------------------------------------------------------------------ degenerate cases and argument checking on the device
def test_empty_and_k0():
    A = torch.zeros((0, 8), dtype=torch.float16, device="cuda")
    B = torch.zeros((8, 5), dtype=torch.float16, device="cuda")
    C = torch.zeros((0, 5), dtype=torch.float16, device="cuda")
    hb.hidet_gemm(A, B, C)  # no-op
    # K = 0: C = epilogue(0)
    bias = torch.tensor([1.0, -2.0, 3.0], dtype=torch.float16, device="cuda")
    C = torch.full((4, 3), float("nan"), dtype=torch.float16, device="cuda")
    hb.hidet_gemm(torch.zeros((4, 0), dtype=torch.float16, device="cuda"),
                  torch.zeros((0, 3), dtype=torch.float16, device="cuda"), C,
                  epilogue=hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True))
    torch.cuda.synchronize()
    assert torch.equal(C.cpu(), torch.tensor([[1.0, 0.0, 3.0]] * 4, dtype=torch.float16))


def test_output_outside_the_problem_is_untouched():
    c = wl.gemm_case(7900, 45, 51, 40, "f16")
    A, B = to_gpu(c["A"], "f16"), to_gpu(c["B"], "f16")
    big = torch.full((64, 64), 7.0, dtype=torch.float16, device="cuda")
    hb.hidet_gemm(A, B, big[:45, :51])
    torch.cuda.synchronize()
    assert torch.all(big[45:, :] == 7.0) and torch.all(big[:, 51:] == 7.0)
    ref = oracle.gemm(wl.widen(c["A"], "f16"), wl.widen(c["B"], "f16"))
    assert oracle.rel_frobenius(to_f64(big[:45, :51]), ref) <= TOL["f16"]


def test_misaligned_pointers_use_element_loads():
    c = wl.gemm_case(7950, 65, 70, 50, "f16")
    buf_a = torch.zeros(65 * 50 + 1, dtype=torch.float16, device="cuda")
    buf_b = torch.zeros(50 * 70 + 3, dtype=torch.float16, device="cuda")
    buf_c = torch.zeros(65 * 70 + 1, dtype=torch.float16, device="cuda")
    A = buf_a[1:].view(65, 50)
    B = buf_b[3:].view(50, 70)
    C = buf_c[1:].view(65, 70)
    A.copy_(to_gpu(c["A"], "f16"))
    B.copy_(to_gpu(c["B"], "f16"))
    hb.hidet_gemm(A, B, C)
    torch.cuda.synchronize()
    ref = oracle.gemm(wl.widen(c["A"], "f16"), wl.widen(c["B"], "f16"))
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL["f16"]


def test_batched_with_shared_operand_and_residual():
    g = wl.rng(8000)
    A = wl.normal(g, (5, 33, 40), "f16")
    B = wl.normal(g, (40, 29), "f16")  # shared by the batch (stride 0)
    R = wl.normal(g, (5, 33, 29), "f16")
    dA, dB, dR = to_gpu(A, "f16"), to_gpu(B, "f16"), to_gpu(R, "f16")
    C = torch.zeros((5, 33, 29), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(residual=dR, relu=True, batched=True)
    hb.hidet_batched_gemm(dA, dB.unsqueeze(0).expand(5, 40, 29), C, epilogue=epi)
    torch.cuda.synchronize()
    ref = oracle.batched_gemm(wl.widen(A, "f16"), np.broadcast_to(wl.widen(B, "f16"), (5, 40, 29)),
                              residual=wl.widen(R, "f16"), relu=True)
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL["f16"]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_fp32_output_from_16_bit_inputs(dtype):
    """The accumulators stored without the final rounding: bias and residual are fp32 too, and the error against the
    oracle is that of the fp32 accumulation alone."""
    g = wl.rng(8060)
    for (M, N, K, tB) in ((150, 203, 333, False), (64, 136, 1024, True)):
        c = wl.gemm_case(8061 + M, M, N, K, dtype, transB=tB)
        A, B = to_gpu(c["A"], dtype), to_gpu(c["B"], dtype)
        Av, Bv = A[:, :K], (B[:, :K] if tB else B[:, :N])
        bias = torch.from_numpy(g.standard_normal(N).astype(np.float32)).cuda()
        res = torch.from_numpy(g.standard_normal((M, N)).astype(np.float32)).cuda()
        A64, B64 = wl.widen(c["A"], dtype)[:, :K], (wl.widen(c["B"], dtype)[:, :K] if tB else wl.widen(c["B"], dtype)[:, :N])
        ref = oracle.gemm(A64, B64, transB=tB, alpha=0.5, bias=bias.cpu().double().numpy(),
                          residual=res.cpu().double().numpy(), relu=True)
        epi = hb.make_epilogue(alpha=0.5, bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, residual=res, relu=True)
        for cfg in [-1] + sliceable_configs(dtype):
            C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
            hb.hidet_gemm(Av, Bv, C, transB=tB, epilogue=epi, config=cfg)
            torch.cuda.synchronize()
            err = oracle.rel_frobenius(to_f64(C), ref)
            assert err <= 1e-5, (cfg, err)
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        hb.hidet_batched_gemm_splitk(Av, Bv, C, make_workspace(1, M, N, 3), k_slices=3, transB=tB, epilogue=epi,
                                     config=sliceable_configs(dtype)[0])
        torch.cuda.synchronize()
        assert oracle.rel_frobenius(to_f64(C), ref) <= 1e-5
        big = [i for i in applicable_configs(dtype) if i not in sliceable_configs(dtype)][0]
        with pytest.raises(hb.HidetError):
            hb.hidet_gemm(Av, Bv, C, transB=tB, epilogue=epi, config=big)


def test_calls_run_on_the_stream_they_are_given():
    """Work queued on a side stream must be ordered with the library's kernels on that stream, not on the default one:
    the operands are produced on the side stream right before the call and consumed right after it."""
    c = wl.gemm_case(8050, 300, 200, 520, "f16")
    hostA, hostB = to_gpu(c["A"], "f16"), to_gpu(c["B"], "f16")
    ref = oracle.gemm(wl.widen(c["A"], "f16"), wl.widen(c["B"], "f16"))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for _ in range(5):
            A = torch.zeros_like(hostA)
            B = torch.zeros_like(hostB)
            C = torch.full((300, 200), float("nan"), dtype=torch.float16, device="cuda")
            A.copy_(hostA, non_blocking=True)
            B.copy_(hostB, non_blocking=True)
            hb.hidet_gemm(A, B, C, stream=side)
            out = C.double()  # consumer on the same stream
        side.synchronize()
    assert oracle.rel_frobenius(out.cpu().numpy(), ref) <= TOL["f16"]


# ------------------------------------------------------------------ tuning
def test_tuner_enumerates_the_space_and_caches(tmp_path):
    c = wl.gemm_case(8100, 128, 768, 256, "f16", bias="col")
    A, B, bias = to_gpu(c["A"], "f16"), to_gpu(c["B"], "f16"), to_gpu(c["bias"], "f16")
    C = torch.zeros((128, 768), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True)
    hb.hidet_tune_clear()
    best, us = hb.hidet_tune_gemm(A, B, C, epilogue=epi, iters=5)
    times = hb.hidet_tune_last_times()
    ok = [i for i, t in enumerate(times) if t > 0]
    assert sorted(ok) == applicable_configs("f16")
    assert best in ok and abs(times[best] - us) < 1e-3 and us == min(times[i] for i in ok)
    ref = oracle.gemm(wl.widen(c["A"], "f16"), wl.widen(c["B"], "f16"), bias=wl.widen(c["bias"], "f16"), relu=True)
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL["f16"]
    path = str(tmp_path / "tuned.txt")
    hb.hidet_tune_save(path)
    text = open(path).read()
    assert "gemm:t1:00:b1:128x768x256" in text and text.strip().endswith("%d 1 0" % best)
    hb.hidet_tune_clear()
    hb.hidet_tune_load(path)
    C.zero_()
    hb.hidet_gemm(A, B, C, epilogue=epi)
    torch.cuda.synchronize()
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL["f16"]


# ------------------------------------------------------------------ parallel reduction on K
@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_splitk_every_sliceable_config(dtype):
    cfgs = sliceable_configs(dtype)
    assert cfgs
    for cfg in cfgs:
        for tB, slices in ((False, 2), (True, 5)):
            # ragged everything: K = 1203 leaves a short last slice and a partial K tile inside it
            c = wl.gemm_case(8200 + cfg, 155, 203, 1203, dtype, transB=tB, bias="col", residual=True)
            err, _, _ = run_gemm_case(c, config=cfg, relu=True, alpha=0.75, k_slices=slices)
            _say("splitk config %d %s tB%d slices %d err %.3e" % (cfg, dtype, tB, slices, err))
            assert err <= TOL[dtype], cfg
        c = wl.gemm_case(8300 + cfg, 136, 200, 1024, dtype, bias="row")  # aligned: vector loads and stores
        err, _, _ = run_gemm_case(c, config=cfg, k_slices=4)
        assert err <= TOL[dtype], cfg


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_splitk_conv_every_sliceable_config(dtype):
    for cfg in sliceable_configs(dtype):
        c = wl.conv_case(8400 + cfg, 2, 37, 11, 9, 7, 3, 3, 2, 1, dtype, residual=True)  # K = 333
        c.update(relu=True)
        err, _, _ = run_conv_case(c, config=cfg, k_slices=3)
        _say("splitk conv config %d %s err %.3e" % (cfg, dtype, err))
        assert err <= TOL[dtype], cfg
    c = wl.conv_case(8450, 1, 64, 14, 14, 32, 3, 3, 1, 1, dtype)  # aligned weights: vector loads on A
    c.update(relu=True)
    for slices in (2, 8):
        err, _, _ = run_conv_case(c, config=sliceable_configs(dtype)[0], k_slices=slices)
        assert err <= TOL[dtype]


def test_splitk_transposed_a_and_default_config():
    for tA, tB in ((True, False), (True, True)):
        c = wl.gemm_case(8500, 72, 88, 900, "f16", transA=tA, transB=tB, residual=True)
        err, _, _ = run_gemm_case(c, k_slices=6)  # config -1: nothing tuned, the default tile must be sliceable or refuse
        assert err <= TOL["f16"]


def test_splitk_is_exact_on_integer_data_and_equals_the_unsliced_result():
    """Small integers: every partial sum is exact in fp32, so slicing K cannot change a single bit."""
    g = np.random.default_rng(8600)
    A = torch.from_numpy(g.integers(-3, 4, (96, 1536)).astype(np.float32)).cuda()
    B = torch.from_numpy(g.integers(-3, 4, (1536, 80)).astype(np.float32)).cuda()
    exact = (A.double().cpu() @ B.double().cpu())
    cfg = sliceable_configs("f32")[0]
    for slices in (1, 2, 7, 16):
        C = torch.full((96, 80), float("nan"), dtype=torch.float32, device="cuda")
        hb.hidet_batched_gemm_splitk(A, B, C, make_workspace(1, 96, 80, slices), k_slices=slices, config=cfg)
        torch.cuda.synchronize()
        assert torch.equal(C.cpu().double(), exact), slices


def test_splitk_degenerate_slice_counts_and_workspace_extent():
    c = wl.gemm_case(8700, 40, 56, 40, "f16", bias="col")
    cfg = sliceable_configs("f16")[0]
    # more slices than K tiles: the effective count shrinks (possibly to one: the unsliced kernel)
    err, _, _ = run_gemm_case(c, config=cfg, k_slices=16)
    assert err <= TOL["f16"]
    # K = 0 with slices: C = epilogue(0), workspace unused
    bias = torch.tensor([1.0, -2.0, 3.0, 0.5], dtype=torch.float16, device="cuda")
    C = torch.full((4, 4), float("nan"), dtype=torch.float16, device="cuda")
    hb.hidet_batched_gemm_splitk(torch.zeros((4, 0), dtype=torch.float16, device="cuda"),
                                 torch.zeros((0, 4), dtype=torch.float16, device="cuda"), C, None, k_slices=4,
                                 epilogue=hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True))
    torch.cuda.synchronize()
    assert torch.equal(C.cpu(), torch.tensor([[1.0, 0.0, 3.0, 0.5]] * 4, dtype=torch.float16))
    # the kernels stay inside the stated workspace size and inside C
    c = wl.gemm_case(8710, 45, 51, 700, "f16")
    A, B = to_gpu(c["A"], "f16"), to_gpu(c["B"], "f16")
    need = hb.hidet_splitk_workspace_bytes(1, 45, 51, 4) // 4
    ws = torch.full((need + 1024,), 5.0, dtype=torch.float32, device="cuda")
    big = torch.full((64, 64), 7.0, dtype=torch.float16, device="cuda")
    hb.hidet_batched_gemm_splitk(A, B, big[:45, :51], ws[:need], k_slices=4, config=cfg)
    torch.cuda.synchronize()
    assert torch.all(ws[need:] == 5.0)
    assert torch.all(big[45:, :] == 7.0) and torch.all(big[:, 51:] == 7.0)
    ref = oracle.gemm(wl.widen(c["A"], "f16"), wl.widen(c["B"], "f16"))
    assert oracle.rel_frobenius(to_f64(big[:45, :51]), ref) <= TOL["f16"]
    # too small a workspace is refused, not overrun
    with pytest.raises(hb.HidetError):
        hb.hidet_batched_gemm_splitk(A, B, big[:45, :51], ws[:need - 1], k_slices=4, config=cfg)


def test_splitk_repeated_calls_are_bit_identical_on_a_grid_that_spans_every_die():
    """4096 workgroups over all compute units, then the reduce pass: slices are added in slice order, so repeated
    calls must agree to the bit."""
    c = wl.gemm_case(8750, 256, 4096, 4096, "f16", bias="col")
    A, B, bias = to_gpu(c["A"], "f16"), to_gpu(c["B"], "f16"), to_gpu(c["bias"], "f16")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True)
    cfg = [i for i in sliceable_configs("f16") if hb.hidet_config_info(i)["block_m"] == 64
           and hb.hidet_config_info(i)["block_n"] == 32][0]
    ws = make_workspace(1, 256, 4096, 8)
    first = torch.empty((256, 4096), dtype=torch.float16, device="cuda")
    hb.hidet_batched_gemm_splitk(A, B, first, ws, k_slices=8, epilogue=epi, config=cfg)
    torch.cuda.synchronize()
    ref = oracle.gemm(wl.widen(c["A"], "f16"), wl.widen(c["B"], "f16"), bias=wl.widen(c["bias"], "f16"), relu=True)
    assert oracle.rel_frobenius(to_f64(first), ref) <= TOL["f16"]
    C = torch.empty_like(first)
    for i in range(20):
        C.fill_(float("nan"))
        hb.hidet_batched_gemm_splitk(A, B, C, ws, k_slices=8, epilogue=epi, config=cfg)
        torch.cuda.synchronize()
        assert torch.equal(C, first), i


def test_splitk_batched_with_shared_operand_and_residual():
    g = wl.rng(8800)
    A = wl.normal(g, (5, 33, 640), "f16")
    B = wl.normal(g, (640, 29), "f16")
    R = wl.normal(g, (5, 33, 29), "f16")
    dA, dB, dR = to_gpu(A, "f16"), to_gpu(B, "f16"), to_gpu(R, "f16")
    C = torch.zeros((5, 33, 29), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(alpha=0.25, residual=dR, relu=True, batched=True)
    hb.hidet_batched_gemm_splitk(dA, dB.unsqueeze(0).expand(5, 640, 29), C, make_workspace(5, 33, 29, 3), k_slices=3,
                                 epilogue=epi)
    torch.cuda.synchronize()
    ref = oracle.batched_gemm(wl.widen(A, "f16"), np.broadcast_to(wl.widen(B, "f16"), (5, 640, 29)), alpha=0.25,
                              residual=wl.widen(R, "f16"), relu=True)
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL["f16"]


def test_splitk_tuner_picks_slices_for_a_few_tile_problem():
    # the small transformer product: 6 x 1 tiles of 128x128 cannot fill 256 compute units without slicing K
    c = wl.gemm_case(8900, 128, 768, 3072, "f16", bias="col")
    A, B, bias = to_gpu(c["A"], "f16"), to_gpu(c["B"], "f16"), to_gpu(c["bias"], "f16")
    C = torch.zeros((128, 768), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL)
    ws = make_workspace(1, 128, 768, 16)
    hb.hidet_tune_clear()
    best, slices, us = hb.hidet_tune_gemm_splitk(A, B, C, ws, epilogue=epi, iters=5)
    _say("splitk tuner: config %d slices %d %.1f us" % (best, slices, us))
    assert best in applicable_configs("f16") and slices in (1, 2, 3, 4, 6, 8, 12, 16)
    ref = oracle.gemm(wl.widen(c["A"], "f16"), wl.widen(c["B"], "f16"), bias=wl.widen(c["bias"], "f16"))
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL["f16"]
    C.zero_()
    hb.hidet_batched_gemm_splitk(A, B, C, ws, k_slices=0, epilogue=epi)  # remembered (config, slices)
    torch.cuda.synchronize()
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL["f16"]
    x = wl.conv_case(8910, 1, 256, 14, 14, 256, 3, 3, 1, 1, "f16")
    x.update(relu=True)
    dx, dw, db = to_gpu(x["x"], "f16"), to_gpu(x["w"], "f16"), to_gpu(x["bias"], "f16")
    y = torch.zeros((1, 256, 14, 14), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(bias=db, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
    best, slices, us = hb.hidet_tune_conv2d_splitk(dx, dw, y, ws, stride=(1, 1), pad=(1, 1), epilogue=epi, iters=5)
    _say("splitk conv tuner: config %d slices %d %.1f us" % (best, slices, us))
    ref = oracle.conv2d(wl.widen(x["x"], "f16"), wl.widen(x["w"], "f16"), stride=(1, 1), pad=(1, 1),
                        bias=wl.widen(x["bias"], "f16"), relu=True)
    assert oracle.rel_frobenius(to_f64(y), ref) <= TOL["f16"]


# ------------------------------------------------------------------ measurement aid
def test_mfma_ceiling_probe_reports_plausible_numbers():
    sample = torch.rand(1 << 16, device="cuda").to(torch.float16) * 2 - 1
    for mfma in (16, 32):
        tflops, mhz = hb.hidet_probe_mfma_peak(sample, mfma=mfma)
        _say("mfma %d ceiling: %.0f TFLOP/s at %.0f MHz" % (mfma, tflops, mhz))
        assert 200.0 < tflops < 2600.0 and 500.0 < mhz < 2600.0
    t32, _ = hb.hidet_probe_mfma_peak(torch.rand(1 << 14, device="cuda"), mfma=32)
    assert 20.0 < t32 < 160.0
    floor = hb.hidet_probe_launch_floor(500)
    _say("launch floor %.2f us" % floor)
    assert 0.5 < floor < 50.0


# ------------------------------------------------------------------ tile quantisation: rows split for whole rounds
@pytest.mark.parametrize("transA,bias", [(False, "row"), (False, "col"), (True, "row")])
def test_untuned_large_gemm_is_cut_into_whole_rounds_and_the_rest(transA, bias):
    """17 x 17 tiles of 256 x 256 are one round of the 256 compute units plus 33 tiles: an untuned call runs the
    first 15 tile rows on the large tile and the remaining rows as a problem of its own (two launches), and the
    result is that of the whole problem -- row bias, residual and a transposed A follow the cut."""
    M = N = 4352
    K = 160
    hb.hidet_tune_clear()
    c = wl.gemm_case(7700 + int(transA) + (1 if bias == "row" else 0) * 2, M, N, K, "f16", transA=transA, bias=bias, residual=True)
    before = hb.hidet_kernel_launch_count()
    err, got, ref = run_gemm_case(c, relu=True, alpha=0.5)
    launches = hb.hidet_kernel_launch_count() - before
    _say("4352^2 x %d tA%d bias %s: err %.3e, %d launches" % (K, transA, bias, err, launches))
    assert err <= TOL["f16"]
    assert launches == 2
    # an explicit configuration is never cut
    before = hb.hidet_kernel_launch_count()
    cfg = next(i for i in applicable_configs("f16") if hb.hidet_config_info(i)["schedule"] == 1
               and hb.hidet_config_info(i)["block_m"] == 256 and hb.hidet_config_info(i)["block_n"] == 256
               and hb.hidet_config_info(i)["mfma"] == (32 if transA else 16))
    err, _, _ = run_gemm_case(c, config=cfg, relu=True, alpha=0.5)
    assert err <= TOL["f16"] and hb.hidet_kernel_launch_count() - before == 1
    # a remembered (tuned) configuration is cut like the size-based one when it is the large ring tile
    A, B = to_gpu(c["A"], "f16"), to_gpu(c["B"], "f16")
    Av = A[:, :M] if transA else A[:, :K]
    epi = hb.make_epilogue(alpha=0.5, bias=to_gpu(c["bias"], "f16"), bias_axis=bias_axis_code(c["bias_axis"]),
                           residual=to_gpu(c["residual"], "f16"), relu=True)
    hb.hidet_tune_gemm(Av, B[:, :N], torch.empty((M, N), dtype=torch.float16, device="cuda"), transA=transA, epilogue=epi,
                       iters=3)
    before = hb.hidet_kernel_launch_count()
    err, _, _ = run_gemm_case(c, relu=True, alpha=0.5)
    assert err <= TOL["f16"] and hb.hidet_kernel_launch_count() - before in (1, 2)
    hb.hidet_tune_clear()


def test_kernel_launch_count_of_plain_and_k_sliced_calls():
    c = wl.gemm_case(7710, 96, 200, 1024, "f16", bias="col")
    before = hb.hidet_kernel_launch_count()
    run_gemm_case(c)
    assert hb.hidet_kernel_launch_count() - before == 1
    before = hb.hidet_kernel_launch_count()
    run_gemm_case(c, k_slices=4, config=sliceable_configs("f16")[0])
    assert hb.hidet_kernel_launch_count() - before == 2


def test_wide_gemm_is_cut_by_columns_for_whole_rounds():
    """8 x 37 tiles of 256 x 256: the whole round is 32 tile columns, the rest (5 x 8 tiles) runs on its own; column
    bias, residual and a transposed B follow the cut."""
    M, N, K = 2048, 9472, 160
    hb.hidet_tune_clear()
    for transB in (False, True):
        c = wl.gemm_case(7720 + int(transB), M, N, K, "f16", transB=transB, bias="col", residual=True)
        before = hb.hidet_kernel_launch_count()
        err, _, _ = run_gemm_case(c, relu=True, alpha=0.5)
        assert err <= TOL["f16"]
        assert hb.hidet_kernel_launch_count() - before == 2, transB
