"""Seeded random sweep over the whole interface: shapes, operand forms, leading-dimension padding, epilogue flags,
tile configuration and K-slice count are all drawn at random (fixed seeds, so every run checks the same cases) and
each case is compared with the oracle element by element."""
import numpy as np
import pytest

from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

from helpers import applicable_configs, run_conv_case, run_gemm_case, sliceable_configs, within_bound

pytestmark = pytest.mark.gpu

DTYPES = ["f16", "bf16", "f32"]


def _log_uniform(g, lo, hi):
    return int(round(float(np.exp(g.uniform(np.log(lo), np.log(hi))))))


@pytest.mark.parametrize("seed", range(8))
def test_random_gemms(seed):
    g = np.random.default_rng(9000 + seed)
    for case in range(12):
        dtype = DTYPES[int(g.integers(3))]
        M, N, K = _log_uniform(g, 1, 400), _log_uniform(g, 1, 400), _log_uniform(g, 1, 700)
        transA, transB = bool(g.integers(2)), bool(g.integers(2))
        bias = [None, "col", "row"][int(g.integers(3))]
        residual, relu = bool(g.integers(2)), bool(g.integers(2))
        alpha = [1.0, 0.5, -2.0, 0.125][int(g.integers(4))]
        lda_pad, ldb_pad = int(g.integers(0, 3)) * int(g.integers(1, 9)), int(g.integers(0, 3)) * int(g.integers(1, 9))
        sliced = bool(g.integers(3) == 0)
        configs = sliceable_configs(dtype) if sliced else applicable_configs(dtype)
        config = -1 if g.integers(4) == 0 else int(configs[int(g.integers(len(configs)))])
        k_slices = int(g.integers(2, 7)) if sliced else None
        c = wl.gemm_case(9100 + 100 * seed + case, M, N, K, dtype, transA=transA, transB=transB, bias=bias,
                         residual=residual, lda_pad=lda_pad, ldb_pad=ldb_pad)
        what = "seed %d case %d: %s %dx%dx%d tA%d tB%d bias=%s res=%d relu=%d alpha=%g pads %d %d config %d slices %s" % (
            seed, case, dtype, M, N, K, transA, transB, bias, residual, relu, alpha, lda_pad, ldb_pad, config, k_slices)
        print(what, flush=True)
        try:
            err, _, ref = run_gemm_case(c, config=config, relu=relu, alpha=alpha, k_slices=k_slices)
        except hb.HidetError as e:
            if e.status != 4 or not transA:  # only some configurations are built for a transposed A
                raise
            print("  (configuration %d has no transposed-A form: size-based default instead)" % config, flush=True)
            err, _, ref = run_gemm_case(c, config=-1, relu=relu, alpha=alpha, k_slices=k_slices)
        assert within_bound(err, ref, dtype), what + " err %.3e" % err


@pytest.mark.parametrize("seed", range(6))
def test_random_convs(seed):
    g = np.random.default_rng(9500 + seed)
    for case in range(8):
        dtype = DTYPES[int(g.integers(3))]
        Nb, IC, OC = int(g.integers(1, 4)), _log_uniform(g, 1, 40), _log_uniform(g, 1, 70)
        KH, KW = int(g.integers(1, 6)), int(g.integers(1, 6))
        sh, sw = int(g.integers(1, 4)), int(g.integers(1, 4))
        ph, pw = int(g.integers(0, 4)), int(g.integers(0, 4))
        H = max(_log_uniform(g, 1, 40), KH - 2 * ph)
        W = max(_log_uniform(g, 1, 40), KW - 2 * pw)
        sliced = bool(g.integers(3) == 0)
        configs = sliceable_configs(dtype) if sliced else applicable_configs(dtype)
        config = -1 if g.integers(4) == 0 else int(configs[int(g.integers(len(configs)))])
        k_slices = int(g.integers(2, 6)) if sliced else None
        c = wl.conv_case(9600 + 100 * seed + case, Nb, IC, H, W, OC, KH, KW, (sh, sw), (ph, pw), dtype,
                         bias=bool(g.integers(2)), residual=bool(g.integers(2)))
        c["relu"] = bool(g.integers(2))
        c["alpha"] = [1.0, 0.5, -1.5][int(g.integers(3))]
        what = "seed %d case %d: %s N%d %d->%d %dx%d k%dx%d s%dx%d p%dx%d config %d slices %s" % (
            seed, case, dtype, Nb, IC, OC, H, W, KH, KW, sh, sw, ph, pw, config, k_slices)
        print(what, flush=True)
        err, _, ref = run_conv_case(c, config=config, k_slices=k_slices)
        assert within_bound(err, ref, dtype), what + " err %.3e" % err


@pytest.mark.parametrize("seed", range(4))
def test_random_pointwise_convs(seed):
    """1x1, stride-1, unpadded convolutions with no configuration named: the batched-GEMM form, unsliced and K-sliced,
    over image sizes with and without 16-byte aligned rows."""
    g = np.random.default_rng(9700 + seed)
    for case in range(10):
        dtype = DTYPES[int(g.integers(3))]
        Nb, IC, OC = int(g.integers(1, 6)), _log_uniform(g, 1, 300), _log_uniform(g, 1, 200)
        H, W = _log_uniform(g, 1, 30), _log_uniform(g, 1, 30)
        k_slices = int(g.integers(2, 6)) if g.integers(3) == 0 else None
        c = wl.conv_case(9700 + 100 * seed + case, Nb, IC, H, W, OC, 1, 1, 1, 0, dtype,
                         bias=bool(g.integers(2)), residual=bool(g.integers(2)))
        c["relu"] = bool(g.integers(2))
        c["alpha"] = [1.0, 0.5, -1.5][int(g.integers(3))]
        what = "seed %d case %d: %s N%d %d->%d %dx%d slices %s" % (seed, case, dtype, Nb, IC, OC, H, W, k_slices)
        print(what, flush=True)
        err, _, ref = run_conv_case(c, k_slices=k_slices)
        assert within_bound(err, ref, dtype), what + " err %.3e" % err


@pytest.mark.parametrize("seed", range(6))
def test_random_batched_wide_and_head_split(seed):
    """The remaining forms of the GEMM interface, drawn at random: batches with an operand shared by all entries
    (stride 0) and a per-entry residual, fp32 output from 16-bit inputs, and the head-split output map."""
    import torch

    import oracle
    from helpers import TORCH_DTYPE, make_workspace, to_f64, to_gpu

    g = np.random.default_rng(9800 + seed)
    for case in range(8):
        kind = ["batched", "wide", "head_split"][int(g.integers(3))]
        dtype = ["f16", "bf16"][int(g.integers(2))] if kind == "wide" else DTYPES[int(g.integers(3))]
        transB, relu = bool(g.integers(2)), bool(g.integers(2))
        alpha = [1.0, 0.5, -2.0][int(g.integers(3))]
        K = _log_uniform(g, 1, 500)
        r = wl.rng(9900 + 100 * seed + case)
        if kind == "batched":
            batch, M, N = int(g.integers(1, 7)), _log_uniform(g, 1, 150), _log_uniform(g, 1, 150)
            share = int(g.integers(3))  # 0: none, 1: A shared, 2: B shared
            A = wl.normal(r, (1 if share == 1 else batch, M, K), dtype)
            B = wl.normal(r, (1 if share == 2 else batch, N, K) if transB else (1 if share == 2 else batch, K, N), dtype)
            R = wl.normal(r, (batch, M, N), dtype) if g.integers(2) else None
            bias = wl.normal(r, (N,), dtype) if g.integers(2) else None
            dA, dB = to_gpu(A, dtype).expand(batch, -1, -1), to_gpu(B, dtype).expand(batch, -1, -1)
            dR, dbias = to_gpu(R, dtype), to_gpu(bias, dtype)
            C = torch.full((batch, M, N), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
            epi = hb.make_epilogue(alpha=alpha, bias=dbias, bias_axis=hb.HIDET_BIAS_PER_COL if bias is not None else 0,
                                   residual=dR, relu=relu, batched=True)
            what = "seed %d case %d: batched %s b%d %dx%dx%d tB%d share %d" % (seed, case, dtype, batch, M, N, K, transB, share)
            print(what, flush=True)
            hb.hidet_batched_gemm(dA, dB, C, transB=transB, epilogue=epi)
            torch.cuda.synchronize()
            ref = oracle.batched_gemm(np.broadcast_to(wl.widen(A, dtype), (batch,) + A.shape[1:]),
                                      np.broadcast_to(wl.widen(B, dtype), (batch,) + B.shape[1:]), transB=transB, alpha=alpha,
                                      bias=None if bias is None else wl.widen(bias, dtype),
                                      residual=None if R is None else wl.widen(R, dtype), relu=relu)
            err = oracle.rel_frobenius(to_f64(C), ref)
            assert within_bound(err, ref, dtype), what + " err %.3e" % err
        elif kind == "wide":
            M, N = _log_uniform(g, 1, 300), _log_uniform(g, 1, 300)
            c = wl.gemm_case(9900 + 100 * seed + case, M, N, K, dtype, transB=transB)
            A, B = to_gpu(c["A"], dtype), to_gpu(c["B"], dtype)
            bias = torch.from_numpy(r.standard_normal(N).astype(np.float32)).cuda()
            res = torch.from_numpy(r.standard_normal((M, N)).astype(np.float32)).cuda() if g.integers(2) else None
            epi = hb.make_epilogue(alpha=alpha, bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, residual=res, relu=relu)
            sliced = bool(g.integers(2))
            configs = sliceable_configs(dtype)
            config = -1 if g.integers(3) == 0 else int(configs[int(g.integers(len(configs)))])
            what = "seed %d case %d: wide %s %dx%dx%d tB%d config %d sliced %d" % (seed, case, dtype, M, N, K, transB, config, sliced)
            print(what, flush=True)
            C = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
            if sliced:
                hb.hidet_batched_gemm_splitk(A, B, C, make_workspace(1, M, N, 3), k_slices=3, transB=transB, epilogue=epi,
                                             config=config)
            else:
                hb.hidet_gemm(A, B, C, transB=transB, epilogue=epi, config=config)
            torch.cuda.synchronize()
            ref = oracle.gemm(wl.widen(c["A"], dtype), wl.widen(c["B"], dtype), transB=transB, alpha=alpha,
                              bias=bias.cpu().double().numpy(), residual=None if res is None else res.cpu().double().numpy(),
                              relu=relu)
            err = oracle.rel_frobenius(to_f64(C), ref)
            assert err <= 1e-5, what + " err %.3e" % err  # no output rounding: the fp32 accumulation alone
        else:
            b, seq, heads, d = int(g.integers(1, 4)), _log_uniform(g, 1, 60), int(g.integers(1, 7)), _log_uniform(g, 1, 40)
            M, N = b * seq, heads * d
            c = wl.gemm_case(9900 + 100 * seed + case, M, N, K, dtype, transB=transB, bias="col" if g.integers(2) else None,
                             residual=bool(g.integers(2)))
            A, B = to_gpu(c["A"], dtype), to_gpu(c["B"], dtype)
            bias, res = to_gpu(c["bias"], dtype), to_gpu(c["residual"], dtype)
            if res is not None:  # the residual has the shape of the stored tensor
                res = res.view(b, seq, heads, d).permute(0, 2, 1, 3).contiguous()
            configs = applicable_configs(dtype)
            config = -1 if g.integers(3) == 0 else int(configs[int(g.integers(len(configs)))])
            what = "seed %d case %d: head split %s b%d s%d h%d d%d K%d tB%d config %d" % (seed, case, dtype, b, seq, heads, d, K,
                                                                                      transB, config)
            print(what, flush=True)
            epi = hb.make_epilogue(alpha=alpha, bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL if bias is not None else 0,
                                   residual=res, relu=relu, head_split=(seq, d))
            C = torch.full((b, heads, seq, d), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
            hb.hidet_gemm(A, B, C, transB=transB, epilogue=epi, config=config)
            torch.cuda.synchronize()
            ref = oracle.gemm(wl.widen(c["A"], dtype), wl.widen(c["B"], dtype), transB=transB, alpha=alpha,
                              bias=None if c["bias"] is None else wl.widen(c["bias"], dtype),
                              residual=None if c["residual"] is None else wl.widen(c["residual"], dtype), relu=relu)
            ref = oracle.head_split(ref, seq, d)
            err = oracle.rel_frobenius(to_f64(C), ref)
            assert within_bound(err, ref, dtype), what + " err %.3e" % err
