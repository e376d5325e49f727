"""Parity at the size limits of the interface: operands and outputs whose element offsets need more than 32
bits.  The tensors are too large to check whole on the host, so the oracle computes sampled rows and windows --
chosen on both sides of the 2^31-element mark -- and device-side properties cover the rest."""
import numpy as np
import pytest
import torch

import oracle
from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

from helpers import TOL, TORCH_DTYPE, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def _ring_config():
    for i in range(hb.hidet_config_count()):
        c = hb.hidet_config_info(i)
        if c["schedule"] == 1 and not c["is_f32"] and c["block_m"] == 256:
            return i
    raise AssertionError("no ring configuration")


@pytest.mark.parametrize("which", ["default", "ring"])
def test_gemm_output_beyond_2_31_elements(which):
    dtype = "f16"
    M, N, K = 50003, 43008, 40  # M * N = 2.15e9 > 2^31; rows from 49933 on start beyond the 2^31-element mark
    assert M * N > 2 ** 31
    c = wl.gemm_case(7101, M, N, K, dtype, bias="col")
    A, B, bias = to_gpu(c["A"], dtype), to_gpu(c["B"], dtype), to_gpu(c["bias"], dtype)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True)
    print("gemm %dx%dx%d, %s config" % (M, N, K, which), flush=True)
    hb.hidet_gemm(A, B, C, epilogue=epi, config=_ring_config() if which == "ring" else -1)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(C).all()) and float(C.min()) >= 0.0  # every element was written
    A64, B64, b64 = wl.widen(c["A"], dtype), wl.widen(c["B"], dtype), wl.widen(c["bias"], dtype)
    first_high = 2 ** 31 // N
    rows = sorted(set([0, 255, 256, 25000, first_high - 1, first_high, first_high + 1, M - 257, M - 2, M - 1]))
    ref = oracle.gemm(A64[rows], B64, bias=b64, relu=True)
    got = to_f64(C[rows])
    err = oracle.rel_frobenius(got, ref)
    print("  sampled rows err %.3e" % err, flush=True)
    assert err <= TOL[dtype]


@pytest.mark.parametrize("lda", [4 << 20, (4 << 20) + 8, (4 << 20) + 3])
def test_gemm_operand_beyond_2_31_elements(lda):
    """A with a leading dimension so large that its rows lie gigabytes apart: 16-byte loads with 32-bit in-tile
    offsets at the largest leading dimension that allows them, element-aligned loads with 64-bit offsets above."""
    dtype = "f16"
    M, N, K = 600, 136, 72
    assert M * lda > 2 ** 31
    c = wl.gemm_case(7200 + lda % 16, M, N, K, dtype)
    big = torch.zeros(M * lda, dtype=TORCH_DTYPE[dtype], device="cuda")
    A = big.view(M, lda)[:, :K]
    A.copy_(to_gpu(c["A"], dtype))
    B = to_gpu(c["B"], dtype)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
    print("gemm %dx%dx%d lda=%d" % (M, N, K, lda), flush=True)
    hb.hidet_gemm(A, B, C)
    torch.cuda.synchronize()
    ref = oracle.gemm(wl.widen(c["A"], dtype), wl.widen(c["B"], dtype))
    err = oracle.rel_frobenius(to_f64(C), ref)
    print("  err %.3e" % err, flush=True)
    assert err <= TOL[dtype]
    # transposed use of the same memory: the buffer read as a K' x M' matrix whose rows are lda apart
    Kt, Mt = 40, 264
    At = big.view(M, lda)[:Kt, :Mt]
    At.copy_(to_gpu(wl.uniform(wl.rng(7250), (Kt, Mt), dtype), dtype))
    Ct = torch.full((Mt, N), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
    Bt = B[:Kt]
    hb.hidet_gemm(At, Bt, Ct, transA=True)
    torch.cuda.synchronize()
    At64 = to_f64(At)
    ref = oracle.gemm(At64, wl.widen(c["B"], dtype)[:Kt], transA=True)
    assert oracle.rel_frobenius(to_f64(Ct), ref) <= TOL[dtype]


def test_conv_input_near_the_limit_and_output_beyond_2_31_elements():
    """x just below the 2^31-element limit of the gather, y above it.  The input is drawn on the device (seeded);
    the oracle convolves windows of it, copied to the host, at the corners, around the 2^31-element mark of y and
    at random places."""
    dtype = "f16"
    IC, H, W, OC = 2, 32700, 32700, 3
    assert IC * H * W <= 2 ** 31 - 65537 < 2 ** 31 < OC * H * W
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7300)
    x = torch.empty((1, IC, H, W), dtype=torch.float16, device="cuda")
    x.uniform_(-1.0, 1.0, generator=gen)
    g = wl.rng(7301)
    w_st = wl.normal(g, (OC, IC, 3, 3), dtype, std=(2.0 / (IC * 9)) ** 0.5)
    b_st = wl.uniform(g, (OC,), dtype)
    w, bias = to_gpu(w_st, dtype), to_gpu(b_st, dtype)
    y = torch.full((1, OC, H, W), float("nan"), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
    print("conv 1x%dx%dx%d -> %d channels" % (IC, H, W, OC), flush=True)
    hb.hidet_conv2d_implicit_gemm(x, w, y, stride=(1, 1), pad=(1, 1), epilogue=epi)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(y).all()) and float(y.min()) >= 0.0
    w64, b64 = wl.widen(w_st, dtype), wl.widen(b_st, dtype)
    WH, WW = 5, 48
    r = np.random.default_rng(7302)
    mark = (2 ** 31 - 2 * H * W) // W  # the row of channel 2 where y's element offset passes 2^31
    assert 0 <= mark < H - WH
    corners = [(0, 0), (0, W - WW), (H - WH, 0), (H - WH, W - WW), (mark - 2, 0), (mark - 2, W - WW)]
    windows = corners + [(int(r.integers(H - WH)), int(r.integers(W - WW))) for _ in range(10)]
    num = den = 0.0
    for oh0, ow0 in windows:
        # the window's receptive field with the zero padding written out
        crop = np.zeros((1, IC, WH + 2, WW + 2))
        h_lo, h_hi = max(oh0 - 1, 0), min(oh0 + WH + 1, H)
        w_lo, w_hi = max(ow0 - 1, 0), min(ow0 + WW + 1, W)
        crop[0, :, h_lo - (oh0 - 1):h_hi - (oh0 - 1), w_lo - (ow0 - 1):w_hi - (ow0 - 1)] = to_f64(x[0, :, h_lo:h_hi, w_lo:w_hi])
        ref = oracle.conv2d(crop, w64, stride=(1, 1), pad=(0, 0), bias=b64, relu=True)
        got = to_f64(y[:, :, oh0:oh0 + WH, ow0:ow0 + WW])
        assert ref.shape == got.shape
        num += float(np.sum((got - ref) ** 2))
        den += float(np.sum(ref ** 2))
    err = (num / den) ** 0.5
    print("  windows err %.3e" % err, flush=True)
    assert err <= TOL[dtype]
