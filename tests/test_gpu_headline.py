"""Parity at the full benchmark size (4096^3 and the skinny K=1024 case, fp16 and bf16), in bench.py's launch
configuration: the whole 4096 x 4096 output against the oracle (relative Frobenius error and every element on its
own), sampled outputs one by one against the oracle's literal dot-product form, and a property that holds at any
size on the full output."""
import numpy as np
import pytest
import torch

import oracle
from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

from helpers import TOL, TORCH_DTYPE, assert_elementwise, gemm_scale, to_f64, to_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype,K", [("f16", 4096), ("bf16", 4096), ("f16", 1024), ("bf16", 1024)])
def test_config5_whole_output(dtype, K):
    c = wl.config5(dtype, K=K)
    M, N = c["M"], c["N"]
    A, B, bias = to_gpu(c["A"], dtype), to_gpu(c["B"], dtype), to_gpu(c["bias"], dtype)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_COL, relu=True)
    hb.hidet_gemm(A, B, C, epilogue=epi)
    torch.cuda.synchronize()
    got = to_f64(C)
    assert np.isfinite(got).all() and got.min() >= 0.0
    A64, B64, b64 = wl.widen(c["A"], dtype), wl.widen(c["B"], dtype), wl.widen(c["bias"], dtype)
    # (a) the whole output: every one of the 16.7 M elements against the oracle's row form
    ref = oracle.gemm(A64, B64, bias=b64, relu=True)
    err = oracle.rel_frobenius(got, ref)
    worst = assert_elementwise(got, ref, gemm_scale(A64, B64, False, False, 1.0, b64, "col"), dtype, K,
                               "cfg5 %s K=%d" % (dtype, K))
    # (b) random single elements, literal dot products (the oracle's other form)
    g = np.random.default_rng(5)
    pts = [(int(g.integers(M)), int(g.integers(N))) for _ in range(2000)]
    ref_pts = np.array([oracle.gemm_element(A64, B64, i, j, bias=b64, relu=True) for i, j in pts])
    got_pts = np.array([got[i, j] for i, j in pts])
    err_pts = oracle.rel_frobenius(got_pts, ref_pts)
    print("cfg5 %s K=%d: whole-output err %.3e (worst element at %.2f of its bound), points err %.3e"
          % (dtype, K, err, worst, err_pts), flush=True)
    assert err <= TOL[dtype] and err_pts <= TOL[dtype]
    # (c) a property that holds at any size: with an all-ones B the result of row i is relu(sum_k A[i,k] + bias[j])
    ones = torch.ones((K, N), dtype=TORCH_DTYPE[dtype], device="cuda")
    hb.hidet_gemm(A, ones, C, epilogue=epi)
    torch.cuda.synchronize()
    ref = np.maximum(A64.sum(axis=1)[:, None] + b64[None, :], 0.0)
    assert oracle.rel_frobenius(to_f64(C), ref) <= TOL[dtype]
