"""The allocation-free K-parallel entry point (static scratch array inside the library) against the entry point
that takes the caller's workspace: same kernels, so the outputs must agree bit for bit -- on two calls in a row,
the second on a smaller problem (the array keeps the first call's partial sums)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

from helpers import TOL, TORCH_DTYPE, bias_axis_code, make_workspace, oracle_bias_axis, to_f64, to_gpu

pytestmark = pytest.mark.gpu


def _both(c, k_slices, config, relu, alpha):
    dt = c["dtype"]
    A, B = to_gpu(c["A"], dt), to_gpu(c["B"], dt)
    M, N, K = c["M"], c["N"], c["K"]
    bias, res = to_gpu(c["bias"], dt), to_gpu(c["residual"], dt)
    epi = hb.make_epilogue(alpha=alpha, bias=bias, bias_axis=bias_axis_code(c["bias_axis"]), residual=res, relu=relu)
    want = torch.full((M, N), float("nan"), dtype=TORCH_DTYPE[dt], device="cuda")
    hb.hidet_batched_gemm_splitk(A, B, want, make_workspace(1, M, N, k_slices), k_slices=k_slices, transB=c["transB"],
                                 epilogue=epi, config=config)
    got = torch.full((M, N), float("nan"), dtype=TORCH_DTYPE[dt], device="cuda")
    before = torch.cuda.memory_allocated()
    hb.hidet_batched_gemm_splitk_static(A, B, got, k_slices=k_slices, transB=c["transB"], epilogue=epi, config=config)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    ref = oracle.gemm(wl.widen(c["A"], dt), wl.widen(c["B"], dt), transB=c["transB"], alpha=alpha,
                      bias=None if c["bias"] is None else wl.widen(c["bias"], dt), bias_axis=oracle_bias_axis(c["bias_axis"]),
                      residual=None if c["residual"] is None else wl.widen(c["residual"], dt), relu=relu)
    return got, want, ref


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    print("static scratch: %d bytes" % hb.hidet_static_scratch_bytes(), flush=True)
    # first call: several tiles and a ragged tail in every dimension, 6 slices of K
    c1 = wl.gemm_case(9100, 300, 411, 1000, "f16", bias="col", residual=True)
    got, want, ref = _both(c1, 6, 3, True, 0.5)
    assert torch.equal(got, want)
    assert oracle.rel_frobenius(to_f64(got), ref) <= TOL["f16"]
    # second call, smaller, other operand form and tile: stale partial sums of the first call lie in the array
    c2 = wl.gemm_case(9101, 70, 129, 333, "bf16", transB=True, bias="row")
    got, want, ref = _both(c2, 4, 11, False, -1.25)
    assert torch.equal(got, want)
    assert oracle.rel_frobenius(to_f64(got), ref) <= TOL["bf16"]
    # third call: the tuned / default path (config < 0, slice count from the caller)
    c3 = wl.gemm_case(9102, 128, 768, 3072, "f16", dist="normal", residual=True, w_std=0.02)
    got, want, ref = _both(c3, 8, -1, False, 1.0)
    assert torch.equal(got, want)
    assert oracle.rel_frobenius(to_f64(got), ref) <= TOL["f16"]


def test_static_scratch_rejects_what_does_not_fit():
    limit = hb.hidet_static_scratch_bytes()
    M = N = 2048  # 16 MiB of fp32 per slice: three slices exceed the 32 MiB array, two fit exactly
    assert hb.hidet_splitk_workspace_bytes(1, M, N, 3) > limit >= hb.hidet_splitk_workspace_bytes(1, M, N, 2)
    A = torch.ones((M, 768), dtype=torch.float16, device="cuda")
    B = torch.ones((768, N), dtype=torch.float16, device="cuda")
    C = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    with pytest.raises(hb.HidetError) as e:
        hb.hidet_batched_gemm_splitk_static(A, B, C, k_slices=3, config=3)
    assert e.value.status == 6 and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(C).all()  # nothing was launched
    hb.hidet_batched_gemm_splitk_static(A, B, C, k_slices=2, config=3)
    torch.cuda.synchronize()
    assert torch.equal(C, torch.full_like(C, 768.0))
