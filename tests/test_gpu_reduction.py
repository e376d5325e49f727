"""Parity of the reduction template (row sum / max / mean, row softmax) and of attention composed from the
library's own calls, against the float64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from oracle import reduction as red
from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

from helpers import TOL, TORCH_DTYPE, to_f64, to_gpu, within_bound

pytestmark = pytest.mark.gpu

# row lengths that hit every lane grouping, every repeat count, ragged last chunks and the streamed kernel
COLS_16 = [1, 7, 8, 33, 64, 100, 128, 257, 512, 513, 1000, 2048, 3001, 8192, 8193, 20000]
COLS_32 = [1, 3, 4, 33, 100, 256, 1000, 4096, 4097, 9001]


def _say(msg):
    print(msg, flush=True)


def _rows_for(cols):
    return 37 if cols <= 4096 else 5


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_softmax_rows(dtype):
    g = wl.rng(9100)
    for cols in (COLS_32 if dtype == "f32" else COLS_16):
        rows = _rows_for(cols)
        x = wl.to_storage((g.standard_normal((rows, cols)) * 3).astype(np.float32), dtype)
        dx = to_gpu(x, dtype)
        dy = torch.full((rows, cols), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
        hb.hidet_softmax_rows(dx, dy)
        torch.cuda.synchronize()
        ref = red.softmax_rows(wl.widen(x, dtype))
        err = oracle.rel_frobenius(to_f64(dy), ref)
        _say("softmax %s cols %d err %.3e" % (dtype, cols, err))
        assert within_bound(err, ref, dtype), cols
        hb.hidet_softmax_rows(dx, dx)  # in place
        torch.cuda.synchronize()
        assert torch.equal(dx, dy), cols


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_softmax_strided_misaligned_and_masked(dtype):
    g = wl.rng(9200)
    es = 4 if dtype == "f32" else 2
    for cols, ld, shift in ((100, 104, 0), (100, 107, 0), (96, 96, 1), (5000 * (4 // es + 1), 5000 * (4 // es + 1) + 3, 1)):
        rows = 9
        x = wl.to_storage((g.standard_normal((rows, cols)) * 2).astype(np.float32), dtype)
        x64 = wl.widen(x, dtype)
        x64[1, : cols // 2] = -np.inf  # a masked prefix, as in causal attention
        buf = torch.full((rows * ld + shift + 8,), 7.0, dtype=TORCH_DTYPE[dtype], device="cuda")
        view = buf[shift: shift + rows * ld].view(rows, ld)[:, :cols]
        view.copy_(torch.from_numpy(x64).to(TORCH_DTYPE[dtype]))
        out = torch.full((rows * ld + shift + 8,), 7.0, dtype=TORCH_DTYPE[dtype], device="cuda")
        oview = out[shift: shift + rows * ld].view(rows, ld)[:, :cols]
        hb.hidet_softmax_rows(view, oview)
        torch.cuda.synchronize()
        ref = red.softmax_rows(x64)
        assert within_bound(oracle.rel_frobenius(to_f64(oview), ref), ref, dtype), (cols, ld, shift)
        assert torch.all(oview[1, : cols // 2] == 0)
        # nothing outside the rows was written
        full = out[shift: shift + rows * ld].view(rows, ld)
        assert torch.all(full[:, cols:] == 7.0) and torch.all(out[:shift] == 7.0) and torch.all(out[shift + rows * ld:] == 7.0)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_reduce_rows(dtype):
    g = wl.rng(9300)
    for cols in (COLS_32 if dtype == "f32" else COLS_16):
        rows = _rows_for(cols)
        x = wl.to_storage(g.standard_normal((rows, cols)).astype(np.float32) + 0.25, dtype)
        dx = to_gpu(x, dtype)
        x64 = wl.widen(x, dtype)
        for op, name in ((hb.HIDET_REDUCE_SUM, red.SUM), (hb.HIDET_REDUCE_MAX, red.MAX), (hb.HIDET_REDUCE_MEAN, red.MEAN)):
            ref = red.reduce_rows(x64, name)
            y32 = torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda")
            hb.hidet_reduce_rows(dx, y32, op)
            y = torch.full((rows,), float("nan"), dtype=TORCH_DTYPE[dtype], device="cuda")
            hb.hidet_reduce_rows(dx, y, op)
            torch.cuda.synchronize()
            if op == hb.HIDET_REDUCE_MAX:
                assert np.array_equal(to_f64(y32), ref) and np.array_equal(to_f64(y), ref), cols  # exact: no arithmetic
            else:
                assert oracle.rel_frobenius(to_f64(y32), ref) <= 1e-5, (cols, op)
                assert within_bound(oracle.rel_frobenius(to_f64(y), ref), ref, dtype), (cols, op)


def test_reduce_closed_forms_and_degenerate_shapes():
    n = 3000
    x = torch.arange(1, n + 1, dtype=torch.float32, device="cuda").repeat(3, 1)
    y = torch.zeros(3, dtype=torch.float32, device="cuda")
    hb.hidet_reduce_rows(x, y, hb.HIDET_REDUCE_SUM)
    torch.cuda.synchronize()
    assert y.tolist() == [n * (n + 1) / 2] * 3  # every partial sum is an integer below 2^24: exact in fp32
    empty = torch.zeros((2, 0), dtype=torch.float16, device="cuda")
    y = torch.full((2,), 5.0, dtype=torch.float32, device="cuda")
    hb.hidet_reduce_rows(empty, y, hb.HIDET_REDUCE_SUM)
    torch.cuda.synchronize()
    assert y.tolist() == [0.0, 0.0]
    hb.hidet_reduce_rows(empty, y, hb.HIDET_REDUCE_MAX)
    torch.cuda.synchronize()
    assert y.tolist() == [-np.inf, -np.inf]
    hb.hidet_softmax_rows(empty, empty)
    hb.hidet_softmax_rows(torch.zeros((0, 5), dtype=torch.float16, device="cuda"),
                          torch.zeros((0, 5), dtype=torch.float16, device="cuda"))
    ones = torch.full((4, 16), 2.5, dtype=torch.float16, device="cuda")
    hb.hidet_softmax_rows(ones, ones)
    torch.cuda.synchronize()
    assert torch.all(ones == 1.0 / 16)


@pytest.mark.parametrize("batch,seq", [(12, 128), (12, 512)])
def test_attention_from_the_three_calls(batch, seq):
    """scores = alpha * Q.K^T (fused scale), softmax in place, context = S.V -- every step in the library."""
    c = wl.attention_case(9400 + seq, batch, seq, "f16")
    Q, K, V = (to_gpu(c[k], "f16") for k in ("Q", "K", "V"))
    scores = torch.empty((batch, seq, seq), dtype=torch.float16, device="cuda")
    ctx = torch.full((batch, seq, c["d"]), float("nan"), dtype=torch.float16, device="cuda")
    hb.hidet_batched_gemm(Q, K, scores, transB=True, epilogue=hb.make_epilogue(alpha=c["alpha"]))
    hb.hidet_softmax_rows(scores, scores)
    hb.hidet_batched_gemm(scores, V, ctx)
    torch.cuda.synchronize()
    ref = red.attention(wl.widen(c["Q"], "f16"), wl.widen(c["K"], "f16"), wl.widen(c["V"], "f16"), c["alpha"])
    err = oracle.rel_frobenius(to_f64(ctx), ref)
    _say("attention b%d s%d err %.3e" % (batch, seq, err))
    assert err <= TOL["f16"]


def test_hip_graph_replays_of_the_attention_chain_match_eager():
    """The library only launches kernels on the caller's stream (no allocation, no memset, no synchronisation),
    so a caller may capture it; every replay must reproduce the eager result bit for bit."""
    c = wl.attention_case(9500, 6, 128, "f16")
    Q, K, V = (to_gpu(c[k], "f16") for k in ("Q", "K", "V"))
    scores = torch.empty((6, 128, 128), dtype=torch.float16, device="cuda")
    ctx = torch.zeros((6, 128, 64), dtype=torch.float16, device="cuda")
    epi = hb.make_epilogue(alpha=c["alpha"])

    def chain():
        hb.hidet_batched_gemm(Q, K, scores, transB=True, epilogue=epi)
        hb.hidet_softmax_rows(scores, scores)
        hb.hidet_batched_gemm(scores, V, ctx)

    chain()
    torch.cuda.synchronize()
    eager = ctx.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        chain()  # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            chain()
    for replay in range(3):
        ctx.zero_()
        scores.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ctx, eager), replay
        V2 = V * 1.0  # unrelated eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(V2, V)


def test_stream_bandwidth_probe_reports_plausible_rates():
    ring = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    rates = [hb.hidet_probe_stream_bandwidth(ring, mode) for mode in range(3)]
    print("read %.0f write %.0f copy %.0f GB/s" % tuple(rates), flush=True)
    for r in rates:
        assert 1000.0 < r < 8000.0  # below the datasheet's HBM rate, far above anything a broken probe reports
    with pytest.raises(hb.HidetError):
        hb.hidet_probe_stream_bandwidth(ring, 3)
    with pytest.raises(hb.HidetError):
        hb.hidet_probe_stream_bandwidth(ring[: 100 << 20], 0)
