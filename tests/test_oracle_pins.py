"""Pins for the CPU oracle: closed forms, exact rational brute force, library routines, invariants.

Each check is chosen so that a plausible mistake in oracle.c (dropped term, wrong sign or index,
transposed operand, wrong epilogue order, padding/stride slip) fails at least one of them.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import BIAS_PER_COL, BIAS_PER_ROW


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (17, 9, 33), (64, 64, 256)])
def test_all_ones_contraction_gives_K(M, N, K):
    C = oracle.gemm(np.ones((M, K)), np.ones((K, N)))
    assert np.array_equal(C, np.full((M, N), float(K)))


def test_all_ones_with_bias_and_relu():
    M, N, K = 5, 6, 11
    bias = np.arange(N, dtype=np.float64) - 2.5
    C = oracle.gemm(np.ones((M, K)), np.ones((K, N)), bias=bias, bias_axis=BIAS_PER_COL)
    assert np.array_equal(C, K + np.broadcast_to(bias, (M, N)))
    rb = np.arange(M, dtype=np.float64) * 0.5
    C = oracle.gemm(np.ones((M, K)), np.ones((K, N)), bias=rb, bias_axis=BIAS_PER_ROW)
    assert np.array_equal(C, K + np.broadcast_to(rb[:, None], (M, N)))
    C = oracle.gemm(-np.ones((M, K)), np.ones((K, N)), relu=True)
    assert np.array_equal(C, np.zeros((M, N)))


def test_identity_and_one_hot():
    g = np.random.default_rng(1)
    A = g.standard_normal((7, 7))
    assert np.array_equal(oracle.gemm(A, np.eye(7)), A)
    assert np.array_equal(oracle.gemm(np.eye(7), A), A)
    B = g.standard_normal((6, 9))
    E = np.zeros((4, 6))
    E[2, 5] = 1.0  # A = e_2 e_5^T  -> row 2 of C is row 5 of B
    C = oracle.gemm(E, B)
    expect = np.zeros((4, 9))
    expect[2] = B[5]
    assert np.array_equal(C, expect)


def test_epilogue_invariants():
    g = np.random.default_rng(2)
    A, B = g.standard_normal((6, 8)), g.standard_normal((8, 5))
    bias, res = g.standard_normal(5), g.standard_normal((6, 5))
    # alpha = 0 leaves ReLU(bias + residual)
    C = oracle.gemm(A, B, alpha=0.0, bias=bias, residual=res, relu=True)
    assert np.array_equal(C, np.maximum(bias[None, :] + res, 0.0))
    # doubling A doubles the un-fused result exactly (power of two)
    assert np.array_equal(oracle.gemm(2.0 * A, B), 2.0 * oracle.gemm(A, B))
    # ReLU is applied last: a negative pre-activation made positive by the residual survives
    C = oracle.gemm(-np.ones((1, 1)), np.ones((1, 1)), residual=np.full((1, 1), 3.0), relu=True)
    assert C[0, 0] == 2.0
    # bias and residual are added after alpha scaling, not before
    C = oracle.gemm(np.ones((1, 2)), np.ones((2, 1)), alpha=0.5, bias=np.array([10.0]), residual=np.array([[100.0]]))
    assert C[0, 0] == 111.0


# ---------------------------------------------------------------- exact rational brute force
def _exact_gemm(A, B, transA, transB, alpha, bias, bias_axis, residual, relu):
    A = [[Fraction(int(v)) for v in row] for row in A]
    B = [[Fraction(int(v)) for v in row] for row in B]
    M, K = (len(A[0]), len(A)) if transA else (len(A), len(A[0]))
    N = len(B) if transB else len(B[0])
    out = [[None] * N for _ in range(M)]
    for j in range(N):  # a different loop order from the oracle's, on purpose
        for i in range(M):
            s = Fraction(0)
            for k in reversed(range(K)):
                a = A[k][i] if transA else A[i][k]
                b = B[j][k] if transB else B[k][j]
                s += a * b
            v = Fraction(alpha) * s
            if bias is not None:
                v += Fraction(int(bias[j] if bias_axis == BIAS_PER_COL else bias[i]))
            if residual is not None:
                v += Fraction(int(residual[i][j]))
            if relu and v < 0:
                v = Fraction(0)
            out[i][j] = v
    return out


@pytest.mark.parametrize("transA", [False, True])
@pytest.mark.parametrize("transB", [False, True])
@pytest.mark.parametrize("flags", range(8))
def test_exact_rational_tiny(transA, transB, flags):
    g = np.random.default_rng(100 + flags + 8 * transA + 16 * transB)
    M, N, K = 3, 4, 5
    A = g.integers(-9, 10, size=(K, M) if transA else (M, K)).astype(np.float64)
    B = g.integers(-9, 10, size=(N, K) if transB else (K, N)).astype(np.float64)
    use_bias, use_res, relu = bool(flags & 1), bool(flags & 2), bool(flags & 4)
    axis = BIAS_PER_ROW if (flags & 1 and transA) else BIAS_PER_COL
    bias = g.integers(-9, 10, size=(M if axis == BIAS_PER_ROW else N)).astype(np.float64) if use_bias else None
    res = g.integers(-30, 30, size=(M, N)).astype(np.float64) if use_res else None
    alpha = 0.25  # exactly representable, so float64 results on these small integers are exact
    C = oracle.gemm(A, B, transA=transA, transB=transB, alpha=alpha, bias=bias, bias_axis=axis, residual=res, relu=relu)
    E = _exact_gemm(A, B, transA, transB, alpha, bias, axis, res, relu)
    for i in range(M):
        for j in range(N):
            assert Fraction(C[i, j]) == E[i][j], (i, j)


# ---------------------------------------------------------------- library routine (special case: no epilogue)
@pytest.mark.parametrize("M,N,K", [(1, 1, 9), (13, 7, 29), (65, 130, 257)])
@pytest.mark.parametrize("transA,transB", [(False, False), (False, True), (True, False), (True, True)])
def test_against_numpy_float64(M, N, K, transA, transB):
    g = np.random.default_rng(M * 1000 + N)
    A = g.standard_normal((K, M) if transA else (M, K))
    B = g.standard_normal((N, K) if transB else (K, N))
    ref = np.matmul(A.T if transA else A, B.T if transB else B)
    C = oracle.gemm(A, B, transA=transA, transB=transB)
    assert oracle.rel_frobenius(C, ref) < 1e-14


def test_element_form_equals_row_form_bitwise():
    g = np.random.default_rng(5)
    A, B = g.standard_normal((9, 31)), g.standard_normal((31, 6))
    bias, res = g.standard_normal(6), g.standard_normal((9, 6))
    C = oracle.gemm(A, B, alpha=0.3, bias=bias, residual=res, relu=True)
    for i in range(9):
        for j in range(6):
            assert C[i, j] == oracle.gemm_element(A, B, i, j, alpha=0.3, bias=bias, residual=res, relu=True)
    Bt = np.ascontiguousarray(B.T)
    assert oracle.gemm_element(A, Bt, 4, 3, transB=True) == oracle.gemm(A, B)[4, 3]


def test_rows_subset_and_batched():
    g = np.random.default_rng(6)
    A, B = g.standard_normal((10, 12)), g.standard_normal((12, 5))
    full = oracle.gemm(A, B)
    part = oracle.gemm(A, B, rows=(3, 7))
    assert np.array_equal(part[3:7], full[3:7]) and not part[:3].any() and not part[7:].any()
    Ab, Bb = g.standard_normal((4, 3, 8)), g.standard_normal((4, 8, 6))
    res = g.standard_normal((4, 3, 6))
    Cb = oracle.batched_gemm(Ab, Bb, alpha=0.125, residual=res)
    for b in range(4):
        assert np.array_equal(Cb[b], oracle.gemm(Ab[b], Bb[b], alpha=0.125, residual=res[b]))
    Bt = np.ascontiguousarray(np.swapaxes(Bb, 1, 2))
    assert np.array_equal(oracle.batched_gemm(Ab, Bt, transB=True), oracle.batched_gemm(Ab, Bb))


def test_batched_bias_is_shared_and_residual_advances_per_entry():
    """The bias of a batched product is one vector shared by every entry (per column or per row); only the
    residual advances with the batch index.  Each entry must equal the plain product of that entry."""
    g = np.random.default_rng(16)
    Ab, Bb = g.standard_normal((5, 4, 7)), g.standard_normal((5, 7, 6))
    res = g.standard_normal((5, 4, 6))
    for axis, n in ((BIAS_PER_COL, 6), (BIAS_PER_ROW, 4)):
        bias = g.standard_normal(n)
        Cb = oracle.batched_gemm(Ab, Bb, alpha=-0.75, bias=bias, bias_axis=axis, residual=res, relu=True)
        for b in range(5):
            one = oracle.gemm(Ab[b], Bb[b], alpha=-0.75, bias=bias, bias_axis=axis, residual=res[b], relu=True)
            assert np.array_equal(Cb[b], one), (axis, b)
    # closed form: all-ones entries of length K with a per-column bias give K + bias[j] in every entry
    bias = np.arange(6, dtype=np.float64) - 2.0
    Cb = oracle.batched_gemm(np.ones((3, 4, 7)), np.ones((3, 7, 6)), bias=bias, bias_axis=BIAS_PER_COL)
    assert np.array_equal(Cb, np.broadcast_to(7.0 + bias, (3, 4, 6)))
    rb = np.array([0.5, -1.0, 2.0, 8.0])
    Cb = oracle.batched_gemm(np.ones((3, 4, 7)), np.ones((3, 7, 6)), bias=rb, bias_axis=BIAS_PER_ROW)
    assert np.array_equal(Cb, np.broadcast_to(7.0 + rb[:, None], (3, 4, 6)))


def test_degenerate_shapes():
    assert oracle.gemm(np.zeros((0, 4)), np.zeros((4, 3))).shape == (0, 3)
    assert oracle.gemm(np.zeros((2, 4)), np.zeros((4, 0))).shape == (2, 0)
    # K = 0: the empty sum is 0, so C = Epi(0)
    C = oracle.gemm(np.zeros((2, 0)), np.zeros((0, 3)), bias=np.array([1.0, -2.0, 3.0]), relu=True)
    assert np.array_equal(C, np.array([[1.0, 0.0, 3.0]] * 2))


# ---------------------------------------------------------------- convolution
def test_conv_all_ones_3x3_pad1_counts_taps():
    IC = 5
    y = oracle.conv2d(np.ones((1, IC, 6, 7)), np.ones((2, IC, 3, 3)), pad=(1, 1))
    assert y.shape == (1, 2, 6, 7)
    assert np.all(y[0, :, 1:-1, 1:-1] == 9 * IC)
    assert np.all(y[0, :, 0, 1:-1] == 6 * IC) and np.all(y[0, :, 1:-1, 0] == 6 * IC)
    for r, c in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(y[0, :, r, c] == 4 * IC)


def test_conv_delta_kernel_is_identity_and_shifts_are_not_flipped():
    g = np.random.default_rng(7)
    x = g.standard_normal((1, 1, 5, 6))
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 1, 1] = 1.0
    assert np.array_equal(oracle.conv2d(x, w, pad=(1, 1)), x)
    # cross-correlation: a tap at (kh=0, kw=2) reads x[oh-1][ow+1]
    w = np.zeros((1, 1, 3, 3))
    w[0, 0, 0, 2] = 1.0
    y = oracle.conv2d(x, w, pad=(1, 1))
    assert y[0, 0, 2, 3] == x[0, 0, 1, 4] and y[0, 0, 0, 0] == 0.0


def test_conv_1x1_is_gemm():
    g = np.random.default_rng(8)
    x, w = g.standard_normal((1, 6, 4, 5)), g.standard_normal((3, 6, 1, 1))
    bias = g.standard_normal(3)
    y = oracle.conv2d(x, w, bias=bias, relu=True)
    ref = oracle.gemm(w.reshape(3, 6), x.reshape(6, 20), bias=bias, bias_axis=BIAS_PER_ROW, relu=True)
    assert np.array_equal(y.reshape(3, 20), ref)


@pytest.mark.parametrize("stride,pad,KH,KW", [((1, 1), (1, 1), 3, 3), ((2, 2), (1, 1), 3, 3), ((1, 2), (0, 2), 2, 5),
                                               ((3, 1), (2, 0), 4, 1)])
def test_conv_equals_im2col_gemm_and_torch(stride, pad, KH, KW):
    g = np.random.default_rng(9)
    Nb, IC, H, W, OC = 2, 3, 9, 8, 4
    x, w = g.standard_normal((Nb, IC, H, W)), g.standard_normal((OC, IC, KH, KW))
    bias = g.standard_normal(OC)
    y = oracle.conv2d(x, w, stride=stride, pad=pad, bias=bias)
    # (a) the paper's decomposition: img2col transform + matmul (+ layout transform back)
    col = oracle.im2col(x, KH, KW, stride=stride, pad=pad)
    OH, OW = y.shape[2:]
    g2 = oracle.gemm(w.reshape(OC, -1), col, bias=bias, bias_axis=BIAS_PER_ROW)
    g2 = g2.reshape(OC, Nb, OH, OW).transpose(1, 0, 2, 3)
    assert oracle.rel_frobenius(y, g2) < 1e-15
    # (b) a library routine in float64
    ref = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), torch.from_numpy(bias), stride=stride,
                                     padding=pad).numpy()
    assert y.shape == ref.shape
    assert oracle.rel_frobenius(y, ref) < 1e-14


def test_conv_residual_and_relu_order():
    x, w = np.ones((1, 1, 2, 2)), -np.ones((1, 1, 1, 1))
    res = np.array([[[[0.5, 1.5], [2.0, 0.0]]]])
    y = oracle.conv2d(x, w, bias=np.array([0.25]), residual=res, relu=True)
    assert np.array_equal(y, np.array([[[[0.0, 0.75], [1.25, 0.0]]]]))


def _exact_conv(x, w, stride, pad, alpha, bias, residual, relu):
    """Direct convolution in exact rationals (integer-valued inputs), loops in another order than the oracle's."""
    Nb, IC, H, W = x.shape
    OC, _, KH, KW = w.shape
    OH = (H + 2 * pad[0] - KH) // stride[0] + 1
    OW = (W + 2 * pad[1] - KW) // stride[1] + 1
    out = np.empty((Nb, OC, OH, OW), dtype=object)
    for ow in range(OW):
        for oh in range(OH):
            for oc in range(OC):
                for n in range(Nb):
                    s = Fraction(0)
                    for kw in range(KW):
                        for kh in range(KH):
                            ih, iw = oh * stride[0] + kh - pad[0], ow * stride[1] + kw - pad[1]
                            if 0 <= ih < H and 0 <= iw < W:
                                for ic in range(IC):
                                    s += Fraction(int(x[n, ic, ih, iw])) * Fraction(int(w[oc, ic, kh, kw]))
                    v = Fraction(alpha) * s
                    if bias is not None:
                        v += Fraction(int(bias[oc]))
                    if residual is not None:
                        v += Fraction(int(residual[n, oc, oh, ow]))
                    if relu and v < 0:
                        v = Fraction(0)
                    out[n, oc, oh, ow] = v
    return out


@pytest.mark.parametrize("alpha", [0.25, -1.5, 0.0])
@pytest.mark.parametrize("flags", range(8))
def test_conv_alpha_scales_the_sum_before_bias_residual_and_relu(alpha, flags):
    """The scale of the fused epilogue multiplies the convolution sum only: exact rationals on integer data,
    for every combination of bias / residual / ReLU."""
    g = np.random.default_rng(17 + flags)
    x = g.integers(-4, 5, size=(2, 3, 5, 6)).astype(np.float64)
    w = g.integers(-3, 4, size=(4, 3, 3, 2)).astype(np.float64)
    stride, pad = (2, 1), (1, 1)
    bias = g.integers(-9, 10, size=4).astype(np.float64) if flags & 1 else None
    y0 = oracle.conv2d(x, w, stride=stride, pad=pad)
    res = g.integers(-9, 10, size=y0.shape).astype(np.float64) if flags & 2 else None
    relu = bool(flags & 4)
    y = oracle.conv2d(x, w, stride=stride, pad=pad, alpha=alpha, bias=bias, residual=res, relu=relu)
    exact = _exact_conv(x, w, stride, pad, alpha, bias, res, relu)
    assert y.shape == exact.shape
    for got, want in zip(y.ravel(), exact.ravel()):
        assert Fraction(float(got)) == want
    # and against alpha * (the unscaled convolution): alpha is a dyadic rational, so the product is exact
    v = alpha * y0
    if bias is not None:
        v = v + bias[None, :, None, None]
    if res is not None:
        v = v + res
    if relu:
        v = np.maximum(v, 0.0)
    assert np.array_equal(y, v)


# ---------------------------------------------------------------- input prologue
def test_input_prologue_relu_on_the_activation_operand():
    """Section 5.2: a fused prologue replaces every access of an input by f(access); f = ReLU on A (GEMM) or x (conv)."""
    # closed forms: a non-positive activation contributes nothing, a non-negative one is untouched
    M, N, K = 4, 5, 6
    bias = np.arange(N, dtype=np.float64) - 1.5
    C = oracle.gemm(-np.ones((M, K)), np.ones((K, N)), bias=bias, relu_input=True)
    assert np.array_equal(C, np.broadcast_to(bias, (M, N)))
    C = oracle.gemm(np.ones((M, K)), -np.ones((K, N)), relu_input=True)  # only A passes through f, B does not
    assert np.array_equal(C, np.full((M, N), -float(K)))
    A = np.array([[1.0, -2.0, 3.0, -4.0]])
    assert oracle.gemm(A, np.ones((4, 1)), relu_input=True)[0, 0] == 4.0   # 1 + 3
    assert oracle.gemm(A, np.ones((4, 1)), relu_input=False)[0, 0] == -2.0
    # exact rationals on integer data, all transposes, with an epilogue behind it
    g = np.random.default_rng(31)
    for transA in (False, True):
        for transB in (False, True):
            A = g.integers(-5, 6, size=(4, 3) if transA else (3, 4)).astype(np.float64)
            B = g.integers(-5, 6, size=(5, 4) if transB else (4, 5)).astype(np.float64)
            res = g.integers(-9, 10, size=(3, 5)).astype(np.float64)
            got = oracle.gemm(A, B, transA=transA, transB=transB, alpha=0.5, residual=res, relu=True, relu_input=True)
            Ap = [[max(int(v), 0) for v in row] for row in A]
            want = _exact_gemm(Ap, B, transA, transB, 0.5, None, BIAS_PER_COL, res, True)
            for i in range(3):
                for j in range(5):
                    assert Fraction(float(got[i, j])) == want[i][j]
    # a library routine: numpy's maximum and matmul in float64
    A, B = g.standard_normal((9, 17)), g.standard_normal((17, 8))
    assert oracle.rel_frobenius(oracle.gemm(A, B, relu_input=True), np.maximum(A, 0.0) @ B) < 1e-15
    Ab, Bb = g.standard_normal((3, 4, 6)), g.standard_normal((3, 6, 5))
    assert oracle.rel_frobenius(oracle.batched_gemm(Ab, Bb, relu_input=True), np.maximum(Ab, 0.0) @ Bb) < 1e-15
    # convolution: the activation is x; padding stays zero; torch in float64
    x, w = g.standard_normal((2, 3, 6, 5)), g.standard_normal((4, 3, 3, 3))
    y = oracle.conv2d(x, w, pad=(1, 1), relu_input=True)
    ref = torch.nn.functional.conv2d(torch.relu(torch.from_numpy(x)), torch.from_numpy(w), padding=1).numpy()
    assert oracle.rel_frobenius(y, ref) < 1e-14
    assert np.array_equal(oracle.conv2d(-np.abs(x), w, pad=(1, 1), bias=np.arange(4.0), relu_input=True),
                          np.broadcast_to(np.arange(4.0)[None, :, None, None], (2, 4, 6, 5)))


# ---------------------------------------------------------------- the error measure itself
def test_rel_frobenius():
    ref = np.array([[3.0, 4.0]])
    assert oracle.rel_frobenius(ref, ref) == 0.0
    assert abs(oracle.rel_frobenius(ref + np.array([[0.0, 0.5]]), ref) - 0.1) < 1e-15
    assert oracle.rel_frobenius(np.zeros(3), np.zeros(3)) == 0.0
    assert oracle.rel_frobenius(np.ones(3), np.zeros(3)) == float("inf")


def test_fp32_accumulation_bound_is_attainable():
    """A float32 running sum over K=4096 products of U(-1,1) data stays within the 1e-5 parity bound;
    a float16 running sum does not stay within 2e-3 -- so the bounds demand fp32 accumulation."""
    g = np.random.default_rng(11)
    K = 4096
    A = g.uniform(-1, 1, (8, K)).astype(np.float16)
    B = g.uniform(-1, 1, (K, 8)).astype(np.float16)
    ref = oracle.gemm(A, B)
    acc32 = np.zeros((8, 8), dtype=np.float32)
    acc16 = np.zeros((8, 8), dtype=np.float16)
    for k in range(K):
        p = np.outer(A[:, k].astype(np.float32), B[k].astype(np.float32))
        acc32 += p
        acc16 = (acc16.astype(np.float32) + p).astype(np.float16)
    assert oracle.rel_frobenius(acc32, ref) < 1e-5
    assert oracle.rel_frobenius(acc16, ref) > 2e-3


def test_head_split_is_the_stated_index_permutation():
    """Brute force over every element of a small case, indices written out by hand."""
    rng = np.random.default_rng(77)
    b, seq, heads, d = 2, 5, 3, 4
    C = rng.standard_normal((b * seq, heads * d))
    out = oracle.head_split(C, seq, d)
    assert out.shape == (b, heads, seq, d)
    for bi in range(b):
        for h in range(heads):
            for s_ in range(seq):
                for f in range(d):
                    assert out[bi, h, s_, f] == C[bi * seq + s_, h * d + f]
    with pytest.raises(ValueError):
        oracle.head_split(C, 4, d)
