"""CPU oracle for the fused GEMM / batched GEMM / conv2d hot path.

TEST INFRASTRUCTURE ONLY: only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import this package.  It shares no code with the HIP path and never
imports it.

* ``gemm`` / ``batched_gemm`` / ``conv2d`` wrap the plain C loops in ``oracle.c`` (matmul
  definition of Section 2.3 of the paper; convolution as the definition that img2col + matmul,
  Section 5.2, must reproduce; elementwise epilogue of Section 4.2).  Arithmetic is IEEE double;
  inputs are widened exactly from whatever dtype they arrive in; outputs stay float64.
* ``head_split`` is the reshape + transpose of the reshape-matmul-transpose sub-graph of Section 3.2,
  written with numpy's reshape/transpose (an index permutation, no arithmetic).
* ``oracle.taskmap`` holds the task-mapping definitions of Section 5.1 in pure Python.
* ``rel_frobenius`` is the error measure used by every parity test.
"""
import ctypes
import os

import numpy as np

from .build import LIB, build_oracle

BIAS_NONE, BIAS_PER_COL, BIAS_PER_ROW = 0, 1, 2

_lib = None
_i64 = ctypes.c_int64
_dp = ctypes.POINTER(ctypes.c_double)


class _Epilogue(ctypes.Structure):
    _fields_ = [
        ("alpha", ctypes.c_double),
        ("bias", _dp),
        ("bias_axis", ctypes.c_int),
        ("residual", _dp),
        ("ld_residual", _i64),
        ("relu", ctypes.c_int),
    ]


def load():
    """Load liboracle.so, compiling it first when it is missing or older than its source."""
    global _lib
    if _lib is None:
        build_oracle(force=False)
        lib = ctypes.CDLL(LIB)
        ep = ctypes.POINTER(_Epilogue)
        lib.oracle_gemm_element.restype = ctypes.c_double
        lib.oracle_gemm_element.argtypes = [ctypes.c_int, ctypes.c_int, _i64, _dp, _i64, _dp, _i64, ep, _i64, _i64]
        lib.oracle_gemm_rows.restype = ctypes.c_int
        lib.oracle_gemm_rows.argtypes = [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _dp, _i64, _dp, _i64, _dp, _i64,
                                         ep, _i64, _i64]
        lib.oracle_batched_gemm.restype = ctypes.c_int
        lib.oracle_batched_gemm.argtypes = [ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _i64, _dp, _i64, _i64, _dp,
                                            _i64, _i64, _dp, _i64, _i64, ep, _i64]
        lib.oracle_conv2d_direct.restype = ctypes.c_int
        lib.oracle_conv2d_direct.argtypes = [_i64] * 11 + [_dp, _dp, _dp, ep]
        lib.oracle_im2col.restype = None
        lib.oracle_im2col.argtypes = [_i64] * 10 + [_dp, _dp]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(load().oracle_num_threads())


def _f64(a):
    """Exact widening to a C-contiguous float64 array (fp16, fp32 and fp64 all embed in fp64)."""
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _ptr(a):
    return a.ctypes.data_as(_dp)


def _make_epilogue(alpha, bias, bias_axis, residual, relu, keep):
    if alpha == 1.0 and bias is None and residual is None and not relu:
        return None
    e = _Epilogue()
    e.alpha = float(alpha)
    e.bias_axis = BIAS_NONE
    if bias is not None:
        b = _f64(bias).reshape(-1)
        keep.append(b)
        e.bias = _ptr(b)
        e.bias_axis = int(bias_axis)
        if e.bias_axis not in (BIAS_PER_COL, BIAS_PER_ROW):
            raise ValueError("bias given without a bias axis")
    if residual is not None:
        r = _f64(residual)
        keep.append(r)
        e.residual = _ptr(r)
        e.ld_residual = r.shape[-1]
    e.relu = 1 if relu else 0
    keep.append(e)
    return ctypes.byref(e)


def input_relu(x):
    """The fused input prologue (Section 5.2: a prologue replaces every access X[i] of an input of the anchor
    operator by f(X[i]); its example scales the accessed element): here f is the ReLU that precedes a matmul or a
    convolution in a network, f(v) = 0 for v < 0, else v.  Every access is replaced, so applying f to the whole
    operand first is the same computation -- which is what the unfused graph does."""
    x = _f64(x)
    return np.where(x < 0.0, 0.0, x)


def _check_bias(bias, bias_axis, M, N):
    if bias is not None:
        want = N if bias_axis == BIAS_PER_COL else M
        if np.asarray(bias).size != want:
            raise ValueError("bias length %d, expected %d" % (np.asarray(bias).size, want))


def gemm(A, B, transA=False, transB=False, alpha=1.0, bias=None, bias_axis=BIAS_PER_COL, residual=None, relu=False,
         rows=None, relu_input=False):
    """C = Epi(op(A) . op(B)) in float64.  A is stored [M,K] ([K,M] if transA); B [K,N] ([N,K] if transB).

    ``rows=(r0, r1)`` computes only that row range (the rest of the returned array is zero).
    ``relu_input``: the input prologue on the activation operand A (see input_relu).
    """
    A, B = _f64(A), _f64(B)
    if relu_input:
        A = input_relu(A)
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    Kb, N = (B.shape[1], B.shape[0]) if transB else B.shape
    if K != Kb:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, Kb))
    _check_bias(bias, bias_axis, M, N)
    if residual is not None and tuple(np.asarray(residual).shape) != (M, N):
        raise ValueError("residual shape")
    C = np.zeros((M, N), dtype=np.float64)
    keep = []
    epi = _make_epilogue(alpha, bias, bias_axis, residual, relu, keep)
    r0, r1 = (0, M) if rows is None else rows
    if M and N:
        rc = load().oracle_gemm_rows(int(transA), int(transB), M, N, K, _ptr(A), max(A.shape[1], 1), _ptr(B),
                                     max(B.shape[1], 1), _ptr(C), max(N, 1), epi, r0, r1)
        if rc:
            raise MemoryError("oracle_gemm_rows")
    return C


def gemm_element(A, B, i, j, transA=False, transB=False, alpha=1.0, bias=None, bias_axis=BIAS_PER_COL, residual=None,
                 relu=False):
    """One output element as a literal dot product over k (A, B must already be float64 arrays)."""
    if A.dtype != np.float64 or B.dtype != np.float64 or not A.flags.c_contiguous or not B.flags.c_contiguous:
        raise ValueError("gemm_element wants contiguous float64 inputs (widen once, outside the sampling loop)")
    K = A.shape[0] if transA else A.shape[1]
    keep = []
    epi = _make_epilogue(alpha, bias, bias_axis, residual, relu, keep)
    return float(load().oracle_gemm_element(int(transA), int(transB), K, _ptr(A), A.shape[1], _ptr(B), B.shape[1], epi,
                                            int(i), int(j)))


def batched_gemm(A, B, transA=False, transB=False, alpha=1.0, bias=None, bias_axis=BIAS_PER_COL, residual=None,
                 relu=False, relu_input=False):
    """Independent GEMMs over the leading batch axis of A [b,..], B [b,..] (and residual [b,M,N])."""
    A, B = _f64(A), _f64(B)
    if relu_input:
        A = input_relu(A)
    batch = A.shape[0]
    if B.shape[0] != batch:
        raise ValueError("batch sizes differ")
    M, K = (A.shape[2], A.shape[1]) if transA else A.shape[1:]
    Kb, N = (B.shape[2], B.shape[1]) if transB else B.shape[1:]
    if K != Kb:
        raise ValueError("inner dimensions differ")
    _check_bias(bias, bias_axis, M, N)
    if residual is not None and tuple(np.asarray(residual).shape) != (batch, M, N):
        raise ValueError("residual shape")
    C = np.zeros((batch, M, N), dtype=np.float64)
    keep = []
    epi = _make_epilogue(alpha, bias, bias_axis, residual, relu, keep)
    if batch and M and N:
        rc = load().oracle_batched_gemm(int(transA), int(transB), batch, M, N, K, _ptr(A), max(A.shape[2], 1),
                                        A.shape[1] * A.shape[2], _ptr(B), max(B.shape[2], 1), B.shape[1] * B.shape[2],
                                        _ptr(C), max(N, 1), M * N, epi, M * N)
        if rc:
            raise MemoryError("oracle_batched_gemm")
    return C


def conv_out_size(H, KH, stride, pad):
    return (H + 2 * pad - KH) // stride + 1


def conv2d(x, w, stride=(1, 1), pad=(0, 0), alpha=1.0, bias=None, residual=None, relu=False, relu_input=False):
    """Direct NCHW convolution (cross-correlation, zero padding) with per-output-channel bias, in float64.
    ``relu_input``: the input prologue on the activation operand x (see input_relu)."""
    x, w = _f64(x), _f64(w)
    if relu_input:
        x = input_relu(x)
    Nb, IC, H, W = x.shape
    OC, IC2, KH, KW = w.shape
    if IC != IC2:
        raise ValueError("channel mismatch")
    OH, OW = conv_out_size(H, KH, stride[0], pad[0]), conv_out_size(W, KW, stride[1], pad[1])
    y = np.zeros((Nb, OC, max(OH, 0), max(OW, 0)), dtype=np.float64)
    if bias is not None and np.asarray(bias).size != OC:
        raise ValueError("bias length")
    if residual is not None and tuple(np.asarray(residual).shape) != y.shape:
        raise ValueError("residual shape")
    keep = []
    epi = _make_epilogue(alpha, bias, BIAS_PER_ROW, residual, relu, keep)
    if y.size:
        load().oracle_conv2d_direct(Nb, IC, H, W, OC, KH, KW, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ptr(w),
                                    _ptr(y), epi)
    return y


def im2col(x, KH, KW, stride=(1, 1), pad=(0, 0)):
    """Explicit img2col matrix [IC*KH*KW, Nb*OH*OW]; only used to pin conv2d against img2col + gemm."""
    x = _f64(x)
    Nb, IC, H, W = x.shape
    OH, OW = conv_out_size(H, KH, stride[0], pad[0]), conv_out_size(W, KW, stride[1], pad[1])
    col = np.zeros((IC * KH * KW, Nb * OH * OW), dtype=np.float64)
    load().oracle_im2col(Nb, IC, H, W, KH, KW, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ptr(col))
    return col


def head_split(C, seq, head_dim):
    """[b*seq + s][h*head_dim + f] -> [b][h][s][f]: what a transformer does to the output of its projection
    matmuls (Section 3.2, reshape-matmul-transpose); the HIP path fuses it into the store."""
    M, N = C.shape
    if M % seq or N % head_dim:
        raise ValueError("seq must divide M and head_dim must divide N")
    return np.ascontiguousarray(C.reshape(M // seq, seq, N // head_dim, head_dim).transpose(0, 2, 1, 3))


def rel_frobenius(got, ref) -> float:
    """||got - ref||_F / ||ref||_F in float64 (0 when both are all-zero, inf when only ref is)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if got.shape != ref.shape:
        raise ValueError("shape mismatch %s vs %s" % (got.shape, ref.shape))
    num = float(np.sqrt(np.sum((got - ref) ** 2)))
    den = float(np.sqrt(np.sum(ref ** 2)))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den
