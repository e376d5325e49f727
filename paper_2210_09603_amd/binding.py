"""ctypes binding over the C ABI in include/hidet_mi355x.h -- argument marshalling only.

Every function here has the name of the C entry point it forwards to.  Tensors are torch tensors on
the GPU; torch is used for device memory and the current HIP stream, nothing else.  There is no
fallback: if libhidet_mi355x.so has not been built, or a call returns a non-zero status, an
exception is raised.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhidet_mi355x.so")

HIDET_F32, HIDET_F16, HIDET_BF16 = 0, 1, 2
HIDET_BIAS_NONE, HIDET_BIAS_PER_COL, HIDET_BIAS_PER_ROW = 0, 1, 2
HIDET_ACT_NONE, HIDET_ACT_RELU = 0, 1
HIDET_MAP_PLAIN, HIDET_MAP_HEAD_SPLIT = 0, 1
HIDET_PROLOGUE_NONE, HIDET_PROLOGUE_RELU = 0, 1
HIDET_REDUCE_SUM, HIDET_REDUCE_MAX, HIDET_REDUCE_MEAN = 0, 1, 2

_DTYPES = {torch.float32: HIDET_F32, torch.float16: HIDET_F16, torch.bfloat16: HIDET_BF16}

_i32, _i64, _vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p


class hidet_epilogue_t(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("alpha", ctypes.c_float),
        ("bias", _vp),
        ("bias_axis", _i32),
        ("act", _i32),
        ("residual", _vp),
        ("ld_residual", _i64),
        ("batch_stride_residual", _i64),
        ("out_map", _i32),
        ("prologue", _i32),
        ("map_seq", _i64),
        ("map_head_dim", _i64),
    ]


class hidet_config_info_t(ctypes.Structure):
    _fields_ = [(n, _i32) for n in ("block_m", "block_n", "block_k", "waves_m", "waves_n", "mfma", "is_f32", "schedule",
                                    "stages", "lds_bytes", "waves_k")]


class HidetError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: status %d (%s)" % (where, status, lib().hidet_status_string(status).decode()))


EXPORTS = (
    "hidet_gemm", "hidet_batched_gemm", "hidet_conv2d_implicit_gemm", "hidet_gemm_cfg", "hidet_batched_gemm_cfg",
    "hidet_conv2d_implicit_gemm_cfg", "hidet_config_count", "hidet_config_info", "hidet_tune_gemm", "hidet_tune_conv2d",
    "hidet_tune_last_times", "hidet_tune_clear", "hidet_tune_save", "hidet_tune_load", "hidet_taskmap_count",
    "hidet_taskmap_info", "hidet_taskmap_tasks", "hidet_block_task", "hidet_status_string", "hidet_version",
    "hidet_kernel_launch_count", "hidet_probe_stream_bandwidth",
    "hidet_probe_mfma_peak", "hidet_probe_scratch_bytes", "hidet_probe_launch_floor", "hidet_splitk_workspace_bytes", "hidet_batched_gemm_splitk",
    "hidet_conv2d_implicit_gemm_splitk", "hidet_tune_gemm_splitk", "hidet_tune_conv2d_splitk", "hidet_reduce_rows",
    "hidet_softmax_rows", "hidet_host_div", "hidet_conv2d_splitk_workspace_bytes", "hidet_static_scratch_bytes",
    "hidet_batched_gemm_splitk_static", "hidet_conv2d_pack_weights", "hidet_conv2d_implicit_gemm_packed",
    "hidet_tune_conv2d_packed",
)

_lib = None


def lib():
    """The loaded shared library.  Raises if it has not been built (python -m paper_2210_09603_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP extension missing: %s (build it with `python -m paper_2210_09603_amd.build`)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        ep = ctypes.POINTER(hidet_epilogue_t)
        gemm_args = [_i32, _i32, _i32, _i32, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, ep, _vp]
        bgemm_args = [_i32, _i32, _i32, _i32, _i64, _i64, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _i64, _vp, _i64, _i64,
                      ep, _vp]
        conv_args = [_i32, _i32] + [_i64] * 11 + [_vp, _vp, _vp, ep, _vp]
        L.hidet_gemm.argtypes = gemm_args
        L.hidet_gemm_cfg.argtypes = [_i32] + gemm_args
        L.hidet_batched_gemm.argtypes = bgemm_args
        L.hidet_batched_gemm_cfg.argtypes = [_i32] + bgemm_args
        L.hidet_conv2d_implicit_gemm.argtypes = conv_args
        L.hidet_conv2d_implicit_gemm_cfg.argtypes = [_i32] + conv_args
        tune_tail = [_i32, ctypes.POINTER(_i32), ctypes.POINTER(ctypes.c_float)]
        L.hidet_tune_gemm.argtypes = bgemm_args + tune_tail
        L.hidet_tune_conv2d.argtypes = conv_args + tune_tail
        L.hidet_splitk_workspace_bytes.argtypes = [_i64, _i64, _i64, _i32]
        L.hidet_splitk_workspace_bytes.restype = _i64
        L.hidet_conv2d_splitk_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, _i32]
        L.hidet_conv2d_splitk_workspace_bytes.restype = _i64
        L.hidet_static_scratch_bytes.restype = _i64
        L.hidet_batched_gemm_splitk_static.argtypes = [_i32, _i32] + bgemm_args
        ws_args = [_vp, _i64, _vp]  # workspace, bytes, stream (replaces the trailing stream argument)
        L.hidet_batched_gemm_splitk.argtypes = [_i32, _i32] + bgemm_args[:-1] + ws_args
        L.hidet_conv2d_implicit_gemm_splitk.argtypes = [_i32, _i32] + conv_args[:-1] + ws_args
        tune_tail_sk = [_i32, ctypes.POINTER(_i32), ctypes.POINTER(_i32), ctypes.POINTER(ctypes.c_float)]
        L.hidet_conv2d_pack_weights.argtypes = [_i32, _i64, _i64, _i64, _i64, _vp, _vp, _vp]
        L.hidet_conv2d_implicit_gemm_packed.argtypes = [_i32, _i32] + conv_args[:-1] + ws_args
        L.hidet_tune_conv2d_packed.argtypes = conv_args[:-1] + ws_args + tune_tail_sk
        L.hidet_tune_gemm_splitk.argtypes = bgemm_args[:-1] + ws_args + tune_tail_sk
        L.hidet_tune_conv2d_splitk.argtypes = conv_args[:-1] + ws_args + tune_tail_sk
        L.hidet_host_div.argtypes = [_i64, _i32, ctypes.POINTER(_i32)]
        L.hidet_reduce_rows.argtypes = [_i32, _i32, _i32, _i64, _i64, _vp, _i64, _vp, _vp]
        L.hidet_softmax_rows.argtypes = [_i32, _i64, _i64, _vp, _i64, _vp, _i64, _vp]
        L.hidet_tune_last_times.argtypes = [ctypes.POINTER(ctypes.c_float), _i32]
        L.hidet_tune_clear.restype = None
        L.hidet_tune_save.argtypes = [ctypes.c_char_p]
        L.hidet_tune_load.argtypes = [ctypes.c_char_p]
        L.hidet_config_info.argtypes = [_i32, ctypes.POINTER(hidet_config_info_t)]
        L.hidet_taskmap_info.argtypes = [_i32, ctypes.c_char_p, _i32] + [ctypes.POINTER(_i32)] * 4
        L.hidet_taskmap_tasks.argtypes = [_i32, _i32, ctypes.POINTER(_i32), _i32]
        L.hidet_block_task.argtypes = [_i32] * 4 + [ctypes.POINTER(_i32)] * 2
        L.hidet_probe_mfma_peak.argtypes = [_i32, _i32, _vp, _i64, _vp, _i64, _vp, ctypes.POINTER(ctypes.c_float),
                                            ctypes.POINTER(ctypes.c_float)]
        L.hidet_probe_scratch_bytes.restype = _i64
        L.hidet_probe_launch_floor.argtypes = [_vp, _i32, ctypes.POINTER(ctypes.c_float)]
        L.hidet_probe_stream_bandwidth.argtypes = [_vp, _i64, _i32, _vp, ctypes.POINTER(ctypes.c_float)]
        L.hidet_status_string.argtypes = [_i32]
        L.hidet_status_string.restype = ctypes.c_char_p
        L.hidet_version.restype = ctypes.c_char_p
        L.hidet_kernel_launch_count.restype = ctypes.c_int64
        _lib = L
    return _lib


def _check(status, where):
    if status != 0:
        raise HidetError(status, where)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype(t):
    if t.dtype not in _DTYPES:
        raise TypeError("unsupported dtype %s" % t.dtype)
    return _DTYPES[t.dtype]


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _ld(t):
    """Leading dimension of a 2-D (or the last two dims of a 3-D) row-major tensor, in elements."""
    if t.stride(-1) != 1 and t.shape[-1] > 1:
        raise ValueError("innermost dimension must be contiguous")
    return t.stride(-2) if t.shape[-2] > 1 else max(t.shape[-1], 1)


def make_epilogue(alpha=1.0, bias=None, bias_axis=HIDET_BIAS_NONE, residual=None, relu=False, batched=False,
                  head_split=None, relu_input=False):
    """Build a hidet_epilogue_t (returns None for the identity epilogue).  head_split=(seq, head_dim) selects the
    [b][h][s][f] output index map; the residual (if any) is then a dense tensor of that shape.  A 3-D residual
    advances by its own batch stride (`batched` is accepted for older callers and ignored).  relu_input: the fused
    prologue, ReLU on the activation operand (A of a GEMM, x of a convolution) as it is loaded."""
    if alpha == 1.0 and bias is None and residual is None and not relu and head_split is None and not relu_input:
        return None
    e = hidet_epilogue_t()
    e.struct_size = ctypes.sizeof(hidet_epilogue_t)
    e.alpha = alpha
    # the struct holds raw device addresses: keep the tensors alive as long as it lives (an asynchronous kernel
    # reads them after the call has returned)
    e._keep = (bias, residual)
    e.bias = bias.data_ptr() if bias is not None else None
    e.bias_axis = bias_axis if bias is not None else HIDET_BIAS_NONE
    e.act = HIDET_ACT_RELU if relu else HIDET_ACT_NONE
    e.prologue = HIDET_PROLOGUE_RELU if relu_input else HIDET_PROLOGUE_NONE
    if head_split is not None:
        e.out_map = HIDET_MAP_HEAD_SPLIT
        e.map_seq, e.map_head_dim = head_split
    if residual is not None:
        e.residual = residual.data_ptr()
        if head_split is None:
            e.ld_residual = _ld(residual)
            e.batch_stride_residual = residual.stride(0) if (residual.dim() == 3 and residual.shape[0] > 1) else 0
    return e


def _epi_ref(e):
    return ctypes.byref(e) if e is not None else None


def _gemm_dims(A, B, transA, transB):
    M, K = (A.shape[-1], A.shape[-2]) if transA else (A.shape[-2], A.shape[-1])
    Kb, N = (B.shape[-1], B.shape[-2]) if transB else (B.shape[-2], B.shape[-1])
    if K != Kb:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, Kb))
    return M, N, K


def hidet_gemm(A, B, C, transA=False, transB=False, epilogue=None, stream=None, config=-1):
    """C[M,N] = epilogue(op(A) . op(B)); A, B, C are 2-D GPU tensors (row-major, any leading dimension)."""
    M, N, K = _gemm_dims(A, B, transA, transB)
    if epilogue is not None and epilogue.out_map == HIDET_MAP_HEAD_SPLIT:
        want = (M // epilogue.map_seq, N // epilogue.map_head_dim, epilogue.map_seq, epilogue.map_head_dim)
        if tuple(C.shape) != want or not C.is_contiguous():
            raise ValueError("C must be a dense tensor of shape %s" % (want,))
        st = lib().hidet_gemm_cfg(config, _dtype(A), _dtype(C), int(transA), int(transB), M, N, K, _ptr(A), _ld(A), _ptr(B),
                                  _ld(B), _ptr(C), N, _epi_ref(epilogue), _stream(stream))
        _check(st, "hidet_gemm")
        return
    if tuple(C.shape) != (M, N):
        raise ValueError("C has shape %s, expected %s" % (tuple(C.shape), (M, N)))
    st = lib().hidet_gemm_cfg(config, _dtype(A), _dtype(C), int(transA), int(transB), M, N, K, _ptr(A), _ld(A), _ptr(B),
                              _ld(B), _ptr(C), _ld(C), _epi_ref(epilogue), _stream(stream))
    _check(st, "hidet_gemm")


def _bstride(t):
    return t.stride(0) if t.shape[0] > 1 else t.shape[-2] * _ld(t)


def hidet_batched_gemm(A, B, C, transA=False, transB=False, epilogue=None, stream=None, config=-1):
    """Batched form: A, B, C are 3-D GPU tensors [batch, rows, cols]."""
    M, N, K = _gemm_dims(A, B, transA, transB)
    batch = A.shape[0]
    if B.shape[0] != batch or tuple(C.shape) != (batch, M, N):
        raise ValueError("batch/shape mismatch")
    st = lib().hidet_batched_gemm_cfg(config, _dtype(A), _dtype(C), int(transA), int(transB), batch, M, N, K, _ptr(A),
                                      _ld(A), _bstride(A), _ptr(B), _ld(B), _bstride(B), _ptr(C), _ld(C), _bstride(C),
                                      _epi_ref(epilogue), _stream(stream))
    _check(st, "hidet_batched_gemm")


def _conv_args(x, w, y, stride, pad):
    for t in (x, w, y):
        if not t.is_contiguous():
            raise ValueError("conv tensors must be dense NCHW / OIHW")
    Nb, IC, H, W = x.shape
    OC, IC2, KH, KW = w.shape
    if IC != IC2:
        raise ValueError("channel mismatch")
    return [_dtype(x), _dtype(y), Nb, IC, H, W, OC, KH, KW, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ptr(w), _ptr(y)]


def conv_out_shape(x_shape, w_shape, stride, pad):
    Nb, _, H, W = x_shape
    OC, _, KH, KW = w_shape
    return (Nb, OC, (H + 2 * pad[0] - KH) // stride[0] + 1, (W + 2 * pad[1] - KW) // stride[1] + 1)


def hidet_conv2d_implicit_gemm(x, w, y, stride=(1, 1), pad=(0, 0), epilogue=None, stream=None, config=-1):
    """y = epilogue(conv2d(x, w)), NCHW / OIHW / NCHW dense GPU tensors; bias (if any) is per output channel."""
    if tuple(y.shape) != conv_out_shape(x.shape, w.shape, stride, pad):
        raise ValueError("y has the wrong shape")
    st = lib().hidet_conv2d_implicit_gemm_cfg(config, *_conv_args(x, w, y, stride, pad), _epi_ref(epilogue),
                                              _stream(stream))
    _check(st, "hidet_conv2d_implicit_gemm")


def hidet_tune_gemm(A, B, C, transA=False, transB=False, epilogue=None, stream=None, iters=10):
    """Enumerate the schedule space on this (possibly batched) problem; returns (best_config, best_us)."""
    if A.dim() == 2:
        A, B, C = A.unsqueeze(0), B.unsqueeze(0), C.unsqueeze(0)
    M, N, K = _gemm_dims(A, B, transA, transB)
    batch = A.shape[0]
    best, us = _i32(-1), ctypes.c_float(0.0)
    st = lib().hidet_tune_gemm(_dtype(A), _dtype(C), int(transA), int(transB), batch, M, N, K, _ptr(A), _ld(A),
                               _bstride(A), _ptr(B), _ld(B), _bstride(B), _ptr(C), _ld(C), _bstride(C),
                               _epi_ref(epilogue), _stream(stream), iters, ctypes.byref(best), ctypes.byref(us))
    _check(st, "hidet_tune_gemm")
    return best.value, us.value


def hidet_tune_conv2d(x, w, y, stride=(1, 1), pad=(0, 0), epilogue=None, stream=None, iters=10):
    best, us = _i32(-1), ctypes.c_float(0.0)
    st = lib().hidet_tune_conv2d(*_conv_args(x, w, y, stride, pad), _epi_ref(epilogue), _stream(stream), iters,
                                 ctypes.byref(best), ctypes.byref(us))
    _check(st, "hidet_tune_conv2d")
    return best.value, us.value


def hidet_splitk_workspace_bytes(batch, M, N, k_slices):
    return lib().hidet_splitk_workspace_bytes(batch, M, N, k_slices)


def hidet_conv2d_splitk_workspace_bytes(y_shape, k_slices):
    """Workspace bytes of the K-parallel convolution that produces y [Nb, OC, OH, OW]."""
    Nb, OC, OH, OW = y_shape
    return lib().hidet_conv2d_splitk_workspace_bytes(Nb, OC, OH, OW, k_slices)


def hidet_static_scratch_bytes():
    return lib().hidet_static_scratch_bytes()


def hidet_batched_gemm_splitk_static(A, B, C, k_slices=0, transA=False, transB=False, epilogue=None, stream=None, config=-1):
    """hidet_batched_gemm_splitk with the library's static scratch array as the workspace (allocates nothing)."""
    if A.dim() == 2:
        A, B, C = A.unsqueeze(0), B.unsqueeze(0), C.unsqueeze(0)
    M, N, K = _gemm_dims(A, B, transA, transB)
    batch = A.shape[0]
    if B.shape[0] != batch or tuple(C.shape) != (batch, M, N):
        raise ValueError("batch/shape mismatch")
    st = lib().hidet_batched_gemm_splitk_static(config, k_slices, _dtype(A), _dtype(C), int(transA), int(transB), batch, M, N,
                                                K, _ptr(A), _ld(A), _bstride(A), _ptr(B), _ld(B), _bstride(B), _ptr(C),
                                                _ld(C), _bstride(C), _epi_ref(epilogue), _stream(stream))
    _check(st, "hidet_batched_gemm_splitk_static")


def _ws(workspace):
    """(pointer, bytes) of a workspace tensor (any dtype, contiguous) or (NULL, 0)."""
    if workspace is None:
        return None, 0
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def hidet_batched_gemm_splitk(A, B, C, workspace, k_slices=0, transA=False, transB=False, epilogue=None, stream=None,
                              config=-1):
    """K-parallel form of hidet_batched_gemm (2-D tensors are taken as batch 1); workspace is a GPU tensor."""
    if A.dim() == 2:
        A, B, C = A.unsqueeze(0), B.unsqueeze(0), C.unsqueeze(0)
    M, N, K = _gemm_dims(A, B, transA, transB)
    batch = A.shape[0]
    if B.shape[0] != batch or tuple(C.shape) != (batch, M, N):
        raise ValueError("batch/shape mismatch")
    wp, wb = _ws(workspace)
    st = lib().hidet_batched_gemm_splitk(config, k_slices, _dtype(A), _dtype(C), int(transA), int(transB), batch, M, N, K,
                                         _ptr(A), _ld(A), _bstride(A), _ptr(B), _ld(B), _bstride(B), _ptr(C), _ld(C),
                                         _bstride(C), _epi_ref(epilogue), wp, wb, _stream(stream))
    _check(st, "hidet_batched_gemm_splitk")


def hidet_conv2d_implicit_gemm_splitk(x, w, y, workspace, k_slices=0, stride=(1, 1), pad=(0, 0), epilogue=None,
                                      stream=None, config=-1):
    """K-parallel form of hidet_conv2d_implicit_gemm; workspace is a GPU tensor."""
    if tuple(y.shape) != conv_out_shape(x.shape, w.shape, stride, pad):
        raise ValueError("y has the wrong shape")
    wp, wb = _ws(workspace)
    st = lib().hidet_conv2d_implicit_gemm_splitk(config, k_slices, *_conv_args(x, w, y, stride, pad), _epi_ref(epilogue),
                                                 wp, wb, _stream(stream))
    _check(st, "hidet_conv2d_implicit_gemm_splitk")


def hidet_conv2d_pack_weights(w, w_packed=None, stream=None):
    """OIHW weights -> the tap-major order [OC][KH][KW][IC] of the packed convolution; returns the packed tensor."""
    if not w.is_contiguous():
        raise ValueError("weights must be dense OIHW")
    OC, IC, KH, KW = w.shape
    if w_packed is None:
        w_packed = torch.empty((OC, KH, KW, IC), dtype=w.dtype, device=w.device)
    if w_packed.numel() != w.numel() or not w_packed.is_contiguous() or w_packed.dtype != w.dtype:
        raise ValueError("w_packed must be a dense tensor of the same dtype and element count")
    _check(lib().hidet_conv2d_pack_weights(_dtype(w), OC, IC, KH, KW, _ptr(w), _ptr(w_packed), _stream(stream)),
           "hidet_conv2d_pack_weights")
    return w_packed


def _packed_conv_args(x, w_packed, y, stride, pad):
    for t in (x, w_packed, y):
        if not t.is_contiguous():
            raise ValueError("conv tensors must be dense")
    Nb, IC, H, W = x.shape
    OC, KH, KW, IC2 = w_packed.shape
    if IC != IC2:
        raise ValueError("channel mismatch")
    if tuple(y.shape) != conv_out_shape(x.shape, (OC, IC, KH, KW), stride, pad):
        raise ValueError("y has the wrong shape")
    return [_dtype(x), _dtype(y), Nb, IC, H, W, OC, KH, KW, stride[0], stride[1], pad[0], pad[1], _ptr(x), _ptr(w_packed),
            _ptr(y)]


def hidet_conv2d_implicit_gemm_packed(x, w_packed, y, stride=(1, 1), pad=(0, 0), epilogue=None, stream=None, config=-1,
                                      k_slices=0, workspace=None):
    """The convolution from weights repacked by hidet_conv2d_pack_weights ([OC][KH][KW][IC])."""
    wp, wb = _ws(workspace)
    st = lib().hidet_conv2d_implicit_gemm_packed(config, k_slices, *_packed_conv_args(x, w_packed, y, stride, pad),
                                                 _epi_ref(epilogue), wp, wb, _stream(stream))
    _check(st, "hidet_conv2d_implicit_gemm_packed")


def hidet_tune_conv2d_packed(x, w_packed, y, workspace=None, stride=(1, 1), pad=(0, 0), epilogue=None, stream=None, iters=10):
    best, sl, us = _i32(-1), _i32(1), ctypes.c_float(0.0)
    wp, wb = _ws(workspace)
    st = lib().hidet_tune_conv2d_packed(*_packed_conv_args(x, w_packed, y, stride, pad), _epi_ref(epilogue), wp, wb,
                                        _stream(stream), iters, ctypes.byref(best), ctypes.byref(sl), ctypes.byref(us))
    _check(st, "hidet_tune_conv2d_packed")
    return best.value, sl.value, us.value


def hidet_tune_gemm_splitk(A, B, C, workspace, transA=False, transB=False, epilogue=None, stream=None, iters=10):
    """Enumerate configurations x slice counts; returns (best_config, best_slices, best_us)."""
    if A.dim() == 2:
        A, B, C = A.unsqueeze(0), B.unsqueeze(0), C.unsqueeze(0)
    M, N, K = _gemm_dims(A, B, transA, transB)
    batch = A.shape[0]
    best, sl, us = _i32(-1), _i32(1), ctypes.c_float(0.0)
    wp, wb = _ws(workspace)
    st = lib().hidet_tune_gemm_splitk(_dtype(A), _dtype(C), int(transA), int(transB), batch, M, N, K, _ptr(A), _ld(A),
                                      _bstride(A), _ptr(B), _ld(B), _bstride(B), _ptr(C), _ld(C), _bstride(C),
                                      _epi_ref(epilogue), wp, wb, _stream(stream), iters, ctypes.byref(best),
                                      ctypes.byref(sl), ctypes.byref(us))
    _check(st, "hidet_tune_gemm_splitk")
    return best.value, sl.value, us.value


def hidet_tune_conv2d_splitk(x, w, y, workspace, stride=(1, 1), pad=(0, 0), epilogue=None, stream=None, iters=10):
    best, sl, us = _i32(-1), _i32(1), ctypes.c_float(0.0)
    wp, wb = _ws(workspace)
    st = lib().hidet_tune_conv2d_splitk(*_conv_args(x, w, y, stride, pad), _epi_ref(epilogue), wp, wb, _stream(stream),
                                        iters, ctypes.byref(best), ctypes.byref(sl), ctypes.byref(us))
    _check(st, "hidet_tune_conv2d_splitk")
    return best.value, sl.value, us.value


def _rows_view(t):
    """[..., cols] tensor whose leading axes collapse to one row axis with a single stride -> (rows, cols, ld)."""
    if t.dim() < 1:
        raise ValueError("need at least one axis")
    if t.dim() == 1:
        return 1, t.shape[0], max(t.shape[0], 1)
    v = t if t.dim() == 2 else (t.view(-1, t.shape[-1]) if t.is_contiguous() else None)
    if v is None:
        raise ValueError("leading axes must be collapsible (pass a 2-D view)")
    return v.shape[0], v.shape[1], _ld(v)


def hidet_reduce_rows(x, y, op=HIDET_REDUCE_SUM, stream=None):
    """y[i] = reduce over the last axis of x; y has one element per row, dtype of x or float32."""
    rows, cols, ld = _rows_view(x)
    if y.numel() != rows or not y.is_contiguous():
        raise ValueError("y must be a dense tensor with one element per row")
    st = lib().hidet_reduce_rows(_dtype(x), _dtype(y), op, rows, cols, _ptr(x), ld, _ptr(y), _stream(stream))
    _check(st, "hidet_reduce_rows")


def hidet_softmax_rows(x, y, stream=None):
    """y = softmax of x along the last axis (same shape and dtype; y may be x itself)."""
    if x.shape != y.shape or x.dtype != y.dtype:
        raise ValueError("x and y must agree in shape and dtype")
    rows, cols, ldx = _rows_view(x)
    _, _, ldy = _rows_view(y)
    st = lib().hidet_softmax_rows(_dtype(x), rows, cols, _ptr(x), ldx, _ptr(y), ldy, _stream(stream))
    _check(st, "hidet_softmax_rows")


def hidet_tune_last_times():
    n = lib().hidet_config_count()
    buf = (ctypes.c_float * n)()
    lib().hidet_tune_last_times(buf, n)
    return list(buf)


def hidet_tune_clear():
    lib().hidet_tune_clear()


def hidet_tune_save(path):
    _check(lib().hidet_tune_save(path.encode()), "hidet_tune_save")


def hidet_tune_load(path):
    _check(lib().hidet_tune_load(path.encode()), "hidet_tune_load")


def hidet_config_count():
    return lib().hidet_config_count()


def hidet_config_info(config):
    info = hidet_config_info_t()
    _check(lib().hidet_config_info(config, ctypes.byref(info)), "hidet_config_info")
    return {n: getattr(info, n) for n, _ in hidet_config_info_t._fields_}


def hidet_taskmap_count():
    return lib().hidet_taskmap_count()


def hidet_taskmap_info(index):
    buf = ctypes.create_string_buffer(256)
    w, s0, s1, t = _i32(), _i32(), _i32(), _i32()
    _check(lib().hidet_taskmap_info(index, buf, 256, ctypes.byref(w), ctypes.byref(s0), ctypes.byref(s1), ctypes.byref(t)),
           "hidet_taskmap_info")
    return dict(expr=buf.value.decode(), workers=w.value, shape=(s0.value, s1.value), tasks=t.value)


def hidet_taskmap_tasks(index, worker):
    info = hidet_taskmap_info(index)
    buf = (_i32 * (2 * info["tasks"]))()
    _check(lib().hidet_taskmap_tasks(index, worker, buf, info["tasks"]), "hidet_taskmap_tasks")
    return [(buf[2 * q], buf[2 * q + 1]) for q in range(info["tasks"])]


def hidet_block_task(tiles_m, tiles_n, group, w):
    i, j = _i32(), _i32()
    _check(lib().hidet_block_task(tiles_m, tiles_n, group, w, ctypes.byref(i), ctypes.byref(j)), "hidet_block_task")
    return i.value, j.value


def hidet_probe_launch_floor(iters=1000, stream=None):
    """Microseconds per launch of an empty kernel (back-to-back launches on one stream)."""
    us = ctypes.c_float(0.0)
    _check(lib().hidet_probe_launch_floor(_stream(stream), iters, ctypes.byref(us)), "hidet_probe_launch_floor")
    return us.value


def hidet_probe_mfma_peak(sample, mfma=16, stream=None):
    """MFMA-only ceiling on operands taken from `sample` (a GPU tensor of the input dtype); returns (TFLOP/s, sclk MHz)."""
    n = lib().hidet_probe_scratch_bytes()
    scratch = torch.empty(n, dtype=torch.uint8, device=sample.device)
    tf, mhz = ctypes.c_float(0.0), ctypes.c_float(0.0)
    flat = sample.reshape(-1)
    st = lib().hidet_probe_mfma_peak(_dtype(sample), mfma, _ptr(flat), flat.numel() * flat.element_size(), _ptr(scratch), n,
                                     _stream(stream), ctypes.byref(tf), ctypes.byref(mhz))
    _check(st, "hidet_probe_mfma_peak")
    return tf.value, mhz.value


def hidet_probe_stream_bandwidth(buffer, mode, stream=None):
    """GB/s of a plain read (mode 0), write (1) or copy (2) kernel walking over `buffer` (a GPU tensor, ideally 1 GiB)."""
    out = ctypes.c_float(0.0)
    flat = buffer.reshape(-1)
    _check(lib().hidet_probe_stream_bandwidth(_ptr(flat), flat.numel() * flat.element_size(), mode, _stream(stream),
                                              ctypes.byref(out)), "hidet_probe_stream_bandwidth")
    return out.value


def hidet_version():
    return lib().hidet_version().decode()


def hidet_kernel_launch_count():
    return int(lib().hidet_kernel_launch_count())
