"""Shared helpers of the GPU parity tests: host <-> device conversion and the comparison itself."""
import numpy as np
import torch

import oracle
from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 2e-3}  # max relative Frobenius error (the stated parity bound)
TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def output_rounding_floor(ref, dtype):
    """Relative Frobenius error of the exact result rounded once (RNE) to the output dtype: no implementation
    that emits `dtype` can do better.  For bf16 this floor is about 1.5e-3 on large tensors and fluctuates
    above the 2e-3 bound on tensors of a few dozen elements."""
    if dtype == "f32":
        return 0.0
    return oracle.rel_frobenius(wl.widen(wl.to_storage(ref.astype(np.float32), dtype), dtype), ref)


def within_bound(err, ref, dtype):
    """The parity bar: the stated bound, or (tiny bf16/fp16 outputs only) 10 % above the floor set by the
    output rounding itself, whichever is larger."""
    return err <= max(TOL[dtype], 1.1 * output_rounding_floor(ref, dtype) + 1e-5)


# Per-element parity bound.  A relative Frobenius norm over millions of outputs hides a single wrong element, so
# every comparison also bounds each element on its own:
#     |got - ref| <= REL * |ref| + ACC * scale + FLOOR
#   REL    twice the half-ulp of the one RNE rounding to the output type (2^-11 fp16, 2^-8 bf16, 2^-24 fp32);
#   scale  |alpha| * ||A_i||_2 * ||B_j||_2 + |bias| + |residual|: what the fp32 accumulation error is proportional
#          to (Cauchy-Schwarz bound on sum |a_k b_k|);  ACC = 1e-5 for K up to 4096 and grows with sqrt(K) beyond --
#          a random-walk fp32 sum of K terms errs by about sqrt(K) * 2^-24 of the term magnitude, far below that;
#   FLOOR  the spacing of fp16 subnormals (outputs below 6.1e-5 are rounded on an absolute grid).
ELEM_REL = {"f32": 2.0 ** -22, "f16": 2.0 ** -10, "bf16": 2.0 ** -7}
ELEM_FLOOR = {"f32": 1e-30, "f16": 2.0 ** -24, "bf16": 1e-30}


def acc_coeff(K):
    return 1e-5 * max(1.0, (K / 4096.0) ** 0.5)


def elementwise_violations(got, ref, scale, dtype, K):
    """Number of elements outside the per-element bound, and the worst ratio error / bound."""
    bound = ELEM_REL[dtype] * np.abs(ref) + acc_coeff(K) * scale + ELEM_FLOOR[dtype]
    ratio = np.abs(got - ref) / bound
    return int(np.count_nonzero(~(ratio <= 1.0))), float(np.nanmax(ratio)) if ratio.size else 0.0


def assert_elementwise(got, ref, scale, dtype, K, what=""):
    bad, worst = elementwise_violations(got, ref, scale, dtype, K)
    assert bad == 0, "%s: %d of %d elements outside the per-element bound (worst %.2f x bound)" % (what, bad, ref.size, worst)
    return worst


def gemm_scale(A64, B64, transA, transB, alpha, bias=None, bias_axis=None, residual=None):
    """|alpha| * ||row i of op(A)|| * ||column j of op(B)|| + |bias| + |residual| for every output element."""
    na = np.sqrt((A64 * A64).sum(axis=0 if transA else 1))
    nb = np.sqrt((B64 * B64).sum(axis=1 if transB else 0))
    s = abs(alpha) * np.outer(na, nb)
    if bias is not None:
        s = s + (np.abs(bias)[:, None] if bias_axis == "row" else np.abs(bias)[None, :])
    if residual is not None:
        s = s + np.abs(residual)
    return s


def conv_scale(x64, w64, stride, pad, alpha, bias=None, residual=None):
    """The same for a convolution: ||w[oc]|| * ||receptive field of the output position|| (the latter from the
    convolution of x^2 with an all-ones filter)."""
    OC = w64.shape[0]
    field = oracle.conv2d(x64 * x64, np.ones((1,) + w64.shape[1:]), stride=stride, pad=pad)  # [Nb,1,OH,OW]
    nw = np.sqrt((w64 * w64).reshape(OC, -1).sum(axis=1))
    s = abs(alpha) * nw[None, :, None, None] * np.sqrt(np.maximum(field, 0.0))
    if bias is not None:
        s = s + np.abs(bias)[None, :, None, None]
    if residual is not None:
        s = s + np.abs(residual)
    return s


def to_gpu(stored, dtype):
    """Stored host array (workloads representation) -> GPU tensor with the same bits."""
    if stored is None:
        return None
    if dtype == "bf16":
        t = torch.from_numpy(np.ascontiguousarray(stored).view(np.int16)).view(torch.bfloat16)
    else:
        t = torch.from_numpy(np.ascontiguousarray(stored))
    return t.cuda()


def to_f64(t):
    """GPU tensor -> float64 numpy array (exact)."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def bias_axis_code(axis):
    return {None: hb.HIDET_BIAS_NONE, "col": hb.HIDET_BIAS_PER_COL, "row": hb.HIDET_BIAS_PER_ROW}[axis]


def oracle_bias_axis(axis):
    return oracle.BIAS_PER_ROW if axis == "row" else oracle.BIAS_PER_COL


def make_workspace(batch, M, N, k_slices):
    """fp32 workspace of the K-parallel entry points, filled with NaN so that a stale read shows."""
    n = hb.hidet_splitk_workspace_bytes(batch, M, N, max(k_slices, 1)) // 4
    return torch.full((max(n, 4),), float("nan"), dtype=torch.float32, device="cuda")


def make_conv_workspace(y_shape, k_slices):
    """The same for the K-parallel convolution that writes y [Nb, OC, OH, OW]."""
    n = hb.hidet_conv2d_splitk_workspace_bytes(tuple(y_shape), max(k_slices, 1)) // 4
    return torch.full((max(n, 4),), float("nan"), dtype=torch.float32, device="cuda")


def run_gemm_case(c, config=-1, relu=None, alpha=None, k_slices=None):
    """Run one workloads.gemm_case through the HIP path and the oracle; returns (rel_error, got, ref).
    With k_slices the K-parallel entry point runs instead of the plain one."""
    dt = c["dtype"]
    relu = c.get("relu", False) if relu is None else relu
    alpha = c.get("alpha", 1.0) if alpha is None else alpha
    A, B = to_gpu(c["A"], dt), to_gpu(c["B"], dt)
    M, N, K = c["M"], c["N"], c["K"]
    Av = A[:, :M] if c["transA"] else A[:, :K]
    Bv = B[:, :K] if c["transB"] else B[:, :N]
    bias, res = to_gpu(c["bias"], dt), to_gpu(c["residual"], dt)
    C = torch.full((M, N), float("nan"), dtype=TORCH_DTYPE[dt], device="cuda")
    epi = hb.make_epilogue(alpha=alpha, bias=bias, bias_axis=bias_axis_code(c["bias_axis"]), residual=res, relu=relu)
    if k_slices is None:
        hb.hidet_gemm(Av, Bv, C, transA=c["transA"], transB=c["transB"], epilogue=epi, config=config)
    else:
        hb.hidet_batched_gemm_splitk(Av, Bv, C, make_workspace(1, M, N, k_slices), k_slices=k_slices, transA=c["transA"],
                                     transB=c["transB"], epilogue=epi, config=config)
    torch.cuda.synchronize()
    A64 = wl.widen(c["A"], dt)
    B64 = wl.widen(c["B"], dt)
    A64 = A64[:, :M] if c["transA"] else A64[:, :K]
    B64 = B64[:, :K] if c["transB"] else B64[:, :N]
    ref = oracle.gemm(A64, B64, transA=c["transA"], transB=c["transB"], alpha=alpha,
                      bias=None if c["bias"] is None else wl.widen(c["bias"], dt),
                      bias_axis=oracle_bias_axis(c["bias_axis"]),
                      residual=None if c["residual"] is None else wl.widen(c["residual"], dt), relu=relu)
    got = to_f64(C)
    assert_elementwise(got, ref, gemm_scale(A64, B64, c["transA"], c["transB"], alpha,
                                            None if c["bias"] is None else wl.widen(c["bias"], dt), c["bias_axis"],
                                            None if c["residual"] is None else wl.widen(c["residual"], dt)),
                       dt, K, "gemm %dx%dx%d %s config %d" % (M, N, K, dt, config))
    return oracle.rel_frobenius(got, ref), got, ref


def run_conv_case(c, config=-1, k_slices=None, packed=False):
    """Run one workloads.conv_case through the HIP path and the oracle.  packed=True: the weights are repacked by
    hidet_conv2d_pack_weights and the packed entry point runs (the oracle always sees the OIHW weights)."""
    dt = c["dtype"]
    x, w = to_gpu(c["x"], dt), to_gpu(c["w"], dt)
    bias, res = to_gpu(c["bias"], dt), to_gpu(c["residual"], dt)
    stride = c["stride"] if isinstance(c["stride"], tuple) else (c["stride"], c["stride"])
    pad = c["pad"] if isinstance(c["pad"], tuple) else (c["pad"], c["pad"])
    y = torch.full(hb.conv_out_shape(x.shape, w.shape, stride, pad), float("nan"), dtype=TORCH_DTYPE[dt], device="cuda")
    epi = hb.make_epilogue(alpha=c.get("alpha", 1.0), bias=bias, bias_axis=hb.HIDET_BIAS_PER_ROW, residual=res,
                           relu=c.get("relu", False))
    if packed:
        wp = hb.hidet_conv2d_pack_weights(w)
        ws = None if k_slices is None else make_conv_workspace(y.shape, k_slices)
        hb.hidet_conv2d_implicit_gemm_packed(x, wp, y, stride=stride, pad=pad, epilogue=epi, config=config,
                                             k_slices=k_slices or 0, workspace=ws)
    elif k_slices is None:
        hb.hidet_conv2d_implicit_gemm(x, w, y, stride=stride, pad=pad, epilogue=epi, config=config)
    else:
        ws = make_conv_workspace(y.shape, k_slices)
        hb.hidet_conv2d_implicit_gemm_splitk(x, w, y, ws, k_slices=k_slices, stride=stride, pad=pad, epilogue=epi,
                                             config=config)
    torch.cuda.synchronize()
    ref = oracle.conv2d(wl.widen(c["x"], dt), wl.widen(c["w"], dt), stride=stride, pad=pad, alpha=c.get("alpha", 1.0),
                        bias=None if c["bias"] is None else wl.widen(c["bias"], dt),
                        residual=None if c["residual"] is None else wl.widen(c["residual"], dt), relu=c.get("relu", False))
    got = to_f64(y)
    x64, w64 = wl.widen(c["x"], dt), wl.widen(c["w"], dt)
    assert_elementwise(got, ref, conv_scale(x64, w64, stride, pad, c.get("alpha", 1.0),
                                            None if c["bias"] is None else wl.widen(c["bias"], dt),
                                            None if c["residual"] is None else wl.widen(c["residual"], dt)),
                       dt, w64[0].size, "conv %s config %d" % (c.get("name", tuple(x.shape)), config))
    return oracle.rel_frobenius(got, ref), got, ref


def sliceable_configs(dtype):
    """Configurations that have a K-parallel form (workgroup tile at most 128x128, or the ring schedule)."""
    return [i for i in applicable_configs(dtype)
            if hb.hidet_config_info(i)["block_m"] * hb.hidet_config_info(i)["block_n"] <= 128 * 128
            or hb.hidet_config_info(i)["schedule"] == 1]


def applicable_configs(dtype):
    out = []
    for i in range(hb.hidet_config_count()):
        info = hb.hidet_config_info(i)
        if bool(info["is_f32"]) == (dtype == "f32"):
            out.append(i)
    return out
