"""Seeded synthetic inputs for the five benchmark/parity workloads.

This module serves both the HIP path's callers and the CPU oracle's callers; it holds none of
the method's arithmetic -- only random draws, the single round-to-nearest-even conversion of
each fp32 draw to its storage type, and the exact widening of stored values to float64.

Storage representation on the host (numpy):  "f32" -> float32, "f16" -> float16,
"bf16" -> uint16 holding the bfloat16 bit pattern.

The paper measures layers of ResNet-50, BERT and GPT-2 with trained weights (Section 6.1); those
models are not available here, so the shapes of their layers with the usual initialisation
distributions stand in for them.  Seeds: config 1 uses seed 0; every other case uses
1000*config + case index.
"""
import math

import numpy as np

DTYPES = ("f32", "f16", "bf16")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def to_storage(x32, dtype):
    """Round an fp32 array once (RNE) to the storage dtype."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "f32":
        return x32
    if dtype == "f16":
        return x32.astype(np.float16)
    if dtype == "bf16":
        bits = x32.view(np.uint32).astype(np.uint64)
        lsb = (bits >> 16) & 1
        return ((bits + 0x7FFF + lsb) >> 16).astype(np.uint16).reshape(x32.shape)
    raise ValueError("unknown dtype %r" % (dtype,))


def widen(stored, dtype):
    """Exact float64 value of a stored array."""
    if dtype in ("f32", "f16"):
        return np.asarray(stored).astype(np.float64)
    if dtype == "bf16":
        return (np.asarray(stored, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError("unknown dtype %r" % (dtype,))


def uniform(g, shape, dtype, lo=-1.0, hi=1.0):
    return to_storage(g.uniform(lo, hi, size=shape).astype(np.float32), dtype)


def normal(g, shape, dtype, std=1.0):
    return to_storage((g.standard_normal(size=shape) * std).astype(np.float32), dtype)


def gemm_case(seed, M, N, K, dtype, dist="uniform", transA=False, transB=False, bias=None, residual=False,
              w_std=None, lda_pad=0, ldb_pad=0):
    """A generic GEMM problem.  dist: "uniform" -> U(-1,1) for everything; "normal" -> A ~ N(0,1),
    B ~ N(0, w_std).  bias: None | "col" | "row".  Leading-dimension padding adds unused columns."""
    g = rng(seed)
    a_shape = (K, M + lda_pad) if transA else (M, K + lda_pad)
    b_shape = (N, K + ldb_pad) if transB else (K, N + ldb_pad)
    if dist == "uniform":
        A = uniform(g, a_shape, dtype)
        B = uniform(g, b_shape, dtype)
        bias_v = uniform(g, (N if bias == "col" else M,), dtype) if bias else None
        res = uniform(g, (M, N), dtype) if residual else None
    else:
        A = normal(g, a_shape, dtype)
        B = normal(g, b_shape, dtype, std=w_std if w_std is not None else 1.0)
        bias_v = normal(g, (N if bias == "col" else M,), dtype, std=w_std if w_std is not None else 1.0) if bias else None
        res = normal(g, (M, N), dtype) if residual else None
    return dict(M=M, N=N, K=K, dtype=dtype, transA=transA, transB=transB, A=A, B=B, lda=a_shape[1], ldb=b_shape[1],
                bias=bias_v, bias_axis=bias, residual=res, seed=seed)


def config1():
    """fp32 GEMM 256^3, bias per column + ReLU, everything U(-1,1), seed 0."""
    c = gemm_case(0, 256, 256, 256, "f32", bias="col")
    c.update(name="cfg1_f32_256", relu=True, alpha=1.0)
    return [c]


def config2(dtype="f16"):
    """Transformer MLP (batch 1 x seq 128): 128x768x3072 bias+ReLU, then 128x3072x768 + residual."""
    a = gemm_case(2000, 128, 3072, 768, dtype, dist="normal", bias="col", w_std=0.02)
    a.update(name="cfg2a_mlp_up", relu=True, alpha=1.0)
    b = gemm_case(2001, 128, 768, 3072, dtype, dist="normal", residual=True, w_std=0.02)
    b.update(name="cfg2b_mlp_down", relu=False, alpha=1.0)
    return [a, b]


RESNET50_CONVS = (
    # (IC, H, W, OC, KH, KW, stride, pad)
    (64, 56, 56, 64, 3, 3, 1, 1),
    (128, 28, 28, 128, 3, 3, 1, 1),
    (256, 14, 14, 1024, 1, 1, 1, 0),
    (512, 7, 7, 2048, 1, 1, 1, 0),
)


def conv_case(seed, Nb, IC, H, W, OC, KH, KW, stride, pad, dtype, bias=True, residual=False):
    g = rng(seed)
    fan_in = IC * KH * KW
    x = normal(g, (Nb, IC, H, W), dtype)
    w = normal(g, (OC, IC, KH, KW), dtype, std=math.sqrt(2.0 / fan_in))
    b = normal(g, (OC,), dtype, std=0.1) if bias else None
    sh, sw = stride if isinstance(stride, tuple) else (stride, stride)
    ph, pw = pad if isinstance(pad, tuple) else (pad, pad)
    OH = (H + 2 * ph - KH) // sh + 1
    OW = (W + 2 * pw - KW) // sw + 1
    res = normal(g, (Nb, OC, OH, OW), dtype) if residual else None
    return dict(Nb=Nb, IC=IC, H=H, W=W, OC=OC, KH=KH, KW=KW, stride=stride, pad=pad, dtype=dtype, x=x, w=w, bias=b,
                residual=res, OH=OH, OW=OW, seed=seed)


def config3(dtype="f16"):
    """ResNet-50 bottleneck convolutions, batch 1, NCHW, He-initialised weights, bias + ReLU."""
    out = []
    for i, (IC, H, W, OC, KH, KW, s, p) in enumerate(RESNET50_CONVS):
        c = conv_case(3000 + i, 1, IC, H, W, OC, KH, KW, s, p, dtype)
        c.update(name="cfg3_conv%d_%dx%d_%dto%d_k%d" % (i, H, W, IC, OC, KH), relu=True, alpha=1.0)
        out.append(c)
    return out


def attention_case(seed, batch, seq, dtype="f16", d=64):
    """Q, K, V ~ N(0,1) of shape [batch, seq, d]; S = U(0,1) rows normalised to sum 1 (in float64, then stored)."""
    g = rng(seed)
    Q = normal(g, (batch, seq, d), dtype)
    Kmat = normal(g, (batch, seq, d), dtype)
    V = normal(g, (batch, seq, d), dtype)
    S64 = g.uniform(0.0, 1.0, size=(batch, seq, seq))
    S64 /= S64.sum(axis=-1, keepdims=True)
    S = to_storage(S64.astype(np.float32), dtype)
    return dict(batch=batch, seq=seq, d=d, dtype=dtype, Q=Q, K=Kmat, V=V, S=S, alpha=1.0 / math.sqrt(d), seed=seed)


def config4(dtype="f16", cases=((12, 128), (12, 512), (192, 128), (192, 512))):
    """Attention products: scores Q.K^T scaled by 1/8 and context S.V, batch x heads in {12, 192}, seq in {128, 512}."""
    out = []
    for i, (batch, seq) in enumerate(cases):
        c = attention_case(4000 + i, batch, seq, dtype)
        c.update(name="cfg4_b%d_s%d" % (batch, seq))
        out.append(c)
    return out


def config5(dtype="f16", K=4096, M=4096, N=4096):
    """Large square GEMM (or the skinny K=1024 case), bias per column + ReLU, U(-1,1)."""
    c = gemm_case(5000 + (0 if K == 4096 else 1), M, N, K, dtype, bias="col")
    c.update(name="cfg5_%s_%dx%dx%d" % (dtype, M, N, K), relu=True, alpha=1.0)
    return c
