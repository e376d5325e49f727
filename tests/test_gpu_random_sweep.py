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
