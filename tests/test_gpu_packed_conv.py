"""The convolution with repacked (tap-major) weights: the repacking kernel against the index permutation it is defined
as, and the packed entry point against the CPU oracle's direct convolution (which always sees the OIHW weights)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2210_09603_amd import binding as hb
from paper_2210_09603_amd import workloads as wl

from helpers import TOL, TORCH_DTYPE, applicable_configs, make_conv_workspace, run_conv_case, to_f64, to_gpu, within_bound

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_pack_weights_is_the_stated_permutation(dtype):
    g = wl.rng(8800)
    for OC, IC, KH, KW in [(5, 8, 3, 3), (64, 64, 3, 3), (7, 24, 5, 2), (3, 16, 1, 1), (130, 40, 1, 7)]:
        w = wl.normal(g, (OC, IC, KH, KW), dtype)
        got = hb.hidet_conv2d_pack_weights(to_gpu(w, dtype))
        torch.cuda.synchronize()
        want = np.ascontiguousarray(np.transpose(np.asarray(w), (0, 2, 3, 1)))  # [oc][kh][kw][ic] = w[oc][ic][kh][kw]
        got_bits = got.cpu().view(torch.int16 if dtype != "f32" else torch.int32).numpy()
        assert np.array_equal(got_bits, want.view(got_bits.dtype)), (OC, IC, KH, KW)


def _packed_configs(dtype, IC):
    return [i for i in applicable_configs(dtype) if IC % hb.hidet_config_info(i)["block_k"] == 0]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_config3_3x3_layers_packed(dtype):
    for c in wl.config3(dtype)[:2]:
        err, _, _ = run_conv_case(c, packed=True)
        _say("%s %s packed err %.3e" % (c["name"], dtype, err))
        assert err <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_every_fitting_config_on_a_packed_conv(dtype):
    # 2 images, 32 -> 24 channels, 3x3, stride 1, pad 1, 13 x 19 pixels (ragged output rows), bias + residual + ReLU
    c = wl.conv_case(8810, 2, 32, 13, 19, 24, 3, 3, 1, 1, dtype, residual=True)
    c.update(relu=True, alpha=0.75)
    cfgs = _packed_configs(dtype, 32)
    assert len(cfgs) >= 3
    for cfg in cfgs:
        err, _, ref = run_conv_case(c, config=cfg, packed=True)
        _say("packed conv config %d %s err %.3e" % (cfg, dtype, err))
        assert within_bound(err, ref, dtype), cfg
    # a configuration whose K tile does not divide IC cannot run the packed form
    bad = [i for i in applicable_configs(dtype) if 32 % hb.hidet_config_info(i)["block_k"] != 0]
    if bad:
        with pytest.raises(hb.HidetError) as e:
            run_conv_case(c, config=bad[0], packed=True)
        assert e.value.status == 4


PACKED_VARIANTS = [
    # Nb, IC, H, W, OC, KH, KW, stride, pad
    (1, 64, 14, 14, 40, 3, 3, 2, 1),          # stride 2
    (3, 32, 9, 11, 20, 5, 5, 1, 2),           # 5x5
    (2, 96, 10, 17, 33, 3, 2, (2, 1), (0, 1)),  # rectangular filter, stride and padding
    (1, 128, 7, 7, 64, 3, 3, 1, 1),           # rows shorter than a chunk
    (4, 32, 20, 6, 16, 1, 3, 1, (0, 2)),      # padding wider than the filter needs
    (1, 256, 28, 28, 256, 3, 3, 2, 1),        # the case-study layer (Section 6.3.1)
]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_packed_conv_variants(dtype):
    for i, (Nb, IC, H, W, OC, KH, KW, s, p) in enumerate(PACKED_VARIANTS):
        c = wl.conv_case(8820 + i, Nb, IC, H, W, OC, KH, KW, s, p, dtype, residual=(i % 2 == 0))
        c.update(relu=(i % 3 != 0), alpha=1.0 if i % 2 else -0.5)
        err, _, ref = run_conv_case(c, packed=True)
        _say("packed variant %d %s err %.3e" % (i, dtype, err))
        assert within_bound(err, ref, dtype), i
        err, _, ref = run_conv_case(c, packed=True, k_slices=3)
        assert within_bound(err, ref, dtype), ("sliced", i)


def test_packed_conv_first_and_last_pixels_and_empty_taps():
    """Windows that would start before the tensor or end after it (first / last pixels, padded corners) and filter
    taps that fall entirely into the padding."""
    for i, (H, W, KH, KW, p) in enumerate([(3, 3, 3, 3, 1), (2, 9, 5, 3, (2, 1)), (1, 8, 3, 3, 1), (5, 4, 3, 7, (1, 3))]):
        c = wl.conv_case(8840 + i, 1, 32, H, W, 8, KH, KW, 1, p, "f16")
        c.update(relu=False)
        err, _, ref = run_conv_case(c, packed=True)
        assert within_bound(err, ref, "f16"), (H, W, KH, KW)


def test_packed_conv_tuner_and_unsupported_shapes():
    dtype = "f16"
    c = wl.conv_case(8850, 2, 64, 28, 28, 64, 3, 3, 1, 1, dtype)
    c.update(relu=True)
    x, w, bias = to_gpu(c["x"], dtype), to_gpu(c["w"], dtype), to_gpu(c["bias"], dtype)
    wp = hb.hidet_conv2d_pack_weights(w)
    y = torch.empty((2, 64, 28, 28), dtype=TORCH_DTYPE[dtype], device="cuda")
    epi = hb.make_epilogue(bias=bias, bias_axis=hb.HIDET_BIAS_PER_ROW, relu=True)
    cfg, slices, us = hb.hidet_tune_conv2d_packed(x, wp, y, None, stride=(1, 1), pad=(1, 1), epilogue=epi, iters=3)
    assert cfg in _packed_configs(dtype, 64) and slices == 1 and us > 0
    ws = make_conv_workspace(y.shape, 16)
    cfg, slices, us = hb.hidet_tune_conv2d_packed(x, wp, y, ws, stride=(1, 1), pad=(1, 1), epilogue=epi, iters=3)
    assert slices >= 1 and us > 0
    y.fill_(float("nan"))
    hb.hidet_conv2d_implicit_gemm_packed(x, wp, y, stride=(1, 1), pad=(1, 1), epilogue=epi, workspace=ws)  # remembered choice
    torch.cuda.synchronize()
    ref = oracle.conv2d(wl.widen(c["x"], dtype), wl.widen(c["w"], dtype), pad=(1, 1), bias=wl.widen(c["bias"], dtype), relu=True)
    assert oracle.rel_frobenius(to_f64(y), ref) <= TOL[dtype]
    hb.hidet_tune_clear()
    # IC not a multiple of 8, stride 3: the packed form says so instead of computing something else; so does an IC
    # that no configuration's K tile divides (the smallest K tile of the 16-bit space is 32)
    for IC, s, status in [(12, 1, 2), (32, 3, 2), (16, 1, 4)]:
        c = wl.conv_case(8851, 1, IC, 12, 12, 8, 3, 3, s, 1, dtype)
        with pytest.raises(hb.HidetError) as e:
            run_conv_case(c, packed=True)
        assert e.value.status == status
