"""Host-only checks of the C ABI: the library loads, exports every declared symbol, validates its
arguments before touching the GPU, and its compile-time task mappings equal the paper's definitions."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import taskmap as otm
from paper_2210_09603_amd import binding as hb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "hidet_mi355x.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hidet_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = hb.lib()
    names = _declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), n
    assert sorted(hb.EXPORTS) == names


def test_version_and_schedule_space():
    assert "gfx950" in hb.hidet_version()
    n = hb.hidet_config_count()
    assert 10 <= n < 200  # "less than 200 schedules" (Section 4.3)
    seen = set()
    for i in range(n):
        c = hb.hidet_config_info(i)
        waves = c["waves_m"] * c["waves_n"]
        assert c["mfma"] in (16, 32) and 1 <= waves <= 16
        assert c["block_m"] % (c["waves_m"] * c["mfma"]) == 0 and c["block_n"] % (c["waves_n"] * c["mfma"]) == 0
        assert c["lds_bytes"] <= 160 * 1024  # LDS of one compute unit
        assert c["waves_k"] == (16 // waves if c["schedule"] == 3 else 1) and waves * c["waves_k"] <= 16
        # accumulators: one fp32 register per output element per lane, at most 256 of the 512 registers
        assert c["block_m"] * c["block_n"] // (waves * 64) <= 256
        key = tuple(c.values())
        assert key not in seen
        seen.add(key)
    with pytest.raises(hb.HidetError):
        hb.hidet_config_info(n)


def _gemm(L, **kw):
    a = dict(config=-1, i=hb.HIDET_F16, o=hb.HIDET_F16, tA=0, tB=0, M=8, N=8, K=8, A=0x1000, lda=8, B=0x2000, ldb=8,
             C=0x3000, ldc=8, epi=None, stream=None)
    a.update(kw)
    return L.hidet_gemm_cfg(a["config"], a["i"], a["o"], a["tA"], a["tB"], a["M"], a["N"], a["K"], a["A"], a["lda"], a["B"],
                            a["ldb"], a["C"], a["ldc"], a["epi"], a["stream"])


def test_gemm_argument_validation_happens_before_any_launch():
    """All pointers below are fake: reaching a launch would fault, so every call must be rejected on the host."""
    L = hb.lib()
    INVALID, UNSUPPORTED, ALIGN, NOCFG = 1, 2, 3, 4
    assert _gemm(L, A=None) == INVALID
    assert _gemm(L, C=None) == INVALID
    assert _gemm(L, M=-1) == INVALID
    assert _gemm(L, lda=7) == INVALID
    assert _gemm(L, ldb=7) == INVALID
    assert _gemm(L, ldc=7) == INVALID
    assert _gemm(L, tA=1, M=16, lda=8) == INVALID  # transposed A is K x M: lda >= M
    assert _gemm(L, i=7) == INVALID
    assert _gemm(L, i=hb.HIDET_F32, o=hb.HIDET_F16) == UNSUPPORTED
    assert _gemm(L, i=hb.HIDET_F16, o=hb.HIDET_BF16) == UNSUPPORTED
    assert _gemm(L, i=hb.HIDET_F16, o=hb.HIDET_F32, C=0x3002) == ALIGN  # fp32 output: 4-byte aligned C
    assert _gemm(L, M=2 ** 31) == UNSUPPORTED
    # 32-bit indices step at most one tile past an extent, so the largest extent stays that far below 2^31
    assert _gemm(L, M=2 ** 31 - 65536, lda=8) == UNSUPPORTED
    assert _gemm(L, K=2 ** 31 - 65536, lda=2 ** 31, ldb=8) == UNSUPPORTED
    assert _gemm(L, N=2 ** 31 - 65536, ldb=2 ** 31, ldc=2 ** 31) == UNSUPPORTED
    # what an operand spans stays below 2^47 elements, so that no offset (and no check) can overflow 64 bits
    assert _gemm(L, lda=2 ** 62) == UNSUPPORTED
    assert _gemm(L, M=2 ** 20, lda=2 ** 28) == UNSUPPORTED
    assert _gemm(L, ldc=2 ** 61) == UNSUPPORTED
    assert _gemm(L, A=0x1001) == ALIGN
    assert _gemm(L, i=hb.HIDET_F32, o=hb.HIDET_F32, C=0x3002) == ALIGN
    assert _gemm(L, config=10 ** 6) == NOCFG
    # an fp32-only configuration cannot run an fp16 problem
    f32_cfg = [i for i in range(hb.hidet_config_count()) if hb.hidet_config_info(i)["is_f32"]][0]
    assert _gemm(L, config=f32_cfg) == NOCFG
    e = hb.hidet_epilogue_t()
    e.struct_size = 4
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID
    e.struct_size = ctypes.sizeof(hb.hidet_epilogue_t)
    e.bias_axis = hb.HIDET_BIAS_PER_COL  # bias axis without a bias pointer
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID
    e.bias_axis = 0
    e.residual = 0x5000
    e.ld_residual = 4
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID
    e.ld_residual = 8
    e.act = 9
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID
    # output index map: head split needs seq | M and head_dim | N, batch 1, a known map id
    e = hb.hidet_epilogue_t()
    e.struct_size = ctypes.sizeof(hb.hidet_epilogue_t)
    e.out_map = hb.HIDET_MAP_HEAD_SPLIT
    e.map_seq, e.map_head_dim = 3, 4
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID  # 3 does not divide M = 8
    e.map_seq, e.map_head_dim = 4, 3
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID
    e.map_seq, e.map_head_dim = 0, 4
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID
    e.map_seq, e.map_head_dim = 4, 4
    e.out_map = 2
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID
    e.out_map = hb.HIDET_MAP_HEAD_SPLIT
    e.prologue = 2
    assert _gemm(L, epi=ctypes.byref(e)) == INVALID
    e.prologue = 0
    f16 = hb.HIDET_F16
    assert L.hidet_batched_gemm(f16, f16, 0, 0, 2, 8, 8, 8, 0x1000, 8, 64, 0x2000, 8, 64, 0x3000, 8, 64, ctypes.byref(e),
                                None) == UNSUPPORTED
    # empty problems are OK no-ops even with null pointers
    assert _gemm(L, M=0, A=None, B=None, C=None) == 0
    assert _gemm(L, N=0, A=None, B=None, C=None) == 0


def test_batched_and_conv_argument_validation():
    L = hb.lib()
    f16 = hb.HIDET_F16
    # overlapping batch entries of C
    assert L.hidet_batched_gemm(f16, f16, 0, 0, 4, 8, 8, 8, 0x1000, 8, 64, 0x2000, 8, 64, 0x3000, 8, 32, None, None) == 1
    assert L.hidet_batched_gemm(f16, f16, 0, 0, -1, 8, 8, 8, 0x1000, 8, 64, 0x2000, 8, 64, 0x3000, 8, 64, None, None) == 1
    assert L.hidet_batched_gemm(f16, f16, 0, 0, 0, 8, 8, 8, None, 8, 64, None, 8, 64, None, 8, 64, None, None) == 0
    # batch * stride beyond 2^47 elements
    assert L.hidet_batched_gemm(f16, f16, 0, 0, 2 ** 20, 8, 8, 8, 0x1000, 8, 2 ** 30, 0x2000, 8, 64, 0x3000, 8, 64, None,
                                None) == 2
    assert L.hidet_batched_gemm(f16, f16, 0, 0, 4, 8, 8, 8, 0x1000, 8, 64, 0x2000, 8, 64, 0x3000, 8, 2 ** 62, None,
                                None) == 2
    conv = lambda **k: L.hidet_conv2d_implicit_gemm(
        k.get("i", f16), k.get("o", f16), k.get("Nb", 1), k.get("IC", 4), k.get("H", 8), k.get("W", 8), k.get("OC", 4),
        k.get("KH", 3), k.get("KW", 3), k.get("sh", 1), k.get("sw", 1), k.get("ph", 1), k.get("pw", 1), k.get("x", 0x1000),
        k.get("w", 0x2000), k.get("y", 0x3000), k.get("epi", None), None)
    assert conv(x=None) == 1
    assert conv(o=hb.HIDET_F32) == 2  # the convolution takes same-type pairs only
    assert conv(sh=0) == 1
    assert conv(KH=0) == 1
    assert conv(ph=-1) == 1
    assert conv(y=0x3001) == 3
    assert conv(H=1, W=1, KH=5, KW=5, ph=0, pw=0, x=None, w=None, y=None) == 0  # empty output
    e = hb.hidet_epilogue_t()
    e.struct_size = ctypes.sizeof(hb.hidet_epilogue_t)
    e.bias = 0x4000
    e.bias_axis = hb.HIDET_BIAS_PER_COL  # conv bias is per output channel = per GEMM row
    assert conv(epi=ctypes.byref(e)) == 1
    e.bias_axis = hb.HIDET_BIAS_PER_ROW
    e.out_map = hb.HIDET_MAP_HEAD_SPLIT  # the convolution has its own (NCHW) index map
    e.map_seq, e.map_head_dim = 1, 1
    assert conv(epi=ctypes.byref(e)) == 1
    assert conv(H=40000) == 2 and conv(pw=20000) == 2  # rows/columns are kept in 16-bit fields
    assert conv(IC=331, H=14322, W=453) == 2  # x has 2^31 - 2 elements: a gather window could step past 2^31
    # every factor is bounded before products are formed: none of these may wrap into an accepted geometry
    assert conv(sh=2 ** 32 + 1) == 2 and conv(sw=2 ** 40) == 2 and conv(ph=2 ** 62) == 2
    assert conv(Nb=2 ** 33, IC=2 ** 31) == 2 and conv(Nb=2 ** 62) == 2 and conv(OC=2 ** 40) == 2
    assert conv(KH=2 ** 32 + 3, H=8) == 2
    assert hb.lib().hidet_status_string(3) == b"misaligned pointer"


def test_splitk_argument_validation():
    """Fake pointers again: every call must be turned down on the host."""
    L = hb.lib()
    f16 = hb.HIDET_F16
    assert L.hidet_splitk_workspace_bytes(2, 3, 5, 4) == 4 * 2 * 4 * 3 * 5
    assert L.hidet_splitk_workspace_bytes(1, 64, 64, 1) == 4 * 64 * 64
    assert L.hidet_splitk_workspace_bytes(1, 64, 64, 0) == -1
    assert L.hidet_splitk_workspace_bytes(-1, 64, 64, 2) == -1
    assert L.hidet_splitk_workspace_bytes(2 ** 31, 2 ** 31, 2 ** 31, 16) == -1  # beyond 64 bits
    assert L.hidet_splitk_workspace_bytes(1, 2 ** 30, 2 ** 20, 2) == 8 * 2 ** 50
    assert L.hidet_tune_last_times(None, 4) >= 0  # a null buffer only asks for the count
    sliceable = [i for i in range(hb.hidet_config_count())
                 if not hb.hidet_config_info(i)["is_f32"]
                 and hb.hidet_config_info(i)["block_m"] * hb.hidet_config_info(i)["block_n"] <= 128 * 128
                 and hb.hidet_config_info(i)["block_k"] <= 256][0]
    need = 4 * 4 * 64 * 64

    def g(config=sliceable, slices=4, ws=0x10000, ws_bytes=need, K=1024, A=0x1000):
        return L.hidet_batched_gemm_splitk(config, slices, f16, f16, 0, 0, 1, 64, 64, K, A, K, 0, 0x2000, 64, 0, 0x3000,
                                           64, 0, None, ws, ws_bytes, None)
    assert g(ws=None) == 1
    assert g(ws_bytes=need - 4) == 1
    assert g(ws_bytes=-1) == 1
    assert g(ws=0x10004) == 3
    assert g(slices=5000) == 1
    assert g(A=None) == 1  # the ordinary validation still comes first
    assert g(config=10 ** 6) == 4
    big = [i for i in range(hb.hidet_config_count()) if hb.hidet_config_info(i)["block_m"] == 256
           and hb.hidet_config_info(i)["schedule"] == 0 and not hb.hidet_config_info(i)["is_f32"]][0]
    assert g(config=big) == 4  # large general-schedule tiles have no K-parallel form

    def c(slices=4, ws=0x10000, ws_bytes=4 * 4 * 8 * 64, x=0x1000):
        return L.hidet_conv2d_implicit_gemm_splitk(sliceable, slices, f16, f16, 1, 64, 8, 8, 8, 3, 3, 1, 1, 1, 1, x,
                                                   0x2000, 0x3000, None, ws, ws_bytes, None)
    assert c(ws=None) == 1
    assert c(ws_bytes=64) == 1
    assert c(x=None) == 1
    f = ctypes.c_float()
    i = ctypes.c_int32()
    assert L.hidet_tune_gemm_splitk(f16, f16, 0, 0, 1, 64, 64, 1024, 0x1000, 1024, 0, 0x2000, 64, 0, 0x3000, 64, 0, None,
                                    None, 0, None, 3, ctypes.byref(i), ctypes.byref(i), ctypes.byref(f)) == 1


def test_tuned_cache_file_round_trip(tmp_path):
    """The cache is a text file of `key configuration slices form` lines; lines without the last field (files written
    before it existed) load with form 0, malformed or out-of-range lines are skipped."""
    L = hb.lib()
    src, dst = tmp_path / "in.txt", tmp_path / "out.txt"
    src.write_text("gemm:t1:00:b1:8x8x8:e0:m0 3 2\nconv:t1:n1:c4:8x8:o4:k1x1:s1x1:p0x0:e0:m0 5 1 1\nnot a line\n"
                   "gemm:t1:00:b1:9x9x9:e0:m0 100000 1 0\ngemm:t1:00:b1:7x7x7:e0:m0 2 1 7\n")
    L.hidet_tune_clear()
    assert L.hidet_tune_load(str(src).encode()) == 0
    assert L.hidet_tune_save(str(dst).encode()) == 0
    L.hidet_tune_clear()
    lines = sorted(dst.read_text().split("\n"))
    assert lines == ["", "conv:t1:n1:c4:8x8:o4:k1x1:s1x1:p0x0:e0:m0 5 1 1", "gemm:t1:00:b1:8x8x8:e0:m0 3 2 0"]
    assert L.hidet_tune_load(str(tmp_path / "missing.txt").encode()) == 1 and L.hidet_tune_load(None) == 1


def test_multiply_shift_division_equals_floor_division():
    """The divider the kernels use for index arithmetic, checked where such schemes go wrong: every n for small
    divisors, and the neighbourhood of every multiple near the top of the 31-bit range for a spread of divisors."""
    L = hb.lib()
    q = ctypes.c_int32()

    def div(d, n):
        assert L.hidet_host_div(d, n, ctypes.byref(q)) == 0
        return q.value
    for d in range(1, 40):
        for n in range(0, 2000):
            assert div(d, n) == n // d, (d, n)
    rng = np.random.default_rng(123)
    top = 2 ** 31 - 1
    divisors = [1, 2, 3, 7, 9, 49, 196, 3136, 12544, 2 ** 16 - 1, 2 ** 16, 2 ** 16 + 1, 2 ** 30, 2 ** 30 + 1, top - 1, top]
    divisors += [int(x) for x in rng.integers(1, top, size=60)]
    for d in divisors:
        probes = {0, 1, d - 1, d, d + 1, top, top - 1, (top // d) * d, (top // d) * d - 1, max((top // d) * d - d, 0)}
        probes |= {int(x) for x in rng.integers(0, top, size=50)}
        for n in probes:
            if 0 <= n <= top:
                assert div(d, n) == n // d, (d, n)
    assert L.hidet_host_div(0, 5, ctypes.byref(q)) == 1 and L.hidet_host_div(3, -1, ctypes.byref(q)) == 1
    assert L.hidet_host_div(3, 5, None) == 1


def test_reduction_argument_validation():
    L = hb.lib()
    f16, f32, bf16 = hb.HIDET_F16, hb.HIDET_F32, hb.HIDET_BF16
    red = lambda **k: L.hidet_reduce_rows(k.get("i", f16), k.get("o", f16), k.get("op", 0), k.get("rows", 4),
                                          k.get("cols", 8), k.get("x", 0x1000), k.get("ldx", 8), k.get("y", 0x2000), None)
    assert red(x=None) == 1 and red(y=None) == 1 and red(ldx=7) == 1 and red(rows=-1) == 1 and red(op=3) == 1
    assert red(i=5) == 1 and red(o=bf16) == 2 and red(x=0x1001) == 3 and red(o=f32, y=0x2002) == 3
    assert red(rows=0, x=None, y=None) == 0
    sm = lambda **k: L.hidet_softmax_rows(k.get("t", f16), k.get("rows", 4), k.get("cols", 8), k.get("x", 0x1000),
                                          k.get("ldx", 8), k.get("y", 0x2000), k.get("ldy", 8), None)
    assert sm(x=None) == 1 and sm(y=None) == 1 and sm(ldx=7) == 1 and sm(ldy=7) == 1 and sm(cols=-1) == 1 and sm(t=3) == 1
    assert sm(y=0x2001) == 3 and sm(cols=2 ** 31) == 2
    assert sm(rows=2 ** 40, ldx=2 ** 20, ldy=2 ** 20) == 2 and sm(ldy=2 ** 62) == 2 and red(rows=2 ** 50, ldx=2 ** 10) == 2
    assert sm(rows=0, x=None, y=None) == 0 and sm(cols=0, ldx=0, ldy=0, x=None, y=None) == 0


def test_probe_argument_validation():
    L = hb.lib()
    n = L.hidet_probe_scratch_bytes()
    assert n >= 256 * 512 * 4
    f = ctypes.c_float()
    assert L.hidet_probe_mfma_peak(hb.HIDET_F16, 16, None, 8192, 0x1000, n, None, ctypes.byref(f), ctypes.byref(f)) == 1
    assert L.hidet_probe_mfma_peak(hb.HIDET_F16, 24, 0x1000, 8192, 0x2000, n, None, ctypes.byref(f), ctypes.byref(f)) == 1
    assert L.hidet_probe_mfma_peak(hb.HIDET_F16, 16, 0x1000, 8192, 0x2000, n - 1, None, ctypes.byref(f), ctypes.byref(f)) == 1
    assert L.hidet_probe_mfma_peak(hb.HIDET_F16, 16, 0x1000, 8192, 0x2004, n, None, ctypes.byref(f), ctypes.byref(f)) == 3
    assert L.hidet_probe_mfma_peak(9, 16, 0x1000, 8192, 0x2000, n, None, ctypes.byref(f), ctypes.byref(f)) == 1
    assert L.hidet_probe_launch_floor(None, 0, ctypes.byref(f)) == 1 and L.hidet_probe_launch_floor(None, 10, None) == 1
    gib = 1 << 30
    assert L.hidet_probe_stream_bandwidth(None, gib, 0, None, ctypes.byref(f)) == 1
    assert L.hidet_probe_stream_bandwidth(0x1000, gib, 0, None, None) == 1
    assert L.hidet_probe_stream_bandwidth(0x1000, gib, 3, None, ctypes.byref(f)) == 1
    assert L.hidet_probe_stream_bandwidth(0x1000, (256 << 20) - 1, 0, None, ctypes.byref(f)) == 1  # fewer than two pieces
    assert L.hidet_probe_stream_bandwidth(0x1008, gib, 0, None, ctypes.byref(f)) == 3


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(hb, "_lib", None)
    monkeypatch.setattr(hb, "LIB_PATH", "/nonexistent/libhidet_mi355x.so")
    with pytest.raises(RuntimeError, match="HIP extension missing"):
        hb.lib()


# ---------------------------------------------------------------- task mappings: templates == definitions
def _parse(expr):
    f = None
    for term in expr.split("*"):
        m = re.fullmatch(r"(repeat|spatial)\((\d+),(\d+)\)", term.strip())
        g = getattr(otm, m.group(1))(int(m.group(2)), int(m.group(3)))
        f = g if f is None else f * g
    return f


def test_compile_time_task_mappings_match_the_definitions():
    n = hb.hidet_taskmap_count()
    assert n >= 8
    for idx in range(n):
        info = hb.hidet_taskmap_info(idx)
        ref = _parse(info["expr"])
        assert info["workers"] == ref.num_workers and info["shape"] == ref.task_shape, info
        for w in range(ref.num_workers):
            assert hb.hidet_taskmap_tasks(idx, w) == ref(w), (info["expr"], w)


def test_block_level_mapping_is_a_permutation_and_groups_rows():
    for tiles_m, tiles_n, group in [(16, 16, 4), (5, 7, 4), (1, 9, 1), (3, 3, 8), (7, 2, 4)]:
        tasks = [hb.hidet_block_task(tiles_m, tiles_n, group, w) for w in range(tiles_m * tiles_n)]
        assert sorted(tasks) == [(i, j) for i in range(tiles_m) for j in range(tiles_n)]
    # 16x16 tiles, group 4: any 32 consecutive workgroups (one die's share) cover a 4 x 8 patch
    tasks = [hb.hidet_block_task(16, 16, 4, w) for w in range(256)]
    for s in range(0, 256, 32):
        rows = {t[0] for t in tasks[s:s + 32]}
        cols = {t[1] for t in tasks[s:s + 32]}
        assert len(rows) == 4 and len(cols) == 8


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_headline_kernel_task_mappings_are_exported():
    """The mappings of the ring-schedule 256x256x32 configuration (its direct global -> LDS loads walk the first two,
    its wavefronts the third) are among the exported ones, so the comparison above covers them."""
    exprs = [hb.hidet_taskmap_info(i)["expr"] for i in range(hb.hidet_taskmap_count())]
    for e in ("repeat(2,1)*spatial(128,4)", "repeat(2,1)*spatial(16,32)", "spatial(2,4)*repeat(8,4)"):
        assert e in exprs
    ring = [i for i in range(hb.hidet_config_count()) if hb.hidet_config_info(i)["schedule"] == 1]
    big = [hb.hidet_config_info(i) for i in ring if hb.hidet_config_info(i)["block_m"] == 256 and
           hb.hidet_config_info(i)["block_n"] == 256 and hb.hidet_config_info(i)["mfma"] == 16]
    assert big and big[0]["block_k"] == 32 and (big[0]["waves_m"], big[0]["waves_n"]) == (2, 4)


def test_conv_workspace_size_and_static_scratch_limits():
    L = hb.lib()
    # y [1, 24, 14, 14] in 3 slices: GEMM N pads every output row of 14 to 16 positions
    assert hb.hidet_conv2d_splitk_workspace_bytes((1, 24, 14, 14), 3) == 4 * 3 * 24 * 14 * 16
    assert hb.hidet_conv2d_splitk_workspace_bytes((2, 8, 7, 8), 1) == 4 * 8 * 2 * 7 * 8
    assert hb.hidet_conv2d_splitk_workspace_bytes((1, 24, 14, 14), 3) == hb.hidet_splitk_workspace_bytes(1, 24, 14 * 16, 3)
    assert hb.hidet_conv2d_splitk_workspace_bytes((-1, 24, 14, 14), 3) == -1
    assert hb.hidet_conv2d_splitk_workspace_bytes((1, 24, 14, 14), 0) == -1
    assert hb.hidet_static_scratch_bytes() == 32 << 20
    # argument validation of the allocation-free entry point happens before anything touches the GPU
    args = [-1, 4, hb.HIDET_F16, hb.HIDET_F16, 0, 0, 1, 8, 8, 8, None, 8, 0, 0x2000, 8, 0, 0x3000, 8, 0, None, None]
    assert L.hidet_batched_gemm_splitk_static(*args) == 1
    args[10] = 0x1000
    args[1] = 2000
    assert L.hidet_batched_gemm_splitk_static(*args) == 1
    args[1], args[0] = 4, 10 ** 6
    assert L.hidet_batched_gemm_splitk_static(*args) == 4
    assert "scratch" in L.hidet_status_string(6).decode()


def test_packed_conv_argument_validation():
    L = hb.lib()
    INVALID, UNSUPPORTED, ALIGN, NOCFG = 1, 2, 3, 4
    assert L.hidet_conv2d_pack_weights(hb.HIDET_F16, 8, 8, 3, 3, None, 0x2000, None) == INVALID
    assert L.hidet_conv2d_pack_weights(hb.HIDET_F16, 8, 8, 0, 3, 0x1000, 0x2000, None) == INVALID
    assert L.hidet_conv2d_pack_weights(7, 8, 8, 3, 3, 0x1000, 0x2000, None) == INVALID
    assert L.hidet_conv2d_pack_weights(hb.HIDET_F16, 8, 8, 3, 3, 0x1001, 0x2000, None) == ALIGN
    assert L.hidet_conv2d_pack_weights(hb.HIDET_F16, 0, 8, 3, 3, None, None, None) == 0  # nothing to do

    def packed(**kw):
        a = dict(config=-1, slices=0, i=hb.HIDET_F16, o=hb.HIDET_F16, Nb=1, IC=16, H=8, W=8, OC=8, KH=3, KW=3, sh=1, sw=1,
                 ph=1, pw=1, x=0x1000, w=0x2000, y=0x3000, epi=None, ws=None, wsb=0, stream=None)
        a.update(kw)
        return L.hidet_conv2d_implicit_gemm_packed(a["config"], a["slices"], a["i"], a["o"], a["Nb"], a["IC"], a["H"], a["W"],
                                                   a["OC"], a["KH"], a["KW"], a["sh"], a["sw"], a["ph"], a["pw"], a["x"],
                                                   a["w"], a["y"], a["epi"], a["ws"], a["wsb"], a["stream"])
    assert packed(x=None) == INVALID
    assert packed(IC=12) == UNSUPPORTED          # rows of the repacked weights must be 16-byte multiples
    assert packed(sw=3) == UNSUPPORTED
    assert packed(w=0x2002) == UNSUPPORTED       # the packed weights are read with 16-byte loads
    assert packed(slices=2000) == INVALID
    assert packed(config=10 ** 6) == NOCFG
    # a tile whose K extent does not divide IC cannot keep a K tile within one filter tap
    cfgs = [i for i in range(hb.hidet_config_count()) if not hb.hidet_config_info(i)["is_f32"]
            and 16 % hb.hidet_config_info(i)["block_k"] != 0]
    assert cfgs and packed(config=cfgs[0]) == NOCFG
