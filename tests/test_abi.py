"""Host-side tests of the C ABI: the library loads, exports what the header declares,
and rejects bad arguments before touching the GPU.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from paper_2010_05680_amd import binding as tb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", h) for h in ("turbo_reduce.h", "turbo_reduce_testing.h", "turbo_serving.h")]

FAKE = 0x10000  # a non-null, 16-byte aligned "device pointer"; validation must fail before it is used


def _declared_functions():
    names = set()
    for header in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(turbo_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = tb.lib()
    declared = _declared_functions()
    assert set(declared) == set(tb.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(L, name), f"{name} is declared in turbo_reduce.h but not exported"


def test_status_strings():
    assert tb.status_string(tb.TURBO_OK) == "ok"
    seen = {tb.status_string(s) for s in range(6)}
    assert len(seen) == 6
    assert "unknown" in tb.status_string(99)


def test_softmax_rejects_bad_arguments_without_a_gpu():
    L = tb.lib()
    f = L.turbo_masked_softmax
    assert f(None, None, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_NULL
    assert f(FAKE, None, 1, 1, 4, 4, 1.0, 7, None) == tb.TURBO_ERR_DTYPE
    for dims in [(0, 1, 4, 4), (1, 0, 4, 4), (1, 1, 0, 4), (1, 1, 4, 0), (-1, 1, 4, 4), (1, 1, 4, -3)]:
        assert f(FAKE, None, *dims, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert f(FAKE, None, 1 << 15, 1 << 15, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE  # 2^32 rows
    big = 2 ** 31 - 1
    assert f(FAKE, None, big, big, big, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE  # no overflow on the way
    assert f(FAKE + 2, None, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_ALIGN
    assert f(FAKE + 1, None, 1, 1, 4, 4, 1.0, tb.TURBO_F16, None) == tb.TURBO_ERR_ALIGN
    assert f(FAKE, FAKE + 0x1002, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_ALIGN
    g = L.turbo_masked_softmax_ex
    assert g(FAKE, FAKE + 0x1000, -4, 0, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert g(FAKE, FAKE + 0x1000, 0, -1, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_SHAPE
    assert g(None, None, 0, 0, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_NULL


def test_layernorm_rejects_bad_arguments_without_a_gpu():
    L = tb.lib()
    f = L.turbo_add_bias_layernorm
    ok = [FAKE, FAKE, FAKE, FAKE, FAKE]
    if not torch.cuda.is_available():  # with a GPU this valid-looking call would launch on pointers that are not real
        assert f(*ok, 4, 8, 1e-5, FAKE, None) == tb.TURBO_ERR_LAUNCH
    for missing in (0, 3, 4):  # x, gamma, beta are required; residual (1) and bias (2) are optional
        args = list(ok)
        args[missing] = None
        assert f(*args, 4, 8, 1e-5, FAKE, None) == tb.TURBO_ERR_NULL
    assert f(*ok, 4, 8, 1e-5, None, None) == tb.TURBO_ERR_NULL
    assert f(*ok, 0, 8, 1e-5, FAKE, None) == tb.TURBO_ERR_SHAPE
    assert f(*ok, 4, 0, 1e-5, FAKE, None) == tb.TURBO_ERR_SHAPE
    assert f(*ok, -4, 8, 1e-5, FAKE, None) == tb.TURBO_ERR_SHAPE
    bad = list(ok)
    bad[1] = FAKE + 2
    assert f(*bad, 4, 8, 1e-5, FAKE, None) == tb.TURBO_ERR_ALIGN
    g = L.turbo_add_bias_layernorm_dt
    assert g(*ok, 4, 8, 1e-5, FAKE, 5, None) == tb.TURBO_ERR_DTYPE
    assert g(*ok, 4, 8, 1e-5, FAKE + 1, tb.TURBO_F16, None) == tb.TURBO_ERR_ALIGN


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the no-GPU failure mode")
def test_valid_call_without_a_gpu_reports_launch_error_not_a_crash():
    L = tb.lib()
    assert L.turbo_masked_softmax(FAKE, None, 1, 1, 4, 4, 1.0, tb.TURBO_F32, None) == tb.TURBO_ERR_LAUNCH


def test_binding_refuses_host_tensors_and_wrong_dtypes():
    s = torch.zeros(1, 1, 2, 2)
    with pytest.raises(ValueError):
        tb.turbo_masked_softmax(s, None, 1.0)
    with pytest.raises(TypeError):
        tb.turbo_masked_softmax(s.double(), None, 1.0)


def test_fastdiv_is_exact():
    L = tb.lib()
    rng = np.random.default_rng(0)
    ds = list(range(1, 70)) + [127, 128, 129, 500, 512, 6000, 2 ** 16, 2 ** 16 + 1, 2 ** 31 - 65536]
    ns = [0, 1, 2, 2 ** 31 - 1, 2 ** 31 - 65536, 2 ** 30, 12345678]
    for d in ds:
        for n in ns + [d - 1, d, d + 1, 2 * d - 1, 2 * d, 7 * d + 3]:
            if 0 <= n < 2 ** 31:
                assert L.turbo_debug_fastdiv(n, d) == n // d, (n, d)
    for _ in range(20000):
        n = int(rng.integers(0, 2 ** 31 - 1))
        d = int(rng.integers(1, 2 ** 31 - 1)) if rng.random() < 0.5 else int(rng.integers(1, 70000))
        assert L.turbo_debug_fastdiv(n, d) == n // d, (n, d)


def test_plan_families_follow_row_length():
    P = tb.turbo_describe_plan
    # "f": the lanes tile the row exactly, no bounds checks
    assert P(0, 192, 16, tb.TURBO_F32) == "wave vec=4f lanes=4 nv=1 rows=8"
    assert P(0, 30720, 128, tb.TURBO_F32).startswith("wave vec=4f lanes=32 nv=1")
    assert P(0, 524288, 512, tb.TURBO_F16).startswith("wave vec=8f lanes=64 nv=1")
    assert P(0, 65536, 4096, tb.TURBO_F32).startswith("block vec=4f waves=8 nv=2")  # long rows: a workgroup per row
    assert P(0, 1000, 100, tb.TURBO_F32).startswith("wave vec=4 lanes=32 nv=1")  # 25 vectors on 32 lanes: masked tail
    # odd row length: still 16-byte accesses, element-aligned ("u"), last vector overlaps its neighbour
    assert P(0, 190000, 497, tb.TURBO_F32).startswith("wave vec=4u lanes=64 nv=2")
    assert P(0, 190000, 498, tb.TURBO_F32).startswith("wave vec=4u")
    assert P(1, 1000, 771, tb.TURBO_F32).startswith("wave vec=4u lanes=64 nv=4")
    assert P(0, 1000, 100, tb.TURBO_F16).startswith("wave vec=8u lanes=16 nv=1")
    assert P(0, 10, 3, tb.TURBO_F32).startswith("wave vec=1 ")  # shorter than one vector: narrow accesses
    assert P(1, 4096, 4096, tb.TURBO_F32).startswith("block vec=4f waves=8 nv=2")
    assert P(1, 2560, 768, tb.TURBO_F32).startswith("wave vec=4f lanes=64 nv=3")
    assert P(0, 100, 8192, tb.TURBO_F32).startswith("block")
    assert P(0, 100, 40000, tb.TURBO_F32).startswith("stream")
    assert P(1, 100, 20000, tb.TURBO_F32).startswith("stream")
    assert P(0, 100, 128, tb.TURBO_F32, aligned16=False).startswith("wave vec=4u lanes=32")
    assert P(0, 100, 40001, tb.TURBO_F32).startswith("stream vec=1 ")  # two-sweep kernels narrow the access instead
    tb.turbo_set_override(tb.TURBO_OVR_MAX_VEC_BYTES, 16)
    try:  # an explicit width cap also selects the aligned narrow kernels
        assert P(0, 190000, 497, tb.TURBO_F32).startswith("wave vec=1 lanes=64 nv=8")
        assert P(0, 190000, 498, tb.TURBO_F32).startswith("wave vec=2")
    finally:
        tb.turbo_set_override(tb.TURBO_OVR_MAX_VEC_BYTES, -1)
    tb.turbo_set_override(tb.TURBO_OVR_PATH, tb.PATH_BLOCK)
    try:
        assert P(0, 30720, 128, tb.TURBO_F32).startswith("block")
    finally:
        tb.turbo_set_override(tb.TURBO_OVR_PATH, -1)
    assert P(0, 30720, 128, tb.TURBO_F32).startswith("wave")
    # LayerNorm: a workgroup of any size up to 8 wavefronts that tiles the row exactly with 3 or 2 vectors per lane
    assert P(1, 1000, 4608, tb.TURBO_F16).startswith("block vec=8f waves=3 nv=3")
    assert P(1, 1000, 5120, tb.TURBO_F16).startswith("block vec=8f waves=5 nv=2")
    assert P(1, 1000, 6144, tb.TURBO_F16).startswith("block vec=8f waves=4 nv=3")
    assert P(1, 1000, 7168, tb.TURBO_F16).startswith("block vec=8f waves=7 nv=2")
    assert P(1, 1000, 2560, tb.TURBO_F32).startswith("block vec=4f waves=5 nv=2")
    # rows of 1152 floats and more leave the wave family; 257..384 vectors take 2 wavefronts x 3 vectors, not 3 x 2
    assert P(1, 1000, 1024, tb.TURBO_F32).startswith("wave vec=4f lanes=64 nv=4")
    assert P(1, 1000, 1152, tb.TURBO_F32).startswith("block vec=4 waves=2 nv=3")
    assert P(1, 1000, 1280, tb.TURBO_F32).startswith("block vec=4 waves=2 nv=3")
    assert P(1, 1000, 2304, tb.TURBO_F16).startswith("block vec=8 waves=2 nv=3")
    assert P(1, 1000, 1280, tb.TURBO_F16).startswith("wave vec=8 lanes=64 nv=3")
    assert P(1, 1000, 2304, tb.TURBO_F32).startswith("block vec=4f waves=3 nv=3")
    assert P(1, 1000, 2560, tb.TURBO_F16).startswith("block vec=8 waves=2 nv=3")  # two wavefronts x 3, bounds-checked
    assert P(0, 1000, 4608, tb.TURBO_F16).startswith("block vec=8 waves=4 nv=3")  # 576 vectors: 4 x 3, not 8 x 2
    assert P(0, 1000, 6144, tb.TURBO_F16).startswith("block vec=8 waves=8 nv=2")
    tb.turbo_set_override(tb.TURBO_OVR_BLOCK_WAVES, 6)
    try:
        assert P(0, 1000, 6144, tb.TURBO_F16).startswith("block vec=8f waves=6 nv=2")
        assert P(0, 100, 32768, tb.TURBO_F32).startswith("block vec=4f waves=16 nv=8")  # does not fit 6: built-in choice
    finally:
        tb.turbo_set_override(tb.TURBO_OVR_BLOCK_WAVES, -1)
    with pytest.raises(tb.TurboError):
        tb.turbo_set_override(99, 0)


def _parse_plan(text):
    fam, rest = text.split(" ", 1)
    kv = dict(item.split("=") for item in rest.split())
    vec = kv["vec"]
    mode = "u" if vec.endswith("u") else "f" if vec.endswith("f") else "r"
    return fam, int(vec.rstrip("uf")), mode, {k: int(v) for k, v in kv.items() if k != "vec"}


def test_planner_invariants_over_many_shapes():
    """Whatever the shape, the chosen variant must be one that is compiled and must cover the row: the kernels trust
    the plan, so a plan outside these bounds would mean wrong results or reads outside the row."""
    rng = np.random.default_rng(7)
    lens = list(range(1, 300)) + [int(v) for v in rng.integers(300, 70000, size=400)] + \
        [512, 768, 1024, 1280, 1536, 2048, 2304, 2560, 3072, 3584, 4096, 4608, 5120, 6144, 7168, 8192, 10240, 12288, 16384, 32768, 32772, 65536, 100000]
    supported_nv = {1, 2, 3, 4, 5, 6, 8, 12, 16}
    # (operation, most elements per lane: wave family, block family, block family with 16-byte vectors of 2-byte elements)
    for op, wave_max, block_max, block_max_2byte in ((0, 64, 32, 32), (1, 24, 16, 24)):
        for dtype, es in ((tb.TURBO_F32, 4), (tb.TURBO_F16, 2)):
            for L in lens:
                for aligned in (True, False):
                    for rows in (7, 100000):
                        fam, vec, mode, kv = _parse_plan(tb.turbo_describe_plan(op, rows, L, dtype, aligned))
                        what = f"op={op} dtype={dtype} L={L} aligned={aligned} rows={rows}: {fam} vec={vec}{mode} {kv}"
                        assert vec in (1, 2, 4, 8) and vec * es <= 16, what
                        if mode == "u":
                            assert vec * es == 16 and L >= vec and (L % vec != 0 or not aligned), what
                        else:
                            assert L % vec == 0 and (aligned or vec == 1), what
                        nvec = -(-L // vec)
                        if fam == "wave":
                            lanes, nv = kv["lanes"], kv["nv"]
                            assert lanes in (4, 8, 16, 32, 64) and nv in supported_nv and kv["rows"] in (1, 2, 4, 8), what
                            assert lanes * nv >= nvec and nv * vec <= wave_max, what
                            if lanes < 64 and nv > 1:
                                assert mode == "f" and (lanes, nv) in ((32, 3), (32, 5), (16, 3)), what
                            if mode == "f":
                                assert lanes * nv * vec == L, what
                        elif fam == "block":
                            w, nv = kv["waves"], kv["nv"]
                            assert nv in supported_nv, what
                            # 5..7 wavefronts only where they tile the row exactly (LayerNorm)
                            assert w in (2, 3, 4, 8, 16) or (op == 1 and mode == "f" and w in (5, 6, 7) and nv in (2, 3)), what
                            budget = block_max_2byte if (es == 2 and vec == 8) else block_max
                            assert 64 * w * nv >= nvec and (nv * vec <= budget or nv == 1), what
                            if vec * es < 16 and op == 1:
                                assert nv <= 6, what  # narrow vectors: every one of them costs address registers
                            if mode == "f":
                                assert 64 * w * nv * vec == L, what
                        else:
                            assert fam == "stream" and mode == "r", what


def test_stream_probe_rejects_bad_arguments_without_a_gpu():
    L = tb.lib()
    fake = 0x10000
    assert L.turbo_stream_probe(None, None, fake, 64, None) == tb.TURBO_ERR_NULL
    assert L.turbo_stream_probe(fake, None, None, 64, None) == tb.TURBO_ERR_NULL
    for bad in (0, -16, 24):
        assert L.turbo_stream_probe(fake, None, fake, bad, None) == tb.TURBO_ERR_SHAPE
    assert L.turbo_stream_probe(fake + 4, None, fake, 64, None) == tb.TURBO_ERR_ALIGN
    assert L.turbo_stream_probe(fake, fake + 8, fake, 64, None) == tb.TURBO_ERR_ALIGN


def test_no_kernel_of_the_built_library_spills_registers():
    """The build writes one line per kernel from hipcc's resource-usage remarks and refuses to link when a kernel
    needs scratch memory (spills would be memory traffic the byte counts do not show).  When that report is there,
    check it again here; a library copied in without its build folder is skipped."""
    import os
    from paper_2010_05680_amd import build as tbuild
    report = os.path.join(tbuild.OBJ_DIR, tbuild.RESOURCE_FILE)
    if not os.path.exists(report):
        pytest.skip("no build report beside the library")
    lines = [ln.split() for ln in open(report) if ln.strip()]
    assert len(lines) > 100
    bad = [ln[0] for ln in lines if "scratch=0" not in ln or "vgpr_spill=0" not in ln]
    assert bad == []


def test_planner_under_sanitizers_with_row_lengths_up_to_int_max(tmp_path):
    """csrc/plan.h is host code: compiled alone with -fsanitize=address,undefined and driven over every element size,
    alignment, override and row lengths up to INT_MAX (tests/native/plan_sanitize.cpp checks the shape invariants)."""
    import subprocess
    exe = tmp_path / "plan_sanitize"
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-static-libubsan", os.path.join(ROOT, "tests", "native", "plan_sanitize.cpp"),
                           "-o", str(exe)])
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0 and res.stdout.startswith("ok"), res.stdout + res.stderr
