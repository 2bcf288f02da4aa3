"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, sizes its workspace, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "diloco_mi355.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2412_01152_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding.load()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined", "sizeof"}


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    from paper_2412_01152_amd import binding
    assert set(binding.EXPORTS) <= names
    assert {"diloco_pseudograd_quantize", "int8_reduce_chunk", "outer_nesterov_step"} <= names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def test_qparams_layout_matches_header():
    from paper_2412_01152_amd import binding
    d = binding.QPARAMS_DTYPE
    assert d.itemsize == 40
    assert [d.fields[k][1] for k in ("mean", "std", "lo", "inv_w", "n", "status", "pad")] == [0, 8, 16, 20, 24, 32, 36]


def test_workspace_bytes(lib):
    from paper_2412_01152_amd import binding
    assert binding.workspace_bytes(0) == 0
    a, b = binding.workspace_bytes(1), binding.workspace_bytes(381)
    assert 0 < a < b
    assert b >= 381 * (8 + 16 + 4 + 256 * 16)
    assert binding.workspace_bytes(65537) == 0


def test_strerror(lib):
    assert lib.diloco_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert len(lib.diloco_strerror(code)) > 3


def _seg(vals):
    return np.asarray(vals, dtype=np.uint64)


def test_bad_arguments_are_rejected_on_the_host(lib):
    """None of these reaches a HIP call: the checks run first."""
    vp = ctypes.c_void_p
    fake = vp(0x1000)          # never dereferenced: every call below fails validation
    so = _seg([0, 16])
    sp = vp(so.ctypes.data)
    q = lib.diloco_pseudograd_quantize
    assert q(vp(0), fake, 0, 16, sp, 1, fake, fake, fake, fake, 1 << 20, vp(0)) == -1
    assert q(fake, fake, 7, 16, sp, 1, fake, fake, fake, fake, 1 << 20, vp(0)) == -5
    assert q(fake, fake, 0, 16, sp, 0, fake, fake, fake, fake, 1 << 20, vp(0)) == -2
    assert q(fake, fake, 0, 17, sp, 1, fake, fake, fake, fake, 1 << 20, vp(0)) == -2      # seg[T] != N
    bad = _seg([0, 9, 5, 16])
    assert q(fake, fake, 0, 16, vp(bad.ctypes.data), 3, fake, fake, fake, fake, 1 << 20, vp(0)) == -2
    assert q(vp(0x1002), fake, 0, 16, sp, 1, fake, fake, fake, fake, 1 << 20, vp(0)) == -3
    assert q(fake, fake, 0, 16, sp, 1, fake, fake, fake, fake, 8, vp(0)) == -4
    assert q(fake, fake, 0, 16, sp, 1, fake, fake, fake, vp(0x1010), 1 << 20, vp(0)) == -3  # workspace align

    r = lib.int8_reduce_chunk
    ptrs = (ctypes.c_void_p * 17)(*([0x1000] * 17))
    pp = ctypes.cast(ptrs, vp)
    assert r(pp, pp, 17, vp(0), 1, 16, sp, 1, vp(0), fake, fake, fake, fake, 1 << 20, vp(0)) == -2
    assert r(pp, pp, 0, vp(0), 1, 16, sp, 1, vp(0), fake, fake, fake, fake, 1 << 20, vp(0)) == -2
    assert r(pp, pp, 2, vp(0), 0, 16, sp, 1, vp(0), fake, fake, fake, fake, 1 << 20, vp(0)) == -2
    assert r(vp(0), pp, 2, vp(0), 2, 16, sp, 1, vp(0), fake, fake, fake, fake, 1 << 20, vp(0)) == -1
    assert r(pp, pp, 2, vp(0), 2, 16, sp, 1, vp(0), fake, fake, fake, fake, 16, vp(0)) == -4

    # the entry point with the library's own static scratch: the segment limit is checked first
    rs = lib.int8_reduce_chunk_static
    big = _seg(list(range(0, 514)))
    assert rs(pp, pp, 2, vp(0), 2, 513, vp(big.ctypes.data), 513, vp(0), fake, fake, fake, vp(0)) == -6
    assert len(lib.diloco_strerror(-6)) > 3

    qv, rv = lib.diloco_pseudograd_quantize_variant, lib.int8_reduce_chunk_variant
    args_q = (fake, fake, 0, 16, sp, 1, fake, fake, fake, fake, 1 << 20, vp(0))
    args_r = (pp, pp, 2, vp(0), 2, 16, sp, 1, vp(0), fake, fake, fake, fake, 1 << 20, vp(0))
    for bad_range in (0.0, 0.25, 65.0, float("nan"), float("inf"), -6.0):
        assert qv(*args_q, bad_range, 0) == -2
        assert rv(*args_r, bad_range, 0) == -2
    assert qv(*args_q, 6.0, 2) == -5 and rv(*args_r, 6.0, 2) == -5
    assert qv(vp(0), *args_q[1:], 4.0, 1) == -1                 # the ordinary checks still run

    o = lib.outer_nesterov_step
    f = ctypes.c_float
    assert o(fake, fake, vp(0), vp(0), vp(0), vp(0), 0, 16, f(.7), f(.9), vp(0), 0, vp(0), 0, vp(0)) == -1
    assert o(fake, fake, fake, fake, fake, sp, 1, 16, f(.7), f(.9), vp(0), 0, vp(0), 0, vp(0)) == -1
    assert o(fake, fake, vp(0), fake, vp(0), sp, 1, 16, f(.7), f(.9), vp(0), 0, vp(0), 0, vp(0)) == -1
    assert o(fake, fake, vp(0), fake, fake, sp, 1, 16, f(.7), f(.9), vp(0), 0, vp(0), 0, vp(0)) == -1   # no workspace
    # the fp32 form takes an optional workspace: if given it must be aligned and large enough
    assert o(fake, fake, fake, vp(0), vp(0), vp(0), 0, 16, f(.7), f(.9), vp(0), 0, vp(0x1010), 1 << 20, vp(0)) == -3
    assert o(fake, fake, fake, vp(0), vp(0), vp(0), 0, 16, f(.7), f(.9), vp(0), 0, fake, 8, vp(0)) == -4
    assert o(fake, fake, fake, vp(0), vp(0), vp(0), 0, 16, f(.7), f(.9), fake, 9, vp(0), 0, vp(0)) == -5
    assert o(vp(0x1001), fake, fake, vp(0), vp(0), vp(0), 0, 16, f(.7), f(.9), vp(0), 0, vp(0), 0, vp(0)) == -3


def test_placement_advice(lib):
    """diloco_placement: three group offsets, 100 GiB apart in a large arena, a third apart in a small one."""
    from paper_2412_01152_amd import binding
    GiB = 1 << 30
    r = binding.placement(280 * GiB)
    assert r == (4 * GiB, 104 * GiB, 204 * GiB)
    r = binding.placement(3 * GiB)
    assert r[1] - r[0] == r[2] - r[1] == GiB and all(v % 4096 == 0 for v in r) and r[2] + GiB // 2 < 3 * GiB
    out = (ctypes.c_uint64 * 3)()
    assert lib.diloco_placement(ctypes.c_uint64(100), ctypes.cast(out, ctypes.c_void_p)) == -2
    assert lib.diloco_placement(ctypes.c_uint64(GiB), ctypes.c_void_p(0)) == -1


def test_write_phase_tuning_validates_its_arguments(lib):
    """The instrumentation call that retimes pass B's staged code writes: host state only, no device use."""
    t = lib.diloco_tune_write_phase
    try:
        assert t(40, 10) == 0 and t(10, 10) == 0 and t(1000000, 1) == 0
        assert t(0, 0) == 0 and t(0, 123) == 0                 # write at once: the window is ignored
        for period, window in ((40, 0), (40, -3), (40, 41), (1000001, 1), (1, 2)):
            assert t(period, window) == -2
    finally:
        assert t(-1, 0) == 0                                   # back to the built-in choice


def test_binding_refuses_to_run_without_the_library(monkeypatch, tmp_path):
    from paper_2412_01152_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError):
        binding.load()


def test_synth_shapes():
    from paper_2412_01152_amd import synth
    assert len(synth.config_segment_sizes(1)) == 9
    assert len(synth.config_segment_sizes(2)) == 381
    assert synth.n_elements(2) == 10_211_381_248
    c4 = synth.config_segment_sizes(4)
    assert len(c4) == 14 and c4[0] == 729_384_375 and c4[-1] == 729_384_373 and sum(c4) == synth.n_elements(2)
