"""CPU-only checks of the C ABI: the library loads, exports every symbol include/qtale.h declares, and
rejects invalid arguments before touching the GPU (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def qt():
    import paper_2602_10431_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2602_10431_amd import build
        build.build(verbose=False)
    pkg.load_library()
    return pkg


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "qtale.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qtale_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(qt):
    lib = qt.load_library()
    names = _declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(qt.EXPORTS)


def test_strerror(qt):
    lib = qt.load_library()
    assert lib.qtale_strerror(0) == b"ok"
    assert b"workspace" in lib.qtale_strerror(-4)


def test_control_validation(qt):
    ctx = qt.Context()
    assert qt.qtale_get_control(ctx) == (qt.QTALE_MODE_RATIO, 1.0)
    for bad in (float("nan"), -0.1, 1.5):
        with pytest.raises(qt.QtaleError) as e:
            qt.qtale_set_exec_ratio(ctx, bad)
        assert e.value.code == -1
    qt.qtale_set_exec_ratio(ctx, 0.4)
    m, v = qt.qtale_get_control(ctx)
    assert m == qt.QTALE_MODE_RATIO and abs(v - 0.4) < 1e-7
    with pytest.raises(qt.QtaleError):
        qt.qtale_set_threshold(ctx, float("nan"))
    qt.qtale_set_threshold(ctx, 0.05)
    assert qt.qtale_get_control(ctx)[0] == qt.QTALE_MODE_THRESHOLD
    assert qt.load_library().qtale_set_exec_ratio(None, 0.5) == -1


def test_size_queries(qt):
    # LLaMA-7B-shaped down projection: 4096 x 11008, group 128
    n = qt.qtale_prepacked_bytes(4096, 11008, 4, 128)
    assert n == 4096 * 11008 // 2 + 4 * 4096 * (11008 // 128)
    # 3-bit codes: 12 bytes per lane per k-tile, same scale/zero section
    assert qt.qtale_prepacked_bytes(4096, 11008, 3, 128) == 4096 * 11008 * 3 // 8 + 4 * 4096 * (11008 // 128)
    assert qt.qtale_prepacked_bytes(4096, 11008, 2, 128) == 4096 * 11008 // 4 + 4 * 4096 * (11008 // 128)
    assert qt.qtale_prepacked_bytes(4096, 11008, 5, 128) == 0
    assert qt.qtale_prepacked_bytes(4096, 11008, 4, 100) == 0
    assert qt.qtale_prepacked_bytes(4096, 11006, 4, 128) == 0
    cfg = qt.make_cfg(4096, 32, 32, 128, 11008)
    w1, w2 = qt.qtale_workspace_bytes(cfg, 8192, 8), qt.qtale_workspace_bytes(cfg, 64, 64)
    assert w1 > w2 > 0 and w1 % 256 == 0
    bad = qt.make_cfg(4096, 32, 5, 128, 11008)
    assert qt.qtale_workspace_bytes(bad, 64, 1) == 0


def test_forward_argument_validation_needs_no_gpu(qt):
    lib = qt.load_library()
    ctx = qt.Context()
    cfg = qt.make_cfg(256, 4, 4, 64, 688, group=32, act_dtype="fp16")
    w = qt.qtale_layer_weights()
    fake = C.c_void_p(256)

    def call(cfg_, T=4, B=1, x=fake, ws=fake, ws_bytes=1 << 30, w_=w):
        return lib.qtale_layer_forward(ctx._h, C.byref(cfg_), C.byref(w_), x, T, fake, B, fake, None, None, None, None,
                                       ws, ws_bytes, None)

    assert call(cfg, x=None) == -1                               # null x
    assert call(cfg, ws_bytes=16) == -4                          # workspace too small
    assert call(cfg, T=-1) == -1
    assert call(cfg) == -1                                       # weights without prepacked buffers
    assert call(qt.make_cfg(256, 4, 3, 64, 688, group=32)) == -2  # heads not divisible
    assert call(qt.make_cfg(256, 4, 4, 64, 688, bits=5, group=32)) == -3
    assert call(qt.make_cfg(256, 4, 4, 64, 688, group=48)) == -3
    assert call(qt.make_cfg(256, 4, 4, 80, 688, group=32)) == -3
    assert call(qt.make_cfg(250, 4, 4, 64, 688, group=32)) == -2
    assert call(cfg, T=0) == 0                                   # empty call is a no-op
    # shape mismatch between cfg and a linear
    w2 = qt.qtale_layer_weights()
    for name in ("q", "k", "v", "o", "gate", "up", "down"):
        setattr(w2, name, qt.qtale_qlinear(None, None, None, 256, 256, 256))
    w2.norm1 = w2.norm2 = w2.router_w = 256
    assert call(cfg, w_=w2) == -2
    # stack: null layers
    assert lib.qtale_stack_forward(ctx._h, C.byref(cfg), None, 2, fake, 4, fake, 1, fake, None, None, None, None, None,
                                   fake, 1 << 30, None) == -1
    ql = qt.qtale_qlinear(None, None, None, None, 64, 64)
    assert lib.qtale_linear_w4a16(C.byref(ql), 4, 32, fake, 4, fake, None) == -1
    assert lib.qtale_linear_w4a16(C.byref(ql), 4, 48, fake, 4, fake, None) == -3
    assert lib.qtale_quantize(None, 8, 64, 4, 32, fake, fake, fake, None, None) == -1
    assert lib.qtale_quantize(fake, 8, 64, 5, 32, fake, fake, fake, None, None) == -3


def test_calibration_argument_validation_needs_no_gpu(qt):
    lib = qt.load_library()
    ctx = qt.Context()
    fake = C.c_void_p(256)
    assert lib.qtale_calibration_scratch_bytes(32) >= 1024 + 32 * 4
    assert lib.qtale_calibration_scratch_bytes(-1) == 0
    nan = float("nan")
    assert lib.qtale_calibrate_threshold_from_scores(ctx._h, fake, 100, nan, fake, None, None, None, None) == -1
    assert lib.qtale_calibrate_threshold_from_scores(ctx._h, fake, 100, 1.5, fake, None, None, None, None) == -1
    assert lib.qtale_calibrate_threshold_from_scores(ctx._h, None, 100, 0.5, fake, None, None, None, None) == -1
    assert lib.qtale_calibrate_threshold_from_scores(ctx._h, fake, 0, 0.5, fake, None, None, None, None) == -1
    assert lib.qtale_calibrate_threshold_from_scores(None, fake, 100, 0.5, fake, None, None, None, None) == -1
    cfg = qt.make_cfg(256, 4, 4, 64, 688, group=32)
    assert lib.qtale_calibrate_threshold(ctx._h, C.byref(cfg), None, 2, fake, fake, 4, fake, 1, fake, 0.5, fake, fake,
                                         1 << 30, None, None, None, None) == -1
    assert lib.qtale_calibrate_threshold(ctx._h, C.byref(cfg), None, 2, fake, fake, 4, fake, 1, fake, -0.1, fake, fake,
                                         1 << 30, None, None, None, None) == -1
    mode, value = qt.qtale_get_control(ctx)                      # failed calls leave the control untouched
    assert mode == qt.QTALE_MODE_RATIO and value == 1.0



def test_static_scratch_entry_validates_before_any_gpu_work(qt):
    lib = qt.load_library()
    ctx = qt.Context()
    fake = C.c_void_p(256)
    w = qt.qtale_layer_weights()
    assert qt.qtale_static_scratch_bytes() == 40 << 20
    big = qt.make_cfg(4096, 32, 32, 128, 11008)
    small = qt.make_cfg(256, 4, 4, 64, 688, group=32, act_dtype="fp16")

    def call(cfg_, T, B=1, x=fake):
        return lib.qtale_layer_forward_static(ctx._h, C.byref(cfg_), C.byref(w), x, T, fake, B, fake, None, None, None,
                                              None, None)

    assert qt.qtale_workspace_bytes(big, 4096, 1) > qt.qtale_static_scratch_bytes()
    assert call(big, 4096) == -4                                 # beyond the array: rejected, nothing launched
    assert call(small, 8, x=None) == -1
    assert call(small, -1) == -1
    assert call(small, 0) == 0
    assert call(small, 8) == -1                                  # fits, but the weights have no prepacked buffers
    assert call(qt.make_cfg(256, 4, 4, 80, 688, group=32), 8) == -3
