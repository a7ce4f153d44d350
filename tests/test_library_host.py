"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol,
and its host-side logic (layout arithmetic, argument validation) behaves."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def evg():
    from paper_2103_07454_amd import evg as m
    if not os.path.exists(m.LIB_PATH):
        from paper_2103_07454_amd import build
        build.build_library()
    return m


def test_exports_every_declared_symbol(evg):
    header = open(os.path.join(ROOT, "include", "evg.h")).read()
    declared = set(re.findall(r"\b(evg_[a-z_]+)\s*\(", header))
    assert declared == set(evg.EXPORTS)
    l = evg.lib()
    for name in declared:
        assert getattr(l, name) is not None


def test_layout_arithmetic(evg):
    assert evg.padded_numel([10, 3, 100352]) == 100416           # 12 + 4 + 100352 -> next multiple of 64
    assert list(evg.layer_offsets([10, 3, 100352])) == [0, 12, 16]
    assert evg.padded_numel([]) == 0 and evg.padded_numel([0]) == 0
    lay = evg.Layout([5, 4, 1])
    flat = np.arange(20, dtype=np.float32).reshape(2, 10)
    assert np.array_equal(lay.unpad(lay.pad(flat)), flat)
    assert lay.npad == 64 and list(lay.offsets) == [0, 8, 12]
    from paper_2103_07454_amd import inputs
    for i, n in ((1, 101_770), (2, 272_474), (3, 11_173_962), (4, 25_557_032), (5, 11_173_962)):
        w = inputs.config(i)
        assert w.N == n and evg.padded_numel(w.layer_numel) >= n


def base_cfg(evg, keep):
    n = np.array([10, 3], np.uint64)
    keep.append(n)
    cfg = evg.Config()
    cfg.P, cfg.L = 3, 2
    cfg.layer_numel = n.ctypes.data_as(C.POINTER(C.c_uint64))
    cfg.lr, cfg.momentum = 0.05, 0.9
    cfg.thr_mode, cfg.horizon, cfg.hist_len = 1, 1.0, 1
    cfg.synth.decay, cfg.synth.sigma0 = 1.0, 0.01
    cfg.x, cfg.xhat, cfg.mbox_l, cfg.mbox_r, cfg.vel = 0x1000, 0x2000, 0x3000, 0x4000, 0x5000
    return cfg


@pytest.mark.parametrize("mut,status", [
    (lambda c: setattr(c, "P", 2), 1),
    (lambda c: setattr(c, "L", 0), 1),
    (lambda c: setattr(c, "lr", float("nan")), 1),
    (lambda c: setattr(c, "thr_mode", 7), 1),
    (lambda c: setattr(c, "hist_len", 0), 1),
    (lambda c: setattr(c, "hist_len", 17), 1),
    (lambda c: setattr(c, "horizon", -1.0), 1),
    (lambda c: setattr(c, "delta_init", float("nan")), 1),
    (lambda c: setattr(c, "topk_ppm", 1_000_001), 1),
    (lambda c: setattr(c, "topk_key", 2), 1),
    (lambda c: setattr(c, "grad_mode", 2), 1),
    (lambda c: setattr(c, "norm_mode", 2), 1),
    (lambda c: setattr(c, "trigger_kind", 2), 1),
    (lambda c: setattr(c, "delivery_delay", 2), 1),
    (lambda c: setattr(c, "access_mode", 3), 1),
    (lambda c: setattr(c, "xhat_reset", 2), 1),
    (lambda c: (setattr(c, "xhat_reset", 1), setattr(c, "delivery_delay", 1)), 1),
    (lambda c: setattr(c, "chunk_elems", 1000), 1),
    (lambda c: setattr(c.synth, "decay", 0.0), 1),
    (lambda c: setattr(c.synth, "sigma0", -1.0), 1),
    (lambda c: setattr(c.synth, "spike_prob", 1.5), 1),
    (lambda c: setattr(c.synth, "fan_in_scaling", 1), 1),      # no fan_in table given
    (lambda c: setattr(c, "x", 0), 1),
    (lambda c: setattr(c, "vel", 0x5004), 2),
    (lambda c: setattr(c, "xhat", 0x1010), 1),                 # overlaps x
])
def test_init_rejects_bad_configurations_before_touching_the_gpu(evg, mut, status):
    keep = []
    cfg = base_cfg(evg, keep)
    mut(cfg)
    h = C.c_void_p()
    rc = evg.lib().evg_init(C.byref(h), C.byref(cfg), None)
    assert rc == status, evg.lib().evg_error_text()
    assert h.value is None and evg.lib().evg_error_text()


def test_fixed_threshold_validation(evg):
    keep = []
    cfg = base_cfg(evg, keep)
    cfg.thr_mode, cfg.thr_fixed = 0, -1.0
    h = C.c_void_p()
    assert evg.lib().evg_init(C.byref(h), C.byref(cfg), None) == 1
    cfg.thr_fixed = float("nan")
    assert evg.lib().evg_init(C.byref(h), C.byref(cfg), None) == 1


def test_null_handles_are_rejected(evg):
    l = evg.lib()
    assert l.evg_step(None, 0, None) == 1
    st = evg.Stats()
    assert l.evg_stats(None, C.byref(st)) == 1
    assert l.evg_destroy(None) == 0
    assert l.evg_strerror(4) == b"HIP runtime error"


def test_no_silent_fallback_without_gpu(evg):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(RuntimeError):
        evg.Ring(np.zeros((3, 4), np.float32), [4])
