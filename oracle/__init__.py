"""ctypes access to the CPU oracle (``evg_oracle.cpp``) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  It never touches the HIP library, and the HIP path never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "evg_oracle.cpp")
_LIB = os.path.join(_HERE, "libevg_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler (single thread, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class OrcConfig(C.Structure):
    _fields_ = [
        ("P", C.c_uint32), ("L", C.c_uint32),
        ("layer_numel", C.POINTER(C.c_uint64)),
        ("layer_fan_in", C.POINTER(C.c_uint32)),
        ("lr", C.c_float), ("momentum", C.c_float),
        ("thr_mode", C.c_uint32), ("thr_fixed", C.c_float),
        ("horizon", C.c_float), ("hist_len", C.c_uint32), ("delta_init", C.c_float),
        ("force_first", C.c_uint32),
        ("topk_ppm", C.c_uint32), ("topk_key", C.c_uint32),
        ("trigger_kind", C.c_uint32), ("grad_mode", C.c_uint32),
        ("seed", C.c_uint64), ("dist", C.c_uint32), ("fan_in_scaling", C.c_uint32),
        ("sigma0", C.c_double), ("decay", C.c_double),
        ("spike_prob", C.c_float), ("spike_gain", C.c_float),
        ("delivery_delay", C.c_uint32), ("xhat_reset", C.c_uint32),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # EVG_ORACLE_LIB: load this build of the oracle instead (the planted-mistake test points
        # it at deliberately broken copies to show that the pins notice them)
        l = C.CDLL(os.environ.get("EVG_ORACLE_LIB") or build())
        vp, u8p, f32p = C.c_void_p, C.POINTER(C.c_uint8), C.POINTER(C.c_float)
        u32p, u64p, i32p, i8p = (C.POINTER(C.c_uint32), C.POINTER(C.c_uint64),
                                 C.POINTER(C.c_int32), C.POINTER(C.c_int8))
        l.orc_create.restype = vp
        l.orc_create.argtypes = [C.POINTER(OrcConfig), f32p]
        l.orc_destroy.argtypes = [vp]
        l.orc_numel.restype = C.c_uint64
        l.orc_numel.argtypes = [vp]
        l.orc_step.restype = C.c_int
        l.orc_step.argtypes = [vp, C.c_uint64, f32p, i8p]
        l.orc_get_state.argtypes = [vp, C.c_int, f32p]
        l.orc_set_state.argtypes = [vp, C.c_int, f32p]
        l.orc_decisions.argtypes = [vp, u8p, u8p, f32p, f32p]
        l.orc_tables.argtypes = [vp, f32p, i32p, u8p, u8p, u64p, u64p]
        l.orc_totals.argtypes = [vp, u64p]
        l.orc_message.restype = C.c_uint64
        l.orc_message.argtypes = [vp, C.c_uint32, C.c_uint32, u32p, f32p, C.c_uint64]
        l.orc_message_hashes.argtypes = [vp, u64p, u64p]
        l.orc_splitmix64.restype = C.c_uint64
        l.orc_splitmix64.argtypes = [C.c_uint64]
        l.orc_grad_tensor.argtypes = [vp, C.c_uint32, C.c_uint64, C.c_uint32, f32p]
        l.orc_average.argtypes = [vp, f32p]
        l.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        l.orc_uniform01.restype = C.c_float
        l.orc_uniform01.argtypes = [C.c_uint32]
        l.orc_log.restype = C.c_float
        l.orc_log.argtypes = [C.c_float]
        l.orc_exp.restype = C.c_float
        l.orc_exp.argtypes = [C.c_float]
        l.orc_sincos2pi.argtypes = [C.c_float, f32p, f32p]
        l.orc_normal4.argtypes = [u32p, f32p]
        l.orc_topk_count.restype = C.c_uint64
        l.orc_topk_count.argtypes = [C.c_uint64, C.c_uint32]
        l.orc_topk_select.argtypes = [u32p, C.c_uint64, C.c_uint64, u32p]
        _lib = l
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


STATE = {"x": 0, "xhat": 1, "mbox_l": 2, "mbox_r": 3, "vel": 4}


class Oracle:
    """One simulated ring of P workers on the CPU.  ``x0`` is [P, N] float32
    (tensors concatenated without padding)."""

    def __init__(self, x0, layer_numel, layer_fan_in=None, *, lr=0.05, momentum=0.9,
                 thr_mode=1, thr_fixed=0.0, horizon=1.0, hist_len=1, delta_init=0.0,
                 force_first=1, topk_ppm=0, topk_key=0, trigger_kind=0, grad_mode=0,
                 seed=0, dist=0, fan_in_scaling=0, sigma0=0.0, decay=1.0,
                 spike_prob=0.0, spike_gain=1.0, delivery_delay=0, xhat_reset=0):
        self._h = None
        x0 = np.ascontiguousarray(x0, dtype=np.float32)
        self.P, self.N = x0.shape
        self._numel = np.ascontiguousarray(layer_numel, dtype=np.uint64)
        self.L = int(self._numel.size)
        assert int(self._numel.sum()) == self.N
        self._fan = (np.ascontiguousarray(layer_fan_in, dtype=np.uint32)
                     if layer_fan_in is not None else np.ones(self.L, dtype=np.uint32))
        cfg = OrcConfig(self.P, self.L, _p(self._numel, C.c_uint64), _p(self._fan, C.c_uint32),
                        lr, momentum, thr_mode, thr_fixed, horizon, hist_len, delta_init,
                        force_first, topk_ppm, topk_key, trigger_kind, grad_mode,
                        seed, dist, fan_in_scaling, sigma0, decay, spike_prob, spike_gain,
                        delivery_delay, xhat_reset)
        self._h = lib().orc_create(C.byref(cfg), _p(x0, C.c_float))
        if not self._h:
            raise ValueError("oracle rejected the configuration")
        self.topk_ppm = topk_ppm

    @classmethod
    def from_workload(cls, w, x0=None, **over):
        """Build from a ``paper_2103_07454_amd.inputs.Workload`` description."""
        from paper_2103_07454_amd import inputs
        if x0 is None:
            x0 = inputs.replicate(w.x0(), w.P)
        kw = dict(lr=w.lr, momentum=w.momentum, thr_mode=w.thr_mode, thr_fixed=w.thr_fixed,
                  horizon=w.horizon, delta_init=w.delta_init, force_first=w.force_first,
                  topk_ppm=w.topk_ppm, seed=w.seed, dist=w.dist,
                  fan_in_scaling=w.fan_in_scaling, sigma0=w.sigma0, decay=w.decay,
                  spike_prob=w.spike_prob, spike_gain=w.spike_gain)
        kw.update(over)
        return cls(x0, w.layer_numel, w.layer_fan_in, **kw)

    def close(self):
        if self._h:
            lib().orc_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def step(self, k, grad=None, override=None):
        g = _p(np.ascontiguousarray(grad, dtype=np.float32), C.c_float) if grad is not None else None
        if grad is not None:
            self._g = np.ascontiguousarray(grad, dtype=np.float32)
            g = _p(self._g, C.c_float)
        ov = None
        if override is not None:
            self._ov = np.ascontiguousarray(override, dtype=np.int8)
            ov = _p(self._ov, C.c_int8)
        rc = lib().orc_step(self._h, int(k), g, ov)
        if rc != 0:
            raise RuntimeError(f"orc_step failed with status {rc}")

    def state(self, name):
        out = np.empty((self.P, self.N), dtype=np.float32)
        lib().orc_get_state(self._h, STATE[name], _p(out, C.c_float))
        return out

    def set_state(self, name, arr):
        a = np.ascontiguousarray(arr, dtype=np.float32)
        assert a.shape == (self.P, self.N)
        lib().orc_set_state(self._h, STATE[name], _p(a, C.c_float))

    def decisions(self):
        PL = self.P * self.L
        fired = np.empty(PL, np.uint8); near = np.empty(PL, np.uint8)
        norm = np.empty(PL, np.float32); dbefore = np.empty(PL, np.float32)
        lib().orc_decisions(self._h, _p(fired, C.c_uint8), _p(near, C.c_uint8),
                            _p(norm, C.c_float), _p(dbefore, C.c_float))
        sh = (self.P, self.L)
        return dict(fired=fired.reshape(sh), near_tie=near.reshape(sh),
                    norm=norm.reshape(sh), delta_before=dbefore.reshape(sh))

    def tables(self):
        PL = self.P * self.L
        delta = np.empty(PL, np.float32); le = np.empty(PL, np.int32)
        vl = np.empty(PL, np.uint8); vr = np.empty(PL, np.uint8)
        ef = np.empty(PL, np.uint64); et = np.empty(PL, np.uint64)
        lib().orc_tables(self._h, _p(delta, C.c_float), _p(le, C.c_int32), _p(vl, C.c_uint8),
                         _p(vr, C.c_uint8), _p(ef, C.c_uint64), _p(et, C.c_uint64))
        sh = (self.P, self.L)
        return dict(delta=delta.reshape(sh), last_event_iter=le.reshape(sh),
                    valid_l=vl.reshape(sh), valid_r=vr.reshape(sh),
                    events_full=ef.reshape(sh), events_topk=et.reshape(sh))

    def totals(self):
        out = np.zeros(8, np.uint64)
        lib().orc_totals(self._h, _p(out, C.c_uint64))
        keys = ["events_total", "value_words", "index_words", "bytes_sent",
                "near_tie_flags", "nonfinite_norms", "iters"]
        return {k: int(out[i]) for i, k in enumerate(keys)}

    def message(self, r, l):
        n = int(lib().orc_message(self._h, r, l, None, None, 0))
        idx = np.empty(n, np.uint32); val = np.empty(n, np.float32)
        if n:
            lib().orc_message(self._h, r, l, _p(idx, C.c_uint32), _p(val, C.c_float), n)
        return idx, val

    def message_hashes(self):
        """Fingerprints of the last step's Top-K messages, [P, L] uint64 each (0 = none)."""
        PL = self.P * self.L
        ih = np.zeros(PL, np.uint64); mh = np.zeros(PL, np.uint64)
        lib().orc_message_hashes(self._h, _p(ih, C.c_uint64), _p(mh, C.c_uint64))
        return ih.reshape(self.P, self.L), mh.reshape(self.P, self.L)

    def grad_tensor(self, r, k, l):
        out = np.empty(int(self._numel[l]), np.float32)
        lib().orc_grad_tensor(self._h, r, int(k), l, _p(out, C.c_float))
        return out

    def average(self):
        out = np.empty(self.N, np.float32)
        lib().orc_average(self._h, _p(out, C.c_float))
        return out


# ---- free functions of the generator and the selection, for pin tests -------

def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32); k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, np.uint32)
    lib().orc_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def uniform01(w):
    return float(lib().orc_uniform01(int(w)))


def log_poly(u):
    return float(lib().orc_log(float(u)))


def exp_poly(y):
    return float(lib().orc_exp(float(y)))


def sincos2pi(u):
    c = C.c_float(); s = C.c_float()
    lib().orc_sincos2pi(float(u), C.byref(c), C.byref(s))
    return c.value, s.value


def normal4(w):
    a = np.ascontiguousarray(w, dtype=np.uint32); z = np.empty(4, np.float32)
    lib().orc_normal4(_p(a, C.c_uint32), _p(z, C.c_float))
    return z


def splitmix64(z):
    return int(lib().orc_splitmix64(int(z)))


def topk_count(n, ppm):
    return int(lib().orc_topk_count(int(n), int(ppm)))


def topk_select(keys, K):
    k = np.ascontiguousarray(keys, dtype=np.uint32)
    out = np.empty(int(K), np.uint32)
    lib().orc_topk_select(_p(k, C.c_uint32), k.size, int(K), _p(out, C.c_uint32))
    return out
