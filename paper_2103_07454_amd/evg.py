"""Thin ctypes binding over ``libevg.so`` (see ``include/evg.h``).

Argument marshalling only: every step of the parameter path runs in the HIP
kernels of the library.  PyTorch is used to allocate the five device arenas and
to provide the stream.  There is no CPU fallback: if the library has not been
built, or no GPU is present, calls fail loudly.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libevg.so")

EVG_OK = 0
THR_FIXED, THR_ADAPTIVE = 0, 1
KEY_ABS_DRIFT, KEY_ABS_VALUE = 0, 1
GRAD_SYNTH, GRAD_BUFFER = 0, 1
DIST_NORMAL, DIST_STUDENT_T3 = 0, 1
NORM_FUSED, NORM_SEPARATE = 0, 1
ACCESS_AUTO, ACCESS_STREAM, ACCESS_CACHED = 0, 1, 2
TRIGGER_DRIFT_NORM, TRIGGER_NORM_DIFF = 0, 1
PHASES = ("norm", "trigger", "send_full", "topk_select", "topk_send", "update", "deliver")

EXPORTS = ("evg_padded_numel", "evg_layer_offsets", "evg_init", "evg_init_static", "evg_step", "evg_step_next", "evg_stats",
           "evg_last_decisions", "evg_message", "evg_message_hashes", "evg_average", "evg_state_size", "evg_state_export",
           "evg_state_import", "evg_timing", "evg_timing_read",
           "evg_destroy", "evg_strerror", "evg_error_text")


class EvgError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"evg status {status}: {text}")
        self.status = status


class Synth(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("dist", C.c_uint32), ("fan_in_scaling", C.c_uint32),
                ("sigma0", C.c_double), ("decay", C.c_double),
                ("spike_prob", C.c_float), ("spike_gain", C.c_float)]


class Config(C.Structure):
    _fields_ = [("P", C.c_uint32), ("L", C.c_uint32),
                ("layer_numel", C.POINTER(C.c_uint64)), ("layer_fan_in", C.POINTER(C.c_uint32)),
                ("lr", C.c_float), ("momentum", C.c_float),
                ("thr_mode", C.c_uint32), ("thr_fixed", C.c_float), ("horizon", C.c_float),
                ("hist_len", C.c_uint32), ("delta_init", C.c_float), ("force_first", C.c_uint32),
                ("topk_ppm", C.c_uint32), ("topk_key", C.c_uint32), ("grad_mode", C.c_uint32),
                ("norm_mode", C.c_uint32), ("chunk_elems", C.c_uint32), ("trigger_kind", C.c_uint32),
                ("delivery_delay", C.c_uint32), ("xhat_reset", C.c_uint32), ("access_mode", C.c_uint32),
                ("synth", Synth),
                ("x", C.c_void_p), ("xhat", C.c_void_p), ("mbox_l", C.c_void_p),
                ("mbox_r", C.c_void_p), ("vel", C.c_void_p)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("iters", "events_total", "events_full", "events_topk", "value_words", "index_words",
                 "bytes_sent", "regular_events", "regular_words", "near_tie_flags", "nonfinite_norms",
                 "chunks_not_staged", "library_bytes")] + \
               [("events_full_rl", C.c_void_p), ("events_topk_rl", C.c_void_p), ("last_norm", C.c_void_p),
                ("delta", C.c_void_p), ("last_event_iter", C.c_void_p), ("valid_l", C.c_void_p),
                ("valid_r", C.c_void_p)]


_lib = None


def lib():
    """Loads the C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2103_07454_amd.build` "
                "(there is no fallback implementation)")
        # PyTorch ships its own HIP runtime; load it first so that the library binds
        # to the runtime that owns the device memory and streams it is handed.
        import torch  # noqa: F401
        l = C.CDLL(LIB_PATH)
        vp, u64p = C.c_void_p, C.POINTER(C.c_uint64)
        l.evg_padded_numel.restype = C.c_uint64
        l.evg_padded_numel.argtypes = [C.c_uint32, u64p]
        l.evg_layer_offsets.argtypes = [C.c_uint32, u64p, u64p]
        l.evg_init.argtypes = [C.POINTER(vp), C.POINTER(Config), vp]
        l.evg_init_static.argtypes = [C.POINTER(vp), C.POINTER(Config), vp]
        l.evg_step.argtypes = [vp, C.c_uint64, vp]
        l.evg_step_next.argtypes = [vp, vp]
        l.evg_stats.argtypes = [vp, C.POINTER(Stats)]
        l.evg_last_decisions.argtypes = [vp, vp, vp, vp, vp]
        l.evg_message.argtypes = [vp, C.c_uint32, C.c_uint32, vp, vp, C.c_uint64, u64p]
        l.evg_message_hashes.argtypes = [vp, vp, vp]
        l.evg_average.argtypes = [vp, vp]
        l.evg_state_size.restype = C.c_uint64
        l.evg_state_size.argtypes = [vp]
        l.evg_state_export.argtypes = [vp, vp, C.c_uint64]
        l.evg_state_import.argtypes = [vp, vp, C.c_uint64]
        l.evg_timing.argtypes = [vp, C.c_int]
        l.evg_timing_read.argtypes = [vp, C.POINTER(C.c_double), u64p]
        l.evg_destroy.argtypes = [vp]
        l.evg_strerror.restype = C.c_char_p
        l.evg_strerror.argtypes = [C.c_int]
        l.evg_error_text.restype = C.c_char_p
        _lib = l
    return _lib


def _check(rc):
    if rc != EVG_OK:
        raise EvgError(rc, lib().evg_error_text().decode() or lib().evg_strerror(rc).decode())


def _u64(a):
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint64))


def padded_numel(layer_numel) -> int:
    a, p = _u64(layer_numel)
    return int(lib().evg_padded_numel(a.size, p))


def layer_offsets(layer_numel) -> np.ndarray:
    a, p = _u64(layer_numel)
    out = np.zeros(a.size, np.uint64)
    _check(lib().evg_layer_offsets(a.size, p, out.ctypes.data_as(C.POINTER(C.c_uint64))))
    return out


class Layout:
    """Where each tensor of a worker sits inside the padded arena slice."""

    def __init__(self, layer_numel):
        self.numel = np.ascontiguousarray(layer_numel, dtype=np.uint64)
        self.offsets = layer_offsets(self.numel)
        self.npad = padded_numel(self.numel)
        self.N = int(self.numel.sum())
        idx = np.concatenate([np.arange(int(o), int(o) + int(n), dtype=np.int64)
                              for o, n in zip(self.offsets, self.numel)])
        self.index = idx             # arena position of every unpadded element

    def pad(self, flat: np.ndarray, fill=0.0) -> np.ndarray:
        """[P, N] unpadded -> [P, npad] arena layout."""
        flat = np.asarray(flat)
        out = np.full((flat.shape[0], self.npad), fill, dtype=flat.dtype)
        out[:, self.index] = flat
        return out

    def unpad(self, arena: np.ndarray) -> np.ndarray:
        return np.ascontiguousarray(np.asarray(arena).reshape(-1, self.npad)[:, self.index])


class Ring:
    """P simulated ring workers resident on one GPU.

    ``x0``: [P, N] float32 initial parameters (numpy, unpadded).  Keyword
    arguments mirror ``evg_config``.  ``mailbox_fill`` pre-fills the mailboxes
    (e.g. with NaN, to show that empty slots are never read).
    """

    def __init__(self, x0, layer_numel, layer_fan_in=None, *, lr=0.05, momentum=0.9,
                 thr_mode=THR_ADAPTIVE, thr_fixed=0.0, horizon=1.0, hist_len=1, delta_init=0.0,
                 force_first=1, topk_ppm=0, topk_key=KEY_ABS_DRIFT, grad_mode=GRAD_SYNTH,
                 norm_mode=NORM_FUSED, chunk_elems=0, trigger_kind=TRIGGER_DRIFT_NORM, delivery_delay=0, xhat_reset=0, access_mode=0, seed=0, dist=DIST_NORMAL, fan_in_scaling=0,
                 sigma0=0.0, decay=1.0, spike_prob=0.0, spike_gain=1.0, device="cuda:0",
                 mailbox_fill=None, stream=None, static_tables=False):
        import torch
        self.torch = torch
        lib()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the EventGraD path only runs on the HIP device")
        self.device = torch.device(device)
        self.layout = Layout(layer_numel)
        x0 = np.asarray(x0, dtype=np.float32)
        self.P, self.L = int(x0.shape[0]), int(self.layout.numel.size)
        if x0.shape[1] != self.layout.N:
            raise ValueError("x0 does not match the tensor sizes")
        npad = self.layout.npad
        self._numel = self.layout.numel
        self._fan = (np.ascontiguousarray(layer_fan_in, dtype=np.uint32)
                     if layer_fan_in is not None else None)
        with torch.cuda.device(self.device):
            self.x = torch.zeros((self.P, npad), dtype=torch.float32, device=self.device)
            if x0.shape[0] and np.all(x0 == x0[0:1]):      # common start: upload one slice
                one = torch.from_numpy(self.layout.pad(x0[0:1])).to(self.device)
                self.x.copy_(one.expand(self.P, npad))
            else:
                self.x.copy_(torch.from_numpy(self.layout.pad(x0)))
            self.xhat = torch.empty_like(self.x)
            self.vel = torch.empty_like(self.x)
            self.mbox_l = torch.empty_like(self.x)
            self.mbox_r = torch.empty_like(self.x)
            if mailbox_fill is not None:
                self.mbox_l.fill_(mailbox_fill)
                self.mbox_r.fill_(mailbox_fill)
            self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
            cfg = Config()
            cfg.P, cfg.L = self.P, self.L
            cfg.layer_numel = self._numel.ctypes.data_as(C.POINTER(C.c_uint64))
            cfg.layer_fan_in = (self._fan.ctypes.data_as(C.POINTER(C.c_uint32))
                                if self._fan is not None else None)
            cfg.lr, cfg.momentum = lr, momentum
            cfg.thr_mode, cfg.thr_fixed, cfg.horizon = thr_mode, thr_fixed, horizon
            cfg.hist_len, cfg.delta_init, cfg.force_first = hist_len, delta_init, force_first
            cfg.topk_ppm, cfg.topk_key, cfg.grad_mode = topk_ppm, topk_key, grad_mode
            cfg.norm_mode, cfg.chunk_elems, cfg.trigger_kind = norm_mode, chunk_elems, trigger_kind
            cfg.delivery_delay = delivery_delay
            cfg.access_mode = access_mode
            cfg.xhat_reset = xhat_reset
            cfg.synth = Synth(seed, dist, fan_in_scaling, sigma0, decay, spike_prob, spike_gain)
            cfg.x, cfg.xhat = self.x.data_ptr(), self.xhat.data_ptr()
            cfg.mbox_l, cfg.mbox_r, cfg.vel = self.mbox_l.data_ptr(), self.mbox_r.data_ptr(), self.vel.data_ptr()
            torch.cuda.synchronize(self.device)
            h = C.c_void_p()
            init = lib().evg_init_static if static_tables else lib().evg_init
            free_before = torch.cuda.mem_get_info(self.device)[0]
            _check(init(C.byref(h), C.byref(cfg), C.c_void_p(self.stream.cuda_stream)))
            # device memory the library took for its own tables (0 for evg_init_static)
            self.library_bytes = free_before - torch.cuda.mem_get_info(self.device)[0]
            self._h = h
        self.topk_ppm = topk_ppm
        self.access_mode = access_mode
        self.momentum = float(momentum)

    @classmethod
    def from_workload(cls, w, x0=None, **over):
        from . import inputs
        if x0 is None:
            x0 = inputs.replicate(w.x0(), w.P)
        kw = dict(lr=w.lr, momentum=w.momentum, thr_mode=w.thr_mode, thr_fixed=w.thr_fixed,
                  horizon=w.horizon, delta_init=w.delta_init, force_first=w.force_first,
                  topk_ppm=w.topk_ppm, seed=w.seed, dist=w.dist, fan_in_scaling=w.fan_in_scaling,
                  sigma0=w.sigma0, decay=w.decay, spike_prob=w.spike_prob, spike_gain=w.spike_gain)
        kw.update(over)
        return cls(x0, w.layer_numel, w.layer_fan_in, **kw)

    # -- the three calls of the hot path -----------------------------------
    def step(self, k, grad=None):
        """Enqueue iteration k (no host synchronisation)."""
        g = None
        if grad is not None:
            g = C.c_void_p(grad.data_ptr())
        _check(lib().evg_step(self._h, int(k), g))

    def step_next(self, grad=None):
        """Enqueue the iteration after the last one; replayable from a captured graph."""
        g = None
        if grad is not None:
            g = C.c_void_p(grad.data_ptr())
        _check(lib().evg_step_next(self._h, g))

    def stats(self, arrays=False):
        st = Stats()
        keep = {}
        if arrays:
            S = self.P * self.L
            for name, dt in (("events_full_rl", np.uint32), ("events_topk_rl", np.uint32),
                             ("last_norm", np.float32), ("delta", np.float32),
                             ("last_event_iter", np.int32), ("valid_l", np.uint8), ("valid_r", np.uint8)):
                keep[name] = np.zeros(S, dt)
                setattr(st, name, keep[name].ctypes.data)
        _check(lib().evg_stats(self._h, C.byref(st)))
        out = {n: int(getattr(st, n)) for n, _ in Stats._fields_[:13]}
        for name, a in keep.items():
            out[name] = a.reshape(self.P, self.L)
        return out

    # -- inspection ----------------------------------------------------------
    def decisions(self):
        S = self.P * self.L
        fired = np.zeros(S, np.uint8); near = np.zeros(S, np.uint8)
        norm = np.zeros(S, np.float32); dbefore = np.zeros(S, np.float32)
        _check(lib().evg_last_decisions(self._h, fired.ctypes.data, near.ctypes.data,
                                        norm.ctypes.data, dbefore.ctypes.data))
        sh = (self.P, self.L)
        return dict(fired=fired.reshape(sh), near_tie=near.reshape(sh), norm=norm.reshape(sh),
                    delta_before=dbefore.reshape(sh))

    def message(self, r, l):
        n = C.c_uint64(0)
        _check(lib().evg_message(self._h, r, l, None, None, 0, C.byref(n)))
        idx = np.zeros(n.value, np.uint32); val = np.zeros(n.value, np.float32)
        if n.value:
            _check(lib().evg_message(self._h, r, l, idx.ctypes.data, val.ctypes.data, n.value, C.byref(n)))
        return idx, val

    def message_hashes(self):
        """Fingerprints of the last step's Top-K messages: two [P, L] uint64 arrays."""
        S = self.P * self.L
        ih = np.zeros(S, np.uint64); mh = np.zeros(S, np.uint64)
        _check(lib().evg_message_hashes(self._h, ih.ctypes.data, mh.ctypes.data))
        return ih.reshape(self.P, self.L), mh.reshape(self.P, self.L)

    def state(self, name) -> np.ndarray:
        """[P, N] host copy of an arena with the padding removed."""
        t = getattr(self, name)
        self.torch.cuda.synchronize(self.device)
        return self.layout.unpad(t.cpu().numpy())

    def average(self) -> np.ndarray:
        out = self.torch.empty(self.layout.npad, dtype=self.torch.float32, device=self.device)
        _check(lib().evg_average(self._h, C.c_void_p(out.data_ptr())))
        self.torch.cuda.synchronize(self.device)
        return out.cpu().numpy()[self.layout.index]

    def export_state(self) -> dict:
        """Checkpoint: host copies of the five arenas (arena layout) plus the library's blob."""
        n = int(lib().evg_state_size(self._h))
        blob = np.zeros(n, np.uint8)
        _check(lib().evg_state_export(self._h, blob.ctypes.data, n))
        ck = {"blob": blob}
        for name in ("x", "xhat", "mbox_l", "mbox_r", "vel"):
            ck[name] = getattr(self, name).cpu().numpy()
        return ck

    def import_state(self, ck: dict):
        """Resume from export_state() of a ring with the same configuration."""
        self.torch.cuda.synchronize(self.device)
        for name in ("x", "xhat", "mbox_l", "mbox_r", "vel"):
            getattr(self, name).copy_(self.torch.from_numpy(ck[name]))
        self.torch.cuda.synchronize(self.device)
        blob = np.ascontiguousarray(ck["blob"], dtype=np.uint8)
        _check(lib().evg_state_import(self._h, blob.ctypes.data, blob.size))

    def timing(self, enable=True):
        _check(lib().evg_timing(self._h, 1 if enable else 0))

    def timing_read(self):
        ms = (C.c_double * len(PHASES))()
        n = (C.c_uint64 * len(PHASES))()
        _check(lib().evg_timing_read(self._h, ms, n))
        return {p: (ms[i], int(n[i])) for i, p in enumerate(PHASES)}

    def synchronize(self):
        self.stream.synchronize()

    def close(self):
        if getattr(self, "_h", None):
            lib().evg_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
