"""Thin ctypes binding of the host controller (``include/faser_controller.h``): argument marshalling only,
every computation happens in the C++ library.  Host memory throughout; needs no GPU and no torch tensors.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence

from .binding import _check, load_library

MAX_LENGTHS = 16
LAT_DRAFT, LAT_TARGET, LAT_EXIT, LAT_PRUNE, LAT_KV = 0, 1, 2, 3, 4

CTL_SYMBOLS = [
    "fsr_ctl_default_config", "fsr_ctl_create", "fsr_ctl_destroy", "fsr_ctl_observe", "fsr_ctl_forget", "fsr_ctl_estimates",
    "fsr_ctl_best_length", "fsr_ctl_posterior", "fsr_ctl_choose", "fsr_expected_rejected", "fsr_prune_trigger",
    "fsr_latency_eval", "fsr_latency_fit", "fsr_chunk_size",
]


class CtlConfig(ctypes.Structure):
    _fields_ = [("n_lengths", ctypes.c_int32), ("lengths", ctypes.c_int32 * MAX_LENGTHS), ("window", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("eps", ctypes.c_double), ("beta", ctypes.c_double), ("delta", ctypes.c_double),
                ("length_scale", ctypes.c_double), ("signal_var", ctypes.c_double), ("noise_var", ctypes.c_double)]


class LatencyModel(ctypes.Structure):
    _fields_ = [("form", ctypes.c_int32), ("reserved", ctypes.c_int32), ("a1", ctypes.c_double), ("g1", ctypes.c_double),
                ("a2", ctypes.c_double), ("g2", ctypes.c_double), ("knee", ctypes.c_double), ("alpha", ctypes.c_double),
                ("beta", ctypes.c_double), ("c", ctypes.c_double)]

    def params(self):
        return (self.a1, self.g1, self.a2, self.g2, self.knee, self.alpha, self.beta, self.c)


def _lib():
    lib = load_library()
    if not getattr(lib, "_fsr_ctl_ready", False):
        lib.fsr_ctl_create.argtypes = [ctypes.POINTER(CtlConfig), ctypes.POINTER(ctypes.c_void_p)]
        lib.fsr_ctl_destroy.argtypes = [ctypes.c_void_p]
        lib.fsr_ctl_destroy.restype = None
        lib.fsr_ctl_observe.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_double]
        lib.fsr_ctl_forget.argtypes = [ctypes.c_void_p, ctypes.c_int64]
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        lib.fsr_ctl_estimates.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, dp, dp, dp]
        lib.fsr_ctl_best_length.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ip]
        lib.fsr_ctl_posterior.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, dp, dp]
        lib.fsr_ctl_choose.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ip]
        lib.fsr_expected_rejected.argtypes = [ctypes.c_int32, ip, dp, dp]
        lib.fsr_prune_trigger.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_double, ctypes.c_double, dp, ip]
        lib.fsr_latency_eval.argtypes = [ctypes.POINTER(LatencyModel), ctypes.c_double, ctypes.c_double, ctypes.c_double, dp]
        lib.fsr_latency_fit.argtypes = [ctypes.c_int32, ctypes.c_int32, dp, dp, dp, dp, ctypes.POINTER(LatencyModel), dp]
        lib.fsr_chunk_size.argtypes = [ctypes.POINTER(LatencyModel), ctypes.POINTER(LatencyModel), ctypes.c_double, ctypes.c_double,
                                       ctypes.c_int32, ctypes.c_double, ctypes.c_int32, ip, ip, dp]
        lib._fsr_ctl_ready = True
    return lib


def default_config() -> CtlConfig:
    cfg = CtlConfig()
    _check(_lib().fsr_ctl_default_config(ctypes.byref(cfg)))
    return cfg


def _doubles(values: Sequence[float]):
    return (ctypes.c_double * len(values))(*[float(v) for v in values])


def _ints(values: Sequence[int]):
    return (ctypes.c_int32 * len(values))(*[int(v) for v in values])


class Controller:
    """Per-request speculative lengths: window statistics, Eq. 1-2 estimates and the GP-LCB choice (Eqs. 3-4)."""

    def __init__(self, lengths: Optional[Sequence[int]] = None, **overrides):
        self._lib = _lib()
        cfg = default_config()
        if lengths is not None:
            if len(lengths) > MAX_LENGTHS:
                raise ValueError(f"at most {MAX_LENGTHS} candidate lengths")
            cfg.n_lengths = len(lengths)
            for k, s in enumerate(lengths):
                cfg.lengths[k] = int(s)
        for name, value in overrides.items():
            if not hasattr(cfg, name):
                raise TypeError(f"unknown configuration field {name}")
            setattr(cfg, name, value)
        self.config = cfg
        self.lengths = [cfg.lengths[k] for k in range(cfg.n_lengths)]
        self._h = ctypes.c_void_p()
        _check(self._lib.fsr_ctl_create(ctypes.byref(cfg), ctypes.byref(self._h)))

    def close(self):
        if self._h:
            self._lib.fsr_ctl_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def observe(self, context: int, request: int, s: int, n_accepted: int, latency: float):
        _check(self._lib.fsr_ctl_observe(self._h, context, request, s, n_accepted, latency))

    def forget(self, request: int):
        _check(self._lib.fsr_ctl_forget(self._h, request))

    def estimates(self, context: int, request: int):
        n = len(self.lengths)
        a, t, j = (ctypes.c_double * n)(), (ctypes.c_double * n)(), (ctypes.c_double * n)()
        _check(self._lib.fsr_ctl_estimates(self._h, context, request, a, t, j))
        return list(a), list(t), list(j)

    def best_length(self, context: int, request: int) -> int:
        s = ctypes.c_int32()
        _check(self._lib.fsr_ctl_best_length(self._h, context, request, ctypes.byref(s)))
        return s.value

    def posterior(self, context: int, request: int):
        n = len(self.lengths)
        mu, sigma = (ctypes.c_double * n)(), (ctypes.c_double * n)()
        _check(self._lib.fsr_ctl_posterior(self._h, context, request, mu, sigma))
        return list(mu), list(sigma)

    def choose(self, context: int, request: int) -> int:
        s = ctypes.c_int32()
        _check(self._lib.fsr_ctl_choose(self._h, context, request, ctypes.byref(s)))
        return s.value


def expected_rejected(s: Sequence[int], a_hat: Sequence[float]) -> float:
    out = ctypes.c_double()
    _check(_lib().fsr_expected_rejected(len(s), _ints(s), _doubles(a_hat), ctypes.byref(out)))
    return out.value


def prune_trigger(L: int, layer: int, T_t: float, T_ee: float, T_pr: float):
    save, prune = ctypes.c_double(), ctypes.c_int32()
    _check(_lib().fsr_prune_trigger(L, layer, T_t, T_ee, T_pr, ctypes.byref(save), ctypes.byref(prune)))
    return save.value, bool(prune.value)


def latency_model(form: int, a1, g1, a2, g2, knee, alpha, beta, c=0.0) -> LatencyModel:
    return LatencyModel(form, 0, a1, g1, a2, g2, knee, alpha, beta, c)


def latency_eval(model: LatencyModel, b: float, s: float, r: float) -> float:
    out = ctypes.c_double()
    _check(_lib().fsr_latency_eval(ctypes.byref(model), b, s, r, ctypes.byref(out)))
    return out.value


def latency_fit(form: int, b: Sequence[float], s: Sequence[float], r: Sequence[float], T: Sequence[float]):
    if not (len(b) == len(s) == len(r) == len(T)):
        raise ValueError("b, s, r, T must have one entry per profiled point")
    model, rms = LatencyModel(), ctypes.c_double()
    _check(_lib().fsr_latency_fit(form, len(T), _doubles(b), _doubles(s), _doubles(r), _doubles(T), ctypes.byref(model), ctypes.byref(rms)))
    return model, rms.value


def chunk_size(draft: LatencyModel, target: LatencyModel, b: float, r: float, s: int, T_hat: float, candidates: Sequence[int]):
    sc, t = ctypes.c_int32(), ctypes.c_double()
    _check(_lib().fsr_chunk_size(ctypes.byref(draft), ctypes.byref(target), b, r, s, T_hat, len(candidates), _ints(candidates),
                                 ctypes.byref(sc), ctypes.byref(t)))
    return sc.value, t.value
