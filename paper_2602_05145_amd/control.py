"""ctypes binding of libtide_control.so (host-only adaptive control): the same names as the C ABI."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtide_control.so")

EXPORTED = [
    "tide_expected_accept_length", "tide_sd_latency", "tide_theoretical_speedup", "tide_speedup",
    "tide_profile_latency", "tide_practical_speedup", "tide_min_acceptance", "tide_should_speculate",
    "tide_controller_init", "tide_controller_observe", "tide_controller_train_alpha", "tide_controller_report",
]

STORE, TRAIN = 1, 2
DEPLOY, STOP_COLLECTING, KEEP = 1, 2, 3


class LatencyProfile(C.Structure):
    _fields_ = [("n_points", C.c_int32), ("n", C.POINTER(C.c_int32)), ("t", C.POINTER(C.c_double)), ("d0", C.c_double)]


class ControllerParams(C.Structure):
    _fields_ = [("lambda_short", C.c_double), ("lambda_long", C.c_double), ("epsilon", C.c_double),
                ("n_init", C.c_int32), ("n_threshold", C.c_int32), ("train_fraction", C.c_double)]


class Controller(C.Structure):
    _fields_ = [("prm", ControllerParams), ("n_seen", C.c_int64), ("init_sum", C.c_double),
                ("ema_short", C.c_double), ("ema_long", C.c_double), ("collection_enabled", C.c_int32),
                ("n_stored", C.c_int32), ("n_train", C.c_int32), ("train_alpha_sum", C.c_double),
                ("awaiting_result", C.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python paper_2602_05145_amd/build.py` first")
    return C.CDLL(LIB_PATH)


_lib = _load()
_d, _i = C.c_double, C.c_int
_pp = C.POINTER(LatencyProfile)
for _name, _res, _args in [
    ("tide_expected_accept_length", _d, [_d, _i]),
    ("tide_sd_latency", _d, [_d, _i, _d, _d]),
    ("tide_theoretical_speedup", _d, [_d, _i, _d]),
    ("tide_speedup", _d, [_d, _i, _d, _d, _d]),
    ("tide_profile_latency", _d, [_pp, _d]),
    ("tide_practical_speedup", _d, [_pp, _d, _i, C.c_int32]),
    ("tide_min_acceptance", _d, [_pp, _i, C.c_int32]),
    ("tide_should_speculate", _i, [_pp, _d, _i, C.c_int32, _d]),
    ("tide_controller_init", _i, [C.POINTER(Controller), C.POINTER(ControllerParams)]),
    ("tide_controller_observe", _i, [C.POINTER(Controller), _d]),
    ("tide_controller_train_alpha", _d, [C.POINTER(Controller)]),
    ("tide_controller_report", _i, [C.POINTER(Controller), _d]),
]:
    getattr(_lib, _name).restype = _res
    getattr(_lib, _name).argtypes = _args


def lib():
    return _lib


def make_profile(ns, ts, d0):
    """Returns (LatencyProfile, keepalive): the struct points into the two ctypes arrays."""
    n_arr = (C.c_int32 * len(ns))(*[int(v) for v in ns])
    t_arr = (C.c_double * len(ts))(*[float(v) for v in ts])
    p = LatencyProfile(len(ns), n_arr, t_arr, float(d0))
    return p, (n_arr, t_arr)


tide_expected_accept_length = _lib.tide_expected_accept_length
tide_sd_latency = _lib.tide_sd_latency
tide_theoretical_speedup = _lib.tide_theoretical_speedup
tide_speedup = _lib.tide_speedup


def tide_profile_latency(p, n_tokens):
    return _lib.tide_profile_latency(C.byref(p) if p is not None else None, float(n_tokens))


def tide_practical_speedup(p, alpha, gamma, batch):
    return _lib.tide_practical_speedup(C.byref(p) if p is not None else None, float(alpha), int(gamma), int(batch))


def tide_min_acceptance(p, gamma, batch):
    return _lib.tide_min_acceptance(C.byref(p) if p is not None else None, int(gamma), int(batch))


def tide_should_speculate(p, alpha, gamma, batch, margin=1.0):
    return _lib.tide_should_speculate(C.byref(p) if p is not None else None, float(alpha), int(gamma), int(batch), float(margin))


def tide_controller_init(c, prm):
    return _lib.tide_controller_init(C.byref(c) if c is not None else None, C.byref(prm) if prm is not None else None)


def tide_controller_observe(c, alpha):
    return _lib.tide_controller_observe(C.byref(c), float(alpha))


def tide_controller_train_alpha(c):
    return _lib.tide_controller_train_alpha(C.byref(c))


def tide_controller_report(c, alpha_eval):
    return _lib.tide_controller_report(C.byref(c), float(alpha_eval))
