"""ctypes binding of the host-side scheduling helpers (include/medha_policy.h): argument
marshalling only; every computation runs in the shared library."""
import ctypes
from typing import Optional, Sequence, Tuple

import numpy as np

from .binding import load_library

EXPORTS = (
    "medha_policy_chunk_time",
    "medha_policy_fit_time_model",
    "medha_policy_max_chunk",
    "medha_policy_get_chunk_size",
    "medha_policy_simulate_prefill",
    "medha_policy_build_prefill_cache",
    "medha_policy_remaining_time",
    "medha_policy_relative_slack",
    "medha_policy_simulate_schedule",
)

FCFS, EDF, LARS = 0, 1, 2


class TimeModel(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("t_fixed", "t_token", "t_pair", "t_decode",
                                               "t_decode_key")]


_READY = False


def _lib():
    global _READY
    lib = load_library()
    if not _READY:
        f64, i64, i32, vp = ctypes.c_double, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        mp = ctypes.POINTER(TimeModel)
        lib.medha_policy_chunk_time.restype = f64
        lib.medha_policy_chunk_time.argtypes = [mp, i64, i64]
        lib.medha_policy_fit_time_model.restype = ctypes.c_int
        lib.medha_policy_fit_time_model.argtypes = [vp, vp, vp, i32, mp, ctypes.POINTER(f64)]
        lib.medha_policy_max_chunk.restype = i64
        lib.medha_policy_max_chunk.argtypes = [mp, i64, f64, i64]
        lib.medha_policy_get_chunk_size.restype = i64
        lib.medha_policy_get_chunk_size.argtypes = [mp, i64, i64, i32, i32, f64, f64, f64, f64, i64]
        lib.medha_policy_simulate_prefill.restype = f64
        lib.medha_policy_simulate_prefill.argtypes = [mp, i64, f64, i64]
        lib.medha_policy_build_prefill_cache.restype = ctypes.c_int
        lib.medha_policy_build_prefill_cache.argtypes = [mp, i64, i64, f64, i64, vp, i64]
        lib.medha_policy_remaining_time.restype = f64
        lib.medha_policy_remaining_time.argtypes = [vp, i64, i64, i64, i64]
        lib.medha_policy_relative_slack.restype = f64
        lib.medha_policy_relative_slack.argtypes = [f64] * 5
        lib.medha_policy_simulate_schedule.restype = ctypes.c_int
        lib.medha_policy_simulate_schedule.argtypes = [i32, vp, vp, vp, i32, f64, vp, vp]
        _READY = True
    return lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def chunk_time(model: TimeModel, kv_size: int, chunk: int) -> float:
    return float(_lib().medha_policy_chunk_time(ctypes.byref(model), kv_size, chunk))


def fit_time_model(kv_size: Sequence[int], chunk: Sequence[int],
                   seconds: Sequence[float]) -> Tuple[TimeModel, float]:
    kv = np.ascontiguousarray(kv_size, np.int64)
    ch = np.ascontiguousarray(chunk, np.int64)
    sec = np.ascontiguousarray(seconds, np.float64)
    model, err = TimeModel(), ctypes.c_double(0.0)
    if _lib().medha_policy_fit_time_model(_p(kv), _p(ch), _p(sec), len(sec), ctypes.byref(model),
                                          ctypes.byref(err)) != 0:
        raise ValueError("fit_time_model: bad samples or singular system")
    return model, err.value


def max_chunk(model: TimeModel, kv_size: int, t_budget: float, max_chunk_tokens: int) -> int:
    r = int(_lib().medha_policy_max_chunk(ctypes.byref(model), kv_size, t_budget,
                                          max_chunk_tokens))
    if r < 0:
        raise ValueError("max_chunk: bad arguments")
    return r


def get_chunk_size(model: TimeModel, kv_size: int, remaining: int, is_long: bool,
                   batch_has_long: bool, rel_slack: float, rho_max: float, t_current: float,
                   t_target: float, max_chunk_tokens: int) -> int:
    r = int(_lib().medha_policy_get_chunk_size(ctypes.byref(model), kv_size, remaining,
                                               int(is_long), int(batch_has_long), rel_slack,
                                               rho_max, t_current, t_target, max_chunk_tokens))
    if r < 0:
        raise ValueError("get_chunk_size: bad arguments")
    return r


def simulate_prefill(model: TimeModel, length: int, t_target: float,
                     max_chunk_tokens: int) -> float:
    return float(_lib().medha_policy_simulate_prefill(ctypes.byref(model), length, t_target,
                                                      max_chunk_tokens))


def build_prefill_cache(model: TimeModel, l_max: int, delta: int, t_target: float,
                        max_chunk_tokens: int) -> np.ndarray:
    cache = np.empty(l_max // delta + 1, np.float64)
    if _lib().medha_policy_build_prefill_cache(ctypes.byref(model), l_max, delta, t_target,
                                               max_chunk_tokens, _p(cache), len(cache)) != 0:
        raise ValueError("build_prefill_cache: bad arguments")
    return cache


def remaining_time(cache: np.ndarray, delta: int, l_total: int, l_processed: int) -> float:
    cache = np.ascontiguousarray(cache, np.float64)
    return float(_lib().medha_policy_remaining_time(_p(cache), len(cache), delta, l_total,
                                                    l_processed))


def relative_slack(arrival: float, deadline: float, now: float, remaining_work: float,
                   total_work: float) -> float:
    return float(_lib().medha_policy_relative_slack(arrival, deadline, now, remaining_work,
                                                    total_work))


def simulate_schedule(policy: int, arrival, work, deadline, quantum: float):
    a = np.ascontiguousarray(arrival, np.float64)
    w = np.ascontiguousarray(work, np.float64)
    d = np.ascontiguousarray(deadline, np.float64)
    finish = np.zeros(len(a), np.float64)
    start = np.zeros(len(a), np.float64)
    if _lib().medha_policy_simulate_schedule(policy, _p(a), _p(w), _p(d), len(a), quantum,
                                             _p(finish), _p(start)) != 0:
        raise ValueError("simulate_schedule: bad arguments")
    return finish, start
