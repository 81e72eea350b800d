"""ctypes binding of include/kvc_policy.h: the host-side KV-cache scheduling policy (CPU only).

Same names as the C ABI without the ``kvcp_`` prefix; argument marshalling only.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

_PKG = os.path.dirname(os.path.abspath(__file__))
# KVC_POLICY_LIBRARY points at another build of the same source (the sanitizer run of the tests)
_LIB_PATH = os.environ.get("KVC_POLICY_LIBRARY") or os.path.join(_PKG, "libkvc_policy.so")
_lib = None

_i64, _f64, _i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_int32
_pi64, _pf64, _pi32 = ctypes.POINTER(_i64), ctypes.POINTER(_f64), ctypes.POINTER(_i32)


WAITING, RUNNING = 0, 1
KEEP, PREEMPT_SWAP, PREEMPT_RECOMPUTE = 0, 1, 2
CASE_EQUAL, CASE_LESS, CASE_MORE = 0, 1, 2


class Request(ctypes.Structure):
    """kvcp_request"""
    _fields_ = [("state", _i32), ("reserved", _i32), ("prompt_len", _i64), ("est_output_len", _i64),
                ("generated", _i64), ("allocated", _i64), ("used", _i64), ("remaining_time", _f64),
                ("tbt_slo", _f64)]


class StepParams(ctypes.Structure):
    """kvcp_step_params"""
    _fields_ = [("unallocated", _i64), ("block_tokens", _i64), ("buffer_tokens", _i64),
                ("token_budget", _i64), ("token_bucket", _i64), ("m", _i32), ("n_slo_edges", _i32),
                ("slo_edges", _pf64), ("max_iteration_latency", _f64), ("eps", _f64),
                ("iter_time_base", _f64), ("iter_time_per_token", _f64), ("sweet_spot", _f64)]


class Decision(ctypes.Structure):
    """kvcp_decision"""
    _fields_ = [("in_batch", _i32), ("critical", _i32), ("preempt", _i32), ("proactive", _i32),
                ("grant", _i64), ("host", _i64), ("s0", _i64), ("lender", _i64), ("shortfall", _i64)]


class StepSummary(ctypes.Structure):
    """kvcp_step_summary"""
    _fields_ = [("unallocated_after", _i64), ("basic_demand", _i64), ("excess", _i64),
                ("batch_tokens", _i64), ("n_preempted", _i32), ("alloc_case", _i32)]


def library_path() -> str:
    return _LIB_PATH


def lib():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: run `python -m paper_2503_13773_amd.build`")
    L = ctypes.CDLL(_LIB_PATH)
    sig = {
        "kvcp_confidence": (_f64, [_f64, _f64, _f64]),
        "kvcp_padding": (_f64, [_f64, _f64]),
        "kvcp_estimated_output_len": (_f64, [_f64, _f64, _f64, ctypes.c_int]),
        "kvcp_embedding_fits": (ctypes.c_int, [_i64, _i64, _i64, _i64, _i64, _pi64]),
        "kvcp_embedding_choose": (_i64, [_pi64, _pi64, _i64, _i64, _i64, _i64, _pi64]),
        "kvcp_is_critical": (ctypes.c_int, [_f64, _f64, _f64]),
        "kvcp_basic_demand": (_i64, [_pi64, _i64, _i64, _i64]),
        "kvcp_allocate": (ctypes.c_int, [_pi64, _pf64, _pi64, _i64, _i64, _pi64, _pi64]),
        "kvcp_preemption_order": (ctypes.c_int, [_pf64, _pi64, _pi64, _i64, _pf64, _i32, _i64, _pi64]),
        "kvcp_sweet_spot": (_f64, [_f64] * 7),
        "kvcp_choose_swap": (ctypes.c_int, [_f64, _f64]),
        "kvcp_fit_linear": (ctypes.c_int, [_pf64, _pf64, _i64, _pf64, _pf64, _pf64]),
        "kvcp_fit_power_law": (ctypes.c_int, [_pf64, _pf64, _i64, _pf64, _pf64, _pf64]),
        "kvcp_schedule_step": (ctypes.c_int, [ctypes.POINTER(Request), _i64, ctypes.POINTER(StepParams),
                                              ctypes.POINTER(Decision), ctypes.POINTER(StepSummary)]),
        "kvcp_embedding_block_range": (ctypes.c_int, [_i64, _i64, _i64, _i64, _i64, _i64, _pi64, _pi64]),
        "kvcp_bm_create": (ctypes.c_void_p, [_i64, _i64]),
        "kvcp_bm_destroy": (None, [ctypes.c_void_p]),
        "kvcp_bm_free_general": (_i64, [ctypes.c_void_p]),
        "kvcp_bm_free_reserved": (_i64, [ctypes.c_void_p]),
        "kvcp_bm_allocate": (ctypes.c_int, [ctypes.c_void_p, _i64, _pi32]),
        "kvcp_bm_allocate_reserved": (ctypes.c_int, [ctypes.c_void_p, _i64, _pi32]),
        "kvcp_bm_release": (ctypes.c_int, [ctypes.c_void_p, _pi32, _i64]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def _arr(ctype, values):
    values = list(values)
    return (ctype * len(values))(*values) if values else None


def confidence(alpha: float, beta: float, arrival_rate: float) -> float:
    return lib().kvcp_confidence(alpha, beta, arrival_rate)


def padding(range_: float, confidence_: float) -> float:
    return lib().kvcp_padding(range_, confidence_)


def estimated_output_len(predicted: float, range_: float, confidence_: float, underpredicted: bool) -> float:
    return lib().kvcp_estimated_output_len(predicted, range_, confidence_, int(bool(underpredicted)))


def embedding_fits(a_j: int, u_j: int, sp_i: int, so_i: int, b: int) -> Optional[int]:
    """s0 (the room left for request i inside r_j's allocation) when it fits, else None."""
    s0 = _i64()
    return int(s0.value) if lib().kvcp_embedding_fits(a_j, u_j, sp_i, so_i, b, ctypes.byref(s0)) else None


def embedding_choose(a: Sequence[int], u: Sequence[int], sp_i: int, so_i: int, b: int) -> Optional[Tuple[int, int]]:
    """(index of the chosen running request, s0) or None."""
    s0 = _i64()
    j = lib().kvcp_embedding_choose(_arr(_i64, a), _arr(_i64, u), len(a), sp_i, so_i, b, ctypes.byref(s0))
    return (int(j), int(s0.value)) if j >= 0 else None


def is_critical(remaining_time: float, max_iteration_latency: float, eps: float) -> bool:
    return bool(lib().kvcp_is_critical(remaining_time, max_iteration_latency, eps))


def basic_demand(sp_critical_waiting: Sequence[int], n_returned: int, B: int) -> int:
    d = lib().kvcp_basic_demand(_arr(_i64, sp_critical_waiting), len(sp_critical_waiting), n_returned, B)
    if d < 0:
        raise ValueError("bad arguments")
    return int(d)


def allocate(M: Sequence[int], RT: Sequence[float], sp: Sequence[int], A_avail: int) -> Tuple[List[int], int]:
    """(allocation per request, slack): slack >= 0 is unallocated room, < 0 is minus the excess demand."""
    n = len(M)
    out = (_i64 * max(n, 1))()
    slack = _i64()
    rc = lib().kvcp_allocate(_arr(_i64, M), _arr(_f64, RT), _arr(_i64, sp), n, A_avail, out, ctypes.byref(slack))
    if rc != 0:
        raise ValueError("bad arguments")
    return [int(out[i]) for i in range(n)], int(slack.value)


def preemption_order(tbt_slo: Sequence[float], remaining_tokens: Sequence[int], occupied_kvc: Sequence[int],
                     slo_edges: Sequence[float] = (0.2, 0.5), token_bucket: int = 128) -> List[int]:
    n = len(tbt_slo)
    out = (_i64 * max(n, 1))()
    rc = lib().kvcp_preemption_order(_arr(_f64, tbt_slo), _arr(_i64, remaining_tokens), _arr(_i64, occupied_kvc),
                                     n, _arr(_f64, slo_edges), len(list(slo_edges)), token_bucket, out)
    if rc != 0:
        raise ValueError("bad arguments")
    return [int(out[i]) for i in range(n)]


def sweet_spot(gamma_s: float, delta_s: float, alpha_r: float, beta_r: float, kappa_r: float = 0.0,
               eps_r: float = 0.0, s_max: float = 1e7) -> float:
    return lib().kvcp_sweet_spot(gamma_s, delta_s, alpha_r, beta_r, kappa_r, eps_r, s_max)


def choose_swap(seq_len: float, sweet_spot_: float) -> bool:
    return bool(lib().kvcp_choose_swap(seq_len, sweet_spot_))


def fit_linear(x: Sequence[float], y: Sequence[float]) -> Tuple[float, float, float]:
    """(gamma, delta, r2) of the least-squares line y = gamma x + delta (kvcp_fit_linear)."""
    g, d, r2 = _f64(), _f64(), _f64()
    if len(x) != len(y) or lib().kvcp_fit_linear(_arr(_f64, x), _arr(_f64, y), len(x), ctypes.byref(g),
                                                 ctypes.byref(d), ctypes.byref(r2)) != 0:
        raise ValueError("need at least two finite samples with distinct x")
    return g.value, d.value, r2.value


def fit_power_law(x: Sequence[float], y: Sequence[float]) -> Tuple[float, float, float]:
    """(alpha, beta, r2) of y = alpha x^beta fitted in log-log space (kvcp_fit_power_law)."""
    a, b, r2 = _f64(), _f64(), _f64()
    if len(x) != len(y) or lib().kvcp_fit_power_law(_arr(_f64, x), _arr(_f64, y), len(x), ctypes.byref(a),
                                                    ctypes.byref(b), ctypes.byref(r2)) != 0:
        raise ValueError("need at least two positive samples with distinct x")
    return a.value, b.value, r2.value


def schedule_step(requests: Sequence[Request], *, unallocated: int, block_tokens: int = 8,
                  buffer_tokens: int = 8, token_budget: int = 2048, token_bucket: int = 128, m: int = 2,
                  slo_edges: Sequence[float] = (0.2, 0.5), max_iteration_latency: float = 0.0,
                  eps: float = 0.0, iter_time_base: float = 0.0, iter_time_per_token: float = 0.0,
                  sweet_spot: float = 0.0) -> Tuple[List[Decision], StepSummary]:
    """kvcp_schedule_step: one decision per request (same order) and the step summary."""
    n = len(requests)
    reqs = (Request * max(n, 1))(*requests)
    out = (Decision * max(n, 1))()
    edges = _arr(_f64, slo_edges)
    params = StepParams(unallocated=unallocated, block_tokens=block_tokens, buffer_tokens=buffer_tokens,
                        token_budget=token_budget, token_bucket=token_bucket, m=m,
                        n_slo_edges=len(list(slo_edges)),
                        slo_edges=ctypes.cast(edges, _pf64) if edges is not None else None,
                        max_iteration_latency=max_iteration_latency, eps=eps,
                        iter_time_base=iter_time_base, iter_time_per_token=iter_time_per_token,
                        sweet_spot=sweet_spot)
    summary = StepSummary()
    if lib().kvcp_schedule_step(reqs, n, ctypes.byref(params), out, ctypes.byref(summary)) != 0:
        raise ValueError("kvcp_schedule_step rejected its arguments")
    return [out[i] for i in range(n)], summary


def embedding_block_range(a_j: int, s0: int, sp_i: int, so_i: int, block_size: int,
                          host_blocks: int) -> Optional[Tuple[int, int]]:
    """(first block, block count) inside the host's block list, or None when it does not fit."""
    first, count = _i64(), _i64()
    rc = lib().kvcp_embedding_block_range(a_j, s0, sp_i, so_i, block_size, host_blocks, ctypes.byref(first),
                                          ctypes.byref(count))
    return (int(first.value), int(count.value)) if rc == 0 else None


class BlockManager:
    """Free-list block allocator with a shared reserved pool (the last `reserved_blocks` ids)."""

    def __init__(self, num_blocks: int, reserved_blocks: int = 0):
        self._h = lib().kvcp_bm_create(num_blocks, reserved_blocks)
        if not self._h:
            raise ValueError("bad arguments")

    def __del__(self):
        if getattr(self, "_h", None):
            lib().kvcp_bm_destroy(self._h)
            self._h = None

    @property
    def free_general(self) -> int:
        return int(lib().kvcp_bm_free_general(self._h))

    @property
    def free_reserved(self) -> int:
        return int(lib().kvcp_bm_free_reserved(self._h))

    def _take(self, fn, n: int) -> Optional[List[int]]:
        out = (_i32 * max(n, 1))()
        return [int(out[i]) for i in range(n)] if fn(self._h, n, out) == 0 else None

    def allocate(self, n: int) -> Optional[List[int]]:
        """n blocks from the general pool, or None (nothing taken) when fewer are free."""
        return self._take(lib().kvcp_bm_allocate, n)

    def allocate_reserved(self, n: int) -> Optional[List[int]]:
        return self._take(lib().kvcp_bm_allocate_reserved, n)

    def release(self, ids: Sequence[int]) -> None:
        ids = list(ids)
        if lib().kvcp_bm_release(self._h, _arr(_i32, ids), len(ids)) != 0:
            raise ValueError("release of a block that is out of range, repeated or not allocated")
