"""ctypes front of the CPU oracle (moe_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by the tests, the smoke check and the benchmark's
CPU-baseline leg.  It never imports the GPU package and the GPU package never imports it.
All arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

MODE_NONE, MODE_TOKEN_DROP, MODE_EXPANDED_DROP = 0, 1, 2
SCOPE_LOCAL, SCOPE_GLOBAL, SCOPE_LOCAL_DEVICE, SCOPE_GLOBAL_DEVICE = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp contraction off, OpenMP on)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32, i64, dbl, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.orc_num_threads.restype = i32
        lib.orc_set_num_threads.argtypes = [i32]
        lib.orc_set_num_threads.restype = None
        lib.orc_router_logits.argtypes = [vp, vp, vp, i32, i32, i32, vp]
        lib.orc_router_logits.restype = None
        lib.orc_softmax_scores.argtypes = [vp, i32, i32, vp]
        lib.orc_softmax_scores.restype = None
        lib.orc_topk.argtypes = [vp, i32, i32, i32, vp, vp]
        lib.orc_topk.restype = None
        lib.orc_capacity.argtypes = [dbl, i32, i32, i32]
        lib.orc_capacity.restype = i32
        lib.orc_candidates.argtypes = [vp, i32, i32, i32, i32, i32, vp]
        lib.orc_candidates.restype = None
        lib.orc_capacity_drop.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, dbl, i32, vp, ctypes.c_uint32, vp]
        lib.orc_pair_hash.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
        lib.orc_pair_hash.restype = ctypes.c_uint32
        lib.orc_device_budget.argtypes = [dbl, i32, i32, i32, i32]
        lib.orc_device_budget.restype = i32
        lib.orc_capacity_drop.restype = i64
        lib.orc_limit_experts.argtypes = [vp, i32, i32, i32, vp]
        lib.orc_limit_experts.restype = i64
        lib.orc_build_plan.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        lib.orc_build_plan.restype = i64
        lib.orc_layer_output.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, i32, vp]
        lib.orc_layer_output.restype = i32
        _lib = lib
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_num_threads(n: int) -> None:
    _load().orc_set_num_threads(int(n))


def router_logits(x, w_router, bias=None):
    x, w = _c(x, np.float32), _c(w_router, np.float32)
    n, d = x.shape
    e = w.shape[0]
    assert w.shape == (e, d)
    b = _c(bias, np.float32) if bias is not None else None
    out = np.empty((n, e), np.float32)
    _load().orc_router_logits(_p(x), _p(w), _p(b) if b is not None else None, n, d, e, _p(out))
    return out


def softmax_scores(logits):
    l = _c(logits, np.float32)
    n, e = l.shape
    out = np.empty((n, e), np.float32)
    _load().orc_softmax_scores(_p(l), n, e, _p(out))
    return out


def topk(scores, k):
    s = _c(scores, np.float32)
    n, e = s.shape
    assert 1 <= k <= e
    idx = np.empty((n, k), np.int32)
    val = np.empty((n, k), np.float32)
    _load().orc_topk(_p(s), n, e, k, _p(idx), _p(val))
    return idx, val


def capacity(gamma, seg_tokens, k, n_experts) -> int:
    return int(_load().orc_capacity(float(gamma), seg_tokens, k, n_experts))


def device_budget(gamma, seg_tokens, k, n_experts, experts_per_device) -> int:
    return int(_load().orc_device_budget(float(gamma), seg_tokens, k, n_experts, experts_per_device))


def candidates(topk_idx, n_experts, device_groups, mode):
    idx = _c(topk_idx, np.int32)
    n, k = idx.shape
    assert n % device_groups == 0 and n_experts % device_groups == 0
    cand = np.empty((n, n_experts), np.uint8)
    _load().orc_candidates(_p(idx), n, n_experts, k, device_groups, mode, _p(cand))
    return cand


METRIC_SCORE, METRIC_ORDER, METRIC_REVERSE_ORDER, METRIC_RANDOM = 0, 1, 2, 3


def pair_hash(seed, counter) -> int:
    return int(_load().orc_pair_hash(seed & 0xFFFFFFFF, counter & 0xFFFFFFFF))


def capacity_drop(scores, cand, k, device_groups, mode, scope, gamma, metric=METRIC_SCORE, token_class=None, seed=0):
    s, c = _c(scores, np.float32), _c(cand, np.uint8)
    n, e = s.shape
    assert c.shape == (n, e) and n % device_groups == 0
    keep = np.empty((n, e), np.uint8)
    tc = _c(token_class, np.uint8) if token_class is not None else None
    assert tc is None or tc.shape == (n,)
    kept = _load().orc_capacity_drop(_p(s), _p(c), n, e, k, device_groups, mode, scope, float(gamma), metric,
                                     _p(tc) if tc is not None else None, seed & 0xFFFFFFFF, _p(keep))
    assert kept == int(keep.sum())
    return keep


def limit_experts(scores, keep, k):
    """At most k surviving experts per token ("w/ max"); returns a new keep matrix."""
    s = _c(scores, np.float32)
    out = np.array(keep, dtype=np.uint8, order="C", copy=True)
    n, e = s.shape
    removed = _load().orc_limit_experts(_p(s), n, e, k, _p(out))
    assert removed == int(np.asarray(keep, np.int64).sum() - out.sum())
    return out


class Plan:
    """The dispatch plan of one layer call (all numpy arrays)."""

    def __init__(self, **kw):
        self.__dict__.update(kw)


def slots_per_token(k, n_experts, device_groups, mode, overselect=0) -> int:
    return k + overselect + (n_experts // device_groups if mode == MODE_EXPANDED_DROP else 0)


def build_plan(scores, cand, keep, slots, n_blocks) -> Plan:
    s, c, kp = _c(scores, np.float32), _c(cand, np.uint8), _c(keep, np.uint8)
    n, e = s.shape
    p_max = int(kp.sum())
    expert_count = np.empty(e, np.int32)
    seg_count = np.empty((n_blocks, e), np.int32)
    expert_offset = np.empty(e + 1, np.int32)
    row_token = np.empty(max(p_max, 1), np.int32)
    row_weight = np.empty(max(p_max, 1), np.float32)
    pair_row = np.empty((n, slots), np.int32)
    rows = _load().orc_build_plan(_p(s), _p(c), _p(kp), n, e, slots, n_blocks, _p(expert_count), _p(seg_count),
                                  _p(expert_offset), _p(row_token), _p(row_weight), _p(pair_row))
    assert rows == p_max
    return Plan(rows=p_max, expert_count=expert_count, seg_count=seg_count, expert_offset=expert_offset,
                row_token=row_token[:p_max], row_weight=row_weight[:p_max], pair_row=pair_row)


def route_and_drop(logits, k, device_groups, mode, scope, gamma, metric=METRIC_SCORE, token_class=None, seed=0,
                   overselect=0, max_experts=False):
    """softmax -> top-(k+overselect) -> candidates -> drop (-> at most k per token) -> plan, from fp32 logits.

    The capacity always uses the model's k; `overselect` only widens the candidate lists.
    """
    scores = softmax_scores(logits)
    topk_idx, topk_score = topk(scores, k + overselect)
    n, e = scores.shape
    cand = candidates(topk_idx, e, device_groups, mode)
    keep = capacity_drop(scores, cand, k, device_groups, mode, scope, gamma, metric, token_class, seed)
    if max_experts:
        keep = limit_experts(scores, keep, k)
    n_blocks = device_groups if scope in (SCOPE_LOCAL, SCOPE_LOCAL_DEVICE) else 1
    plan = build_plan(scores, cand, keep, slots_per_token(k, e, device_groups, mode, overselect), n_blocks)
    seg_tokens = n // n_blocks
    span = e // device_groups if scope in (SCOPE_LOCAL_DEVICE, SCOPE_GLOBAL_DEVICE) else 1
    if mode == MODE_NONE:
        cap = seg_tokens * span
    elif span > 1 or scope in (SCOPE_LOCAL_DEVICE, SCOPE_GLOBAL_DEVICE):
        cap = device_budget(gamma, seg_tokens, k, e, span)
    else:
        cap = capacity(gamma, seg_tokens, k, e)
    return Plan(scores=scores, topk_idx=topk_idx, topk_score=topk_score, cand=cand, keep=keep, cap=cap, plan=plan)


def layer_output(x, scores, keep, w_gate, w_up, w_down, token_list=None):
    """y (fp64) for all tokens or for `token_list`.

    w_gate / w_up / w_down: sequences of length E of fp32 arrays ([h,d], [h,d], [d,h]) or None
    for experts that no listed token keeps.
    """
    x, s, kp = _c(x, np.float32), _c(scores, np.float32), _c(keep, np.uint8)
    n, d = x.shape
    e = s.shape[1]
    hold = []

    def table(ws, shape_of):
        arr = (ctypes.c_void_p * e)()
        for i, w in enumerate(ws):
            if w is None:
                arr[i] = None
            else:
                wc = _c(w, np.float32)
                assert wc.shape == shape_of, (wc.shape, shape_of)
                hold.append(wc)
                arr[i] = wc.ctypes.data
        return arr

    h = next(w for w in w_gate if w is not None).shape[0]
    tg, tu, td = table(w_gate, (h, d)), table(w_up, (h, d)), table(w_down, (d, h))
    if token_list is not None:
        tl = _c(token_list, np.int32)
        n_list = tl.shape[0]
        tlp = _p(tl)
    else:
        n_list, tlp = n, None
    y = np.empty((n_list, d), np.float64)
    st = _load().orc_layer_output(_p(x), _p(s), _p(kp), tg, tu, td, n, d, e, h, tlp, n_list, _p(y))
    if st != 0:
        raise ValueError("a listed token keeps an expert whose weights were not supplied")
    return y


def is_inf(gamma) -> bool:
    return math.isinf(gamma)
