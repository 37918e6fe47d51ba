"""Python front-end of the CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It compiles ``adaptra_oracle.c`` with gcc
and calls it through ctypes; the per-scenario search and the bubble histogram
are written out in numpy on top of the simulator's outputs.  Nothing here is
shared with the GPU path.

Parity status: every function below is pinned by ``tests/test_oracle_pins.py``
(explicit-DAG longest path, closed forms, brute force, invariants).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adaptra_oracle.c")
_SRC_ZB = os.path.join(_HERE, "zb_oracle.c")
_LIB = os.path.join(_HERE, "libadaptra_oracle.so")
_lib = None

INT32_MAX = 2 ** 31 - 1
FLAG_OK, FLAG_DEADLOCK, FLAG_MEMCAP = 1, 2, 4


def build(force: bool = False) -> str:
    """Compile the simulator (gcc, -O2).  Building the checker is not using it."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_ZB))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-pthread", _SRC, _SRC_ZB, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        p32 = ctypes.POINTER(ctypes.c_int32)
        p64 = ctypes.POINTER(ctypes.c_int64)
        pu8 = ctypes.POINTER(ctypes.c_uint8)
        lib.adaptra_oracle_eval.restype = ctypes.c_int64
        lib.adaptra_oracle_eval.argtypes = [
            ctypes.c_int, ctypes.c_int, p32, p32, p32,
            ctypes.c_int64, p32, ctypes.c_int64, p32, p32,
            ctypes.c_int64, p64, p64, p32, p32, pu8, p32, ctypes.c_int]
        lib.adaptra_oracle_timeline.restype = ctypes.c_int
        lib.adaptra_oracle_timeline.argtypes = [
            ctypes.c_int, ctypes.c_int, p32, p32, p32, p32, p32,
            p64, p64, p64, p64, p64, p32, p64]
        lib.adaptra_oracle_zb.restype = ctypes.c_int64
        lib.adaptra_oracle_zb.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, p32, p32, p32, p32, p32, p32, p32,
                                          p32, p64, p64, p64]
        lib.adaptra_oracle_zb_batch.restype = ctypes.c_int64
        lib.adaptra_oracle_zb_batch.argtypes = [ctypes.c_int, ctypes.c_int, p32, p32, p32, ctypes.c_int64, p32,
                                                ctypes.c_int64, p32, p32, p32, p32]
        _lib = lib
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _c32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def default_threads() -> int:
    return len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)


def eval_pairs(S: int, M: int, t_f, t_b, mem_cap, w, c_fwd, c_bwd, *,
               pair_cand=None, pair_scen=None, want_bubble: bool = True,
               want_peak: bool = False, threads: Optional[int] = None) -> dict:
    """Simulate pairs.  w is [S, C]; c_fwd / c_bwd are [S-1, K].

    Without a pair list every pair is simulated and the outputs are shaped
    [K, C] (bubble / peak: [S, K, C]); with one they are [n] (and [S, n]).
    """
    lib = _load()
    t_f, t_b, mem_cap, w = _c32(t_f), _c32(t_b), _c32(mem_cap), _c32(w)
    c_fwd, c_bwd = _c32(c_fwd), _c32(c_bwd)
    C, K = int(w.shape[1]), int(c_fwd.shape[1])
    assert w.shape == (S, C) and c_fwd.shape == (S - 1, K) and c_bwd.shape == (S - 1, K)
    if pair_cand is None:
        n = C * K
        pc = ps = None
    else:
        pc = np.ascontiguousarray(pair_cand, dtype=np.int64)
        ps = np.ascontiguousarray(pair_scen, dtype=np.int64)
        n = len(pc)
        assert len(ps) == n
        if n and (pc.min() < 0 or pc.max() >= C or ps.min() < 0 or ps.max() >= K):
            raise ValueError("pair index out of range")
    mk = np.empty(n, dtype=np.int32)
    fl = np.empty(n, dtype=np.uint8)
    bub = np.empty((S, n), dtype=np.int32) if want_bubble else None
    peak = np.empty((S, n), dtype=np.int32) if want_peak else None
    rc = lib.adaptra_oracle_eval(S, M, _p(t_f, ctypes.c_int32), _p(t_b, ctypes.c_int32),
                                 _p(mem_cap, ctypes.c_int32), C, _p(w, ctypes.c_int32),
                                 K, _p(c_fwd, ctypes.c_int32), _p(c_bwd, ctypes.c_int32),
                                 n, _p(pc, ctypes.c_int64), _p(ps, ctypes.c_int64),
                                 _p(mk, ctypes.c_int32), _p(bub, ctypes.c_int32),
                                 _p(fl, ctypes.c_uint8), _p(peak, ctypes.c_int32),
                                 int(threads or default_threads()))
    if rc < 0:
        raise ValueError(f"oracle rejected the inputs (code {rc})")
    if rc > 0:
        raise OverflowError(f"{rc} makespans do not fit int32")
    if pair_cand is None:
        mk, fl = mk.reshape(K, C), fl.reshape(K, C)
        bub = None if bub is None else bub.reshape(S, K, C)
        peak = None if peak is None else peak.reshape(S, K, C)
    return {"makespan": mk, "flag": fl, "bubble": bub, "peak": peak}


def eval_workload(wl, **kw) -> dict:
    return eval_pairs(wl.S, wl.M, wl.t_f, wl.t_b, wl.mem_cap, wl.w, wl.c_fwd, wl.c_bwd, **kw)


def eval_scenario_times(S: int, M: int, t_f_scen, t_b_scen, mem_cap, w, c_fwd, c_bwd, **kw) -> dict:
    """Computation stragglers (Section 2.2): scenario k has its own stage times
    t_f_scen[:, k], t_b_scen[:, k] ([S, K]).  One plain simulation per scenario; outputs
    shaped as eval_pairs' full sweep ([K, C], bubble [S, K, C])."""
    t_f_scen, t_b_scen = _c32(t_f_scen), _c32(t_b_scen)
    c_fwd, c_bwd = _c32(c_fwd), _c32(c_bwd)
    K = t_f_scen.shape[1]
    rows = [eval_pairs(S, M, t_f_scen[:, k], t_b_scen[:, k], mem_cap, w,
                       c_fwd[:, k:k + 1], c_bwd[:, k:k + 1], **kw) for k in range(K)]
    out = {"makespan": np.concatenate([r["makespan"] for r in rows], axis=0),
           "flag": np.concatenate([r["flag"] for r in rows], axis=0)}
    for name in ("bubble", "peak"):
        out[name] = None if rows[0][name] is None else np.concatenate([r[name] for r in rows], axis=1)
    return out


def sensitivity(S: int, M: int, t_f, t_b, mem_cap, w, c_fwd, c_bwd, delta: int = 1, *,
                direction: str = "fwd", t_f_scen=None, t_b_scen=None) -> dict:
    """Which link's delay is on the critical path (Section 3.1, Theorem 1), by plain
    perturb-and-simulate: sens[c, l, k] = makespan with the delay of link l (forward
    direction, or backward with direction="bwd") raised by delta, minus the makespan of
    the scenario as given.  INT32_MAX where the candidate is deadlocked.
    Returns makespan / flag [C, K] and sens [C, S-1, K]."""
    def run(cf, cb):
        if t_f_scen is None:
            r = eval_pairs(S, M, t_f, t_b, mem_cap, w, cf, cb, want_bubble=False)
        else:
            r = eval_scenario_times(S, M, t_f_scen, t_b_scen, mem_cap, w, cf, cb, want_bubble=False)
        return r["makespan"].T.astype(np.int64), r["flag"].T
    c_fwd, c_bwd = _c32(c_fwd), _c32(c_bwd)
    base, flag = run(c_fwd, c_bwd)
    C, K = base.shape
    sens = np.empty((C, max(S - 1, 0), K), dtype=np.int64)
    for l in range(S - 1):
        cf, cb = c_fwd.copy(), c_bwd.copy()
        (cf if direction == "fwd" else cb)[l] += delta
        up, _ = run(cf, cb)
        sens[:, l, :] = up - base
    dead = (flag & FLAG_DEADLOCK) != 0
    sens[np.broadcast_to(dead[:, None, :], sens.shape)] = INT32_MAX
    return {"makespan": base.astype(np.int32), "flag": flag, "sens": sens.astype(np.int32)}


def best_from_eval(makespan: np.ndarray, flag: np.ndarray, bubble: Optional[np.ndarray] = None) -> dict:
    """Per-scenario search, written out: among candidates whose flag is 1 take the
    smallest makespan, ties to the lowest candidate index; -1 / INT32_MAX (and
    INT32_MAX bubbles) when no candidate is feasible.  Inputs are [K, C] ([S, K, C])."""
    K, C = makespan.shape
    idx = np.full(K, -1, dtype=np.int32)
    val = np.full(K, INT32_MAX, dtype=np.int32)
    bb = None if bubble is None else np.full((K, bubble.shape[0]), INT32_MAX, dtype=np.int32)
    for k in range(K):
        ok = np.flatnonzero(flag[k] == FLAG_OK)
        if len(ok) == 0:
            continue
        j = ok[np.argmin(makespan[k, ok])]       # argmin returns the first minimum
        idx[k] = j
        val[k] = makespan[k, j]
        if bb is not None:
            bb[k] = bubble[:, k, j]
    return {"best_idx": idx, "best_makespan": val, "best_bubble": bb}


def hist_from_eval(bubble: np.ndarray, flag: np.ndarray, bins: int, shift: int) -> np.ndarray:
    """Per-stage histogram of bubble times over feasible pairs: bin = min(bins-1, bubble >> shift).
    bubble is [S, K, C], flag [K, C]; returns uint64 [S, bins]."""
    S = bubble.shape[0]
    ok = (flag == FLAG_OK)
    out = np.zeros((S, bins), dtype=np.uint64)
    for s in range(S):
        b = np.minimum(bins - 1, bubble[s][ok].astype(np.int64) >> shift)
        out[s] = np.bincount(b, minlength=bins).astype(np.uint64)
    return out


def timeline(S: int, M: int, t_f, t_b, w, cf, cb) -> dict:
    """Start / finish time of every op of one pair (w [S], cf / cb [S-1])."""
    lib = _load()
    t_f, t_b, w = _c32(t_f), _c32(t_b), _c32(w)
    cf = _c32(cf if S > 1 else np.zeros(0))
    cb = _c32(cb if S > 1 else np.zeros(0))
    a = {k: np.empty((S, M), dtype=np.int64) for k in ("start_f", "fin_f", "start_b", "fin_b")}
    idle = np.empty(S, dtype=np.int64)
    peak = np.empty(S, dtype=np.int32)
    mk = ctypes.c_int64(0)
    rc = lib.adaptra_oracle_timeline(S, M, _p(t_f, ctypes.c_int32), _p(t_b, ctypes.c_int32),
                                     _p(w, ctypes.c_int32), _p(cf, ctypes.c_int32), _p(cb, ctypes.c_int32),
                                     _p(a["start_f"], ctypes.c_int64), _p(a["fin_f"], ctypes.c_int64),
                                     _p(a["start_b"], ctypes.c_int64), _p(a["fin_b"], ctypes.c_int64),
                                     _p(idle, ctypes.c_int64), _p(peak, ctypes.c_int32), ctypes.byref(mk))
    if rc < 0:
        raise ValueError(f"oracle rejected the inputs (code {rc})")
    a.update(idle=idle, peak=peak, makespan=int(mk.value), completed=bool(rc))
    return a


# ---------------------------------------------------------------------------------------
# ZeroBubble-style schedules with F / B / W ops (zb_oracle.c)
OP_NAMES = "FBW"


def zb_simulate(S: int, N: int, t_f, t_b, t_w, cf, cb, *, x=None, order=None) -> dict:
    """One pair.  With x (warm-up quotas, [S]) the schedule is generated by the two-phase
    selection policy under the given delays; with order ([S, 3N], ops as type * N + m) that
    fixed order is executed under the delays.  Returns makespan (None on deadlock), the
    order run, start / fin [S, 3, N] and idle [S]."""
    lib = _load()
    t_f, t_b, t_w = _c32(t_f), _c32(t_b), _c32(t_w)
    cf = _c32(cf if S > 1 else np.zeros(0))
    cb = _c32(cb if S > 1 else np.zeros(0))
    mode = 0 if order is None else 1
    xs = _c32(x) if x is not None else None
    od = _c32(order) if order is not None else None
    out_order = np.empty((S, 3 * N), dtype=np.int32)
    start = np.empty((S, 3, N), dtype=np.int64)
    fin = np.empty((S, 3, N), dtype=np.int64)
    idle = np.empty(S, dtype=np.int64)
    mk = lib.adaptra_oracle_zb(S, N, mode, _p(t_f, ctypes.c_int32), _p(t_b, ctypes.c_int32), _p(t_w, ctypes.c_int32),
                               _p(xs, ctypes.c_int32), _p(od, ctypes.c_int32), _p(cf, ctypes.c_int32),
                               _p(cb, ctypes.c_int32), _p(out_order, ctypes.c_int32), _p(start, ctypes.c_int64),
                               _p(fin, ctypes.c_int64), _p(idle, ctypes.c_int64))
    if mk == -2:
        raise ValueError("zb oracle rejected the inputs")
    return {"makespan": None if mk < 0 else int(mk), "order": out_order, "start": start, "fin": fin, "idle": idle}


def zb_batch(S: int, N: int, t_f, t_b, t_w, x, c_fwd, c_bwd, want_idle: bool = True) -> dict:
    """Policy-generated schedules for every (candidate, scenario) pair: x [S, C], c [S-1, K];
    makespan [K, C] (INT32_MAX on deadlock), idle [S, K, C]."""
    lib = _load()
    t_f, t_b, t_w, x, c_fwd, c_bwd = _c32(t_f), _c32(t_b), _c32(t_w), _c32(x), _c32(c_fwd), _c32(c_bwd)
    C, K = int(x.shape[1]), int(c_fwd.shape[1])
    mk = np.empty((K, C), dtype=np.int32)
    idle = np.empty((S, K, C), dtype=np.int32) if want_idle else None
    rc = lib.adaptra_oracle_zb_batch(S, N, _p(t_f, ctypes.c_int32), _p(t_b, ctypes.c_int32), _p(t_w, ctypes.c_int32),
                                     C, _p(x, ctypes.c_int32), K, _p(c_fwd, ctypes.c_int32), _p(c_bwd, ctypes.c_int32),
                                     _p(mk, ctypes.c_int32), _p(idle, ctypes.c_int32))
    if rc != 0:
        raise ValueError("zb oracle rejected the inputs")
    return {"makespan": mk, "idle": idle}
