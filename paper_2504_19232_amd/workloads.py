"""Seeded synthetic inputs for the batched pipeline-schedule evaluation.

This module only draws numbers and lays them out; it contains none of the
schedule model's arithmetic (no recurrence, no feasibility test, no makespan).
Both the GPU path's tests/benchmark and the CPU oracle's tests read their
inputs from here so that they see the same bytes.

The paper measures on GPT-2 training runs (4-8 pipeline stages in its
micro-benchmarks, Table 2; backward about twice the forward; 1-3 concurrent
slow links with delays of tens of milliseconds, Section 7 and the injection
trace in the Appendix).  None of that data is available, so the five
configurations below stand in for it with the same structure.

Notation: S stages, M micro-batches, w[s] = number of warm-up forwards of
stage s counted so that the last stage of plain 1F1B has w = 0 (the paper's
x_s equals w[s] + 1), c_fwd[l] / c_bwd[l] = delay of link l <-> l+1 in the
forward / backward direction.  All times are int32 microseconds.

Layouts (structure of arrays, candidate / scenario index fastest):
    w      int32 [S,   C]
    c_fwd  int32 [S-1, K]
    c_bwd  int32 [S-1, K]
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

BASE_SEED = 250419232
BASE_LINK_DELAY = 10  # microseconds on every link that is not a straggler


@dataclass
class Workload:
    name: str
    S: int
    M: int
    t_f: np.ndarray            # int32 [S]
    t_b: np.ndarray            # int32 [S]
    mem_cap: Optional[np.ndarray]  # int32 [S] or None (no cap)
    w: np.ndarray              # int32 [S, C]
    c_fwd: np.ndarray          # int32 [S-1, K]
    c_bwd: np.ndarray          # int32 [S-1, K]
    hist_bins: int = 0
    hist_shift: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def n_cand(self) -> int:
        return int(self.w.shape[1])

    @property
    def n_scen(self) -> int:
        return int(self.c_fwd.shape[1])

    @property
    def n_pairs(self) -> int:
        return self.n_cand * self.n_scen

    def sha256(self) -> str:
        h = hashlib.sha256()
        h.update(np.array([self.S, self.M, self.hist_bins, self.hist_shift], dtype="<i4").tobytes())
        for a in (self.t_f, self.t_b, self.mem_cap, self.w, self.c_fwd, self.c_bwd):
            if a is None:
                h.update(b"none")
            else:
                h.update(np.ascontiguousarray(a, dtype="<i4").tobytes())
        return h.hexdigest()


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _log_uniform(rng: np.random.Generator, lo: float, hi: float, size) -> np.ndarray:
    u = rng.random(size)
    return np.floor(lo * (hi / lo) ** u).astype(np.int64)


def default_warmup(S: int) -> np.ndarray:
    """Plain 1F1B warm-up counts: w[s] = S - s - 1."""
    return np.arange(S - 1, -1, -1, dtype=np.int64)


def enumerate_offsets(S: int, n_off: int) -> np.ndarray:
    """Every offset vector d in {0..n_off-1}^(S-1); candidate index c = sum_s d[s] * n_off**s.

    Returns w = default + d as int32 [S, n_off**(S-1)]; the last stage keeps w = 0.
    """
    C = n_off ** (S - 1)
    c = np.arange(C, dtype=np.int64)
    w = np.zeros((S, C), dtype=np.int64)
    base = default_warmup(S)
    for s in range(S - 1):
        w[s] = base[s] + (c // (n_off ** s)) % n_off
    w[S - 1] = base[S - 1]
    return _i32(w)


def sample_offsets(rng: np.random.Generator, S: int, C: int, d_max: int, repair_mod: int = 8) -> np.ndarray:
    """C sampled offset vectors, d[s] uniform in {0..d_max} for the S-1 non-last stages.

    Independent sampling leaves almost no vector with non-increasing warm-up
    counts once S is large, so every candidate whose index is not a multiple
    of ``repair_mod`` is made non-increasing by a suffix maximum
    (w[s] <- max(w[s], w[s+1]) from the last stage backwards); the others stay
    raw so that invalid vectors are still present.
    """
    d = rng.integers(0, d_max + 1, size=(S - 1, C), dtype=np.int64)
    w = np.zeros((S, C), dtype=np.int64)
    w[: S - 1] = default_warmup(S)[: S - 1, None] + d
    fix = (np.arange(C) % repair_mod) != 0
    for s in range(S - 2, -1, -1):
        w[s] = np.where(fix, np.maximum(w[s], w[s + 1]), w[s])
    return _i32(w)


def _single_link_scenarios(S: int, link: np.ndarray, delay: np.ndarray):
    K = len(delay)
    cf = np.full((S - 1, K), BASE_LINK_DELAY, dtype=np.int64)
    cf[link, np.arange(K)] = delay
    return _i32(cf), _i32(cf.copy())


def _directed_link_scenarios(rng, S: int, K: int, n_lo: int, n_hi: int, lo: float, hi: float):
    """Each scenario slows n in [n_lo, n_hi] distinct directed links (forward
    and backward directions are separate links), delays log-uniform in [lo, hi]."""
    L = 2 * (S - 1)
    c = np.full((L, K), BASE_LINK_DELAY, dtype=np.int64)
    n = rng.integers(n_lo, n_hi + 1, size=K)
    for k in range(K):
        links = rng.permutation(L)[: n[k]]
        c[links, k] = _log_uniform(rng, lo, hi, n[k])
    return _i32(c[: S - 1]), _i32(c[S - 1:])


def config(index: int) -> Workload:
    """The five benchmark configurations (index 0..4); draw order: times, caps,
    candidates, scenarios."""
    rng = _rng(BASE_SEED + index)
    if index == 0:
        S, M = 4, 8
        t_f = np.rint(100 * rng.uniform(0.9, 1.1, S))
        t_b = np.rint(200 * rng.uniform(0.9, 1.1, S))
        w = enumerate_offsets(S, 4)
        link = int(rng.integers(0, S - 1))
        delay = np.arange(0, 1001, 50, dtype=np.int64)
        cf, cb = _single_link_scenarios(S, np.full(len(delay), link), delay)
        return Workload("cfg0_S4_M8", S, M, _i32(t_f), _i32(t_b), None, w, cf, cb,
                        notes={"straggler_link": link})
    if index == 1:
        S, M = 8, 32
        t_f = rng.integers(80, 121, S)
        t_b = np.rint(2 * t_f * rng.uniform(0.95, 1.05, S))
        cap = np.full(S, 8)
        w = enumerate_offsets(S, 4)
        K = 64
        link = rng.integers(0, S - 1, K)
        delay = _log_uniform(rng, 10, 5000, K)
        cf, cb = _single_link_scenarios(S, link, delay)
        return Workload("cfg1_S8_M32", S, M, _i32(t_f), _i32(t_b), _i32(cap), w, cf, cb)
    if index == 2:
        S, M = 16, 64
        t_f = rng.integers(150, 251, S).astype(np.int64)
        t_b = 2 * t_f
        for s in (0, S - 1):
            t_f[s] = (t_f[s] * 3) // 2
            t_b[s] = (t_b[s] * 3) // 2
        cap = np.full(S, 24)
        w = sample_offsets(rng, S, 1 << 18, 4)
        cf, cb = _directed_link_scenarios(rng, S, 256, 1, 3, 10, 20000)
        return Workload("cfg2_S16_M64", S, M, _i32(t_f), _i32(t_b), _i32(cap), w, cf, cb)
    if index == 3:
        S, M = 32, 128
        t_f = np.rint(np.exp(rng.normal(np.log(200.0), 0.2, S))).astype(np.int64)
        t_b = 2 * t_f + np.rint(np.exp(rng.normal(np.log(20.0), 0.5, S))).astype(np.int64)
        cap = rng.integers(16, 65, S)
        # the 1F1B default (S - s in flight) plus two extra warm-up forwards always
        # fits; a floor of S - s alone leaves no sampled candidate inside the caps
        cap = np.maximum(cap, S - np.arange(S) + 2)
        w = sample_offsets(rng, S, 1 << 16, 4)
        cf, cb = _directed_link_scenarios(rng, S, 1024, 6, 6, 50, 50000)
        return Workload("cfg3_S32_M128", S, M, _i32(t_f), _i32(t_b), _i32(cap), w, cf, cb)
    if index == 4:
        S, M = 8, 256
        t_f = rng.integers(50, 151, S).astype(np.int64)
        t_b = 2 * t_f
        w = sample_offsets(rng, S, 1 << 20, 7)
        K = 64
        link = int(rng.integers(0, S - 1))
        delay = np.rint(np.arange(K) * 10000.0 / (K - 1)).astype(np.int64)
        cf, cb = _single_link_scenarios(S, np.full(K, link), delay)
        return Workload("cfg4_S8_M256", S, M, _i32(t_f), _i32(t_b), None, w, cf, cb,
                        hist_bins=64, hist_shift=17, notes={"straggler_link": link})
    raise ValueError(f"config index {index} out of range 0..4")


def random_workload(seed: int, S: int, M: int, C: int, K: int, *, t_lo: int = 20, t_hi: int = 300,
                    d_max: int = 3, c_hi: int = 4000, cap: bool = True, raw_every: int = 4,
                    w_extra: int = 0, hist_bins: int = 0, hist_shift: int = 0) -> Workload:
    """An arbitrary-shape workload for tests: ragged C and K, mixed valid and
    invalid warm-up vectors, some out-of-range w (negative, above M), optional caps.

    ``w_extra`` shifts every non-last stage's warm-up count up (deep warm-up)."""
    rng = _rng(seed)
    t_f = rng.integers(t_lo, t_hi + 1, S)
    t_b = rng.integers(t_lo, 2 * t_hi + 1, S)
    mem_cap = rng.integers(max(1, S // 2), 2 * S + d_max + w_extra + 2, S) if cap else None
    if S > 1:
        w = sample_offsets(rng, S, C, d_max, repair_mod=raw_every).astype(np.int64)
        w[: S - 1] += w_extra
    else:
        w = rng.integers(0, d_max + 1, size=(1, C)).astype(np.int64)
    if C >= 8:
        # a few out-of-range entries: the model clamps them into [0, M-1]
        idx = rng.integers(0, C, size=max(1, C // 16))
        w[0, idx] += M + rng.integers(0, 5, size=len(idx))
        idx = rng.integers(0, C, size=max(1, C // 16))
        w[S - 1, idx] -= rng.integers(0, 3, size=len(idx))
    L = max(S - 1, 0)
    if L:
        cf = rng.integers(0, 40, size=(L, K)).astype(np.int64)
        cb = rng.integers(0, 40, size=(L, K)).astype(np.int64)
        slow = rng.random((2 * L, K)) < 0.25
        big = _log_uniform(rng, 10, max(11, c_hi), (2 * L, K))
        cf = np.where(slow[:L], big[:L], cf)
        cb = np.where(slow[L:], big[L:], cb)
    else:
        cf = np.zeros((0, K), dtype=np.int64)
        cb = np.zeros((0, K), dtype=np.int64)
    return Workload(f"rand_s{seed}_S{S}_M{M}_C{C}_K{K}", S, M, _i32(t_f), _i32(t_b),
                    None if mem_cap is None else _i32(mem_cap), _i32(w), _i32(cf), _i32(cb),
                    hist_bins=hist_bins, hist_shift=hist_shift)


def near_bound_workload(seed: int, S: int, M: int, C: int, K: int, frac: float = 0.99, **kw) -> Workload:
    """A random_workload whose times and delays are rescaled so that the precondition of the
    int32 path, 2 M S (max time + max delay) < 2^31, holds with only (1 - frac) to spare: the
    largest time is planted at 60 % and the largest delay at 40 % of frac * 2^31 / (2 M S), the
    other entries spread below them.  Input generation only."""
    wl = random_workload(seed, S, M, C, K, **kw)
    rng = _rng(seed + 7919)
    budget = int(frac * 2 ** 31 / (2 * M * S))
    t_max, c_max = (budget * 6) // 10, budget - (budget * 6) // 10
    wl.t_f = _i32(rng.integers(t_max // 8, t_max + 1, S))
    wl.t_b = _i32(rng.integers(t_max // 8, t_max + 1, S))
    wl.t_b[int(rng.integers(0, S))] = t_max
    if S > 1:
        slow = rng.random((2 * (S - 1), K)) < 0.3
        c = np.where(slow, rng.integers(c_max // 2, c_max + 1, slow.shape), rng.integers(0, max(1, c_max // 64), slow.shape))
        c[int(rng.integers(0, 2 * (S - 1))), int(rng.integers(0, K))] = c_max
        wl.c_fwd, wl.c_bwd = _i32(c[: S - 1]), _i32(c[S - 1:])
    wl.name = f"nearbound_s{seed}_S{S}_M{M}_C{C}_K{K}"
    return wl


def sample_pairs(seed: int, n_cand: int, n_scen: int, n: int):
    """n seeded (candidate, scenario) index pairs, for sampled parity at sizes
    the oracle cannot sweep."""
    rng = _rng(seed)
    return (rng.integers(0, n_cand, n, dtype=np.int64), rng.integers(0, n_scen, n, dtype=np.int64))


def straggler_stage_times(seed: int, wl: Workload, p_slow: float = 0.15, slow_lo: float = 1.1,
                          slow_hi: float = 4.0):
    """Per-scenario stage times [S, K] for computation stragglers (Section 2.2): in every
    scenario each stage is slowed with probability p_slow by a log-uniform factor in
    [slow_lo, slow_hi] (forward and backward alike), else runs at the workload's t_f / t_b.
    Input generation only."""
    rng = _rng(seed)
    S, K = wl.S, wl.n_scen
    slow = rng.random((S, K)) < p_slow
    factor = np.where(slow, slow_lo * (slow_hi / slow_lo) ** rng.random((S, K)), 1.0)
    t_f = np.rint(wl.t_f[:, None] * factor)
    t_b = np.rint(wl.t_b[:, None] * factor)
    return _i32(t_f), _i32(t_b)
