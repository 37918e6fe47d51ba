"""Guided search over warm-up vectors -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

For pipelines whose schedule space cannot be enumerated (5^31 vectors at 32 stages) the
exhaustive per-scenario argmin is replaced by a neighbourhood descent driven by batched
evaluation of the paper's analytical model (Section 3.1; the coordinates are the slacks
Delta_i = w_i - w_{i+1} that Section 4.2's algorithms plan with).  This file states the
procedure step by step on top of the oracle's simulator; it shares nothing with the GPU path.

Procedure.  Every scenario k descends on its own: it keeps a current point w^k (all start
from the same vector) and its makespan (INT32_MAX before the first round).  One round:
  1. scenario k's pool: its point, then the point's neighbours in move order, every entry
     clamped into [0, M-1];
  2. every pool entry is evaluated under scenario k; the scenario's best is the feasible
     entry of smallest makespan, ties to the lowest pool index;
  3. the scenario moves to its best entry iff that is strictly better than what it has.
The search stops after the first round in which no scenario moved, or after max_iters rounds
(a scenario that has stopped moving keeps being evaluated until all have: its result does
not change).

Moves.  neighbourhood 0: for l = 0..S-1, subtract then add 1 on stages 0..l (slack Delta_l
one down / up, everything upstream shifted along).  neighbourhood 1: for a = 0..S-1, for
b = a..S-1, subtract then add 1 on stages a..b (moves one unit of slack from one link to
another; contains neighbourhood 0 and the single-stage moves).

Parity status: pinned by tests/test_oracle_search_pins.py (a hand-worked descent, local
optimality by direct enumeration, bounds against the exhaustive optimum)."""
import numpy as np

from . import oracle

INT32_MAX = 2 ** 31 - 1


def moves(S: int, neighbourhood: int):
    """List of (a, b, sign): add sign to stages a..b inclusive."""
    out = []
    if neighbourhood == 0:
        for l in range(S):
            out += [(0, l, -1), (0, l, +1)]
    elif neighbourhood == 1:
        for a in range(S):
            for b in range(a, S):
                out += [(a, b, -1), (a, b, +1)]
    else:
        raise ValueError("neighbourhood must be 0 or 1")
    return out


def search(S: int, M: int, t_f, t_b, mem_cap, w_start, c_fwd, c_bwd, *, neighbourhood: int = 0,
           max_iters: int = 1000, t_f_scen=None, t_b_scen=None) -> dict:
    c_fwd = np.asarray(c_fwd)
    K = c_fwd.shape[1] if S > 1 else np.asarray(c_bwd).shape[1]
    mv = moves(S, neighbourhood)
    cur = np.repeat(np.clip(np.asarray(w_start, dtype=np.int64), 0, M - 1)[:, None], K, axis=1)
    cur_mk = np.full(K, INT32_MAX, dtype=np.int64)
    rounds = 0
    evaluated = 0
    history = []                                        # every scenario's makespan after each round
    per_point = len(mv) + 1
    while rounds < max_iters:
        rounds += 1
        pool = []                                       # step 1
        for k in range(K):
            p = cur[:, k]
            pool.append(p.copy())
            for a, b, sign in mv:
                q = p.copy()
                q[a:b + 1] += sign
                pool.append(np.clip(q, 0, M - 1))
        pool = np.stack(pool, axis=1)
        n = pool.shape[1]
        owner = np.arange(n) // per_point
        if t_f_scen is None:                            # step 2
            r = oracle.eval_pairs(S, M, t_f, t_b, mem_cap, pool, c_fwd, c_bwd, pair_cand=np.arange(n),
                                  pair_scen=owner, want_bubble=False)
            mk, fl = r["makespan"], r["flag"]
        else:
            mk = np.empty(n, dtype=np.int64)
            fl = np.empty(n, dtype=np.uint8)
            for k in range(K):
                sl = slice(k * per_point, (k + 1) * per_point)
                r = oracle.eval_pairs(S, M, np.asarray(t_f_scen)[:, k], np.asarray(t_b_scen)[:, k], mem_cap,
                                      pool[:, sl], c_fwd[:, k:k + 1], np.asarray(c_bwd)[:, k:k + 1],
                                      want_bubble=False)
                mk[sl], fl[sl] = r["makespan"][0], r["flag"][0]
        evaluated += n
        moved = 0                                       # step 3
        for k in range(K):
            sl = slice(k * per_point, (k + 1) * per_point)
            best = oracle.best_from_eval(mk[sl][None, :], fl[sl][None, :])
            j = int(best["best_idx"][0])
            if j >= 0 and best["best_makespan"][0] < cur_mk[k]:
                cur[:, k] = pool[:, k * per_point + j]
                cur_mk[k] = best["best_makespan"][0]
                moved += 1
        history.append(cur_mk.copy())
        if moved == 0:
            break
    return {"w": cur.astype(np.int32), "makespan": cur_mk.astype(np.int32), "rounds": rounds,
            "evaluated": evaluated, "makespan_history": np.stack(history).astype(np.int32)}
