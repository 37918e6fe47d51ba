"""The two arguments the fixed-plan kernels of the ZeroBubble row rest on, checked on the CPU
against the oracle (Section 3.1 dependencies; Section 4.3 / Algorithm 3 policy; Algorithm 4):

  * the stages of a pipeline may take their next actions TOGETHER whenever those lie before
    t + L (t = the earliest next action, L = the least duration + link delay of any op that posts
    a ready time): the schedule is the one the policy produces one decision at a time;
  * a fixed plan's times do not need its weight ops one by one: a weight op starts the moment its
    stage is free, so adding the time a stage spent on them to its busy-until time before its
    next forward or backward op gives the same times.

Both procedures are restated here in plain Python (they are what k_zb_record_stages and
k_zb_replay_folded do on the GPU) and compared with oracle.zb_simulate op by op."""
import numpy as np
import pytest

from oracle import oracle

NEVER = 1 << 62


def _problem(seed):
    rng = np.random.default_rng(seed)
    S, N = int(rng.integers(1, 7)), int(rng.integers(1, 10))
    small = seed % 3 == 0                     # durations of 1..3 and delays of 0..2: many equal instants
    t_f = rng.integers(1, 4 if small else 60, S)
    t_b = rng.integers(1, 4 if small else 90, S)
    t_w = rng.integers(0, 3 if small else 50, S)
    cf = rng.integers(0, 3 if small else 300, max(S - 1, 0))
    cb = rng.integers(0, 3 if small else 300, max(S - 1, 0))
    x = np.sort(rng.integers(1, N + 1, S))[::-1].copy()
    if seed % 4 == 0:
        x = rng.integers(1, N + 1, S)         # quotas that are not monotone
    return S, N, t_f, t_b, t_w, cf, cb, x


def _together(S, N, t_f, t_b, t_w, cf, cb, x, widen=0):
    """Start times [S][3][N] under the policy with the stages advancing together."""
    posts_f = [i < S - 1 for i in range(S)]
    posts_b = [i > 0 for i in range(S)]
    look = min([t_f[i] + cf[i] for i in range(S) if posts_f[i]] + [t_b[i] + cb[i - 1] for i in range(S) if posts_b[i]] + [1 << 30])
    look += widen
    done = [[0, 0, 0] for _ in range(S)]
    ready = [[[], []] for _ in range(S)]      # ready times posted to a stage, per type, in micro-batch order
    busy = [0] * S
    start = np.full((S, 3, N), -1, dtype=np.int64)

    def heads(i):
        nF, nB, nW = done[i]
        hF = (0 if i == 0 else ready[i][0][nF]) if nF < (N if i == 0 else len(ready[i][0])) else NEVER
        if i == S - 1:
            hB = 0 if nB < nF else NEVER
        else:
            hB = ready[i][1][nB] if nB < len(ready[i][1]) else NEVER
        return hF, hB, (0 if nW < nB else NEVER)

    def key(i):
        hF, hB, hW = heads(i)
        soonest = hF if done[i][0] < x[i] else min(hF, hB, hW)
        return NEVER if soonest == NEVER else max(busy[i], soonest)

    left = 3 * S * N
    while left:
        keys = [key(i) for i in range(S)]
        t = min(keys)
        if t == NEVER:
            return None
        posted = []
        for i in range(S):
            if keys[i] == NEVER or keys[i] - t >= look:
                continue
            hF, hB, _ = heads(i)
            ty = 0 if done[i][0] < x[i] else (1 if hB <= keys[i] else (0 if hF <= keys[i] else 2))
            m = done[i][ty]
            start[i, ty, m] = keys[i]
            fin = keys[i] + (t_f[i], t_b[i], t_w[i])[ty]
            busy[i] = fin
            done[i][ty] += 1
            left -= 1
            if ty == 0 and posts_f[i]:
                posted.append((i + 1, 0, fin + cf[i]))
            if ty == 1 and posts_b[i]:
                posted.append((i - 1, 1, fin + cb[i - 1]))
        for j, ty, r in posted:
            ready[j][ty].append(r)
    return start


@pytest.mark.parametrize("seed", range(60))
def test_stages_advancing_together_reproduce_the_policy(seed):
    S, N, t_f, t_b, t_w, cf, cb, x = _problem(seed)
    ref = oracle.zb_simulate(S, N, t_f, t_b, t_w, cf, cb, x=x)
    got = _together(S, N, t_f, t_b, t_w, cf, cb, x)
    assert ref["makespan"] is not None and got is not None
    assert np.array_equal(got, ref["start"])


def test_a_wider_window_than_the_look_ahead_is_caught():
    """The comparison above does see a window that is too wide: decisions taken before everything
    that may precede them has been posted differ from the policy's somewhere."""
    differs = 0
    for seed in range(60):
        S, N, t_f, t_b, t_w, cf, cb, x = _problem(seed)
        ref = oracle.zb_simulate(S, N, t_f, t_b, t_w, cf, cb, x=x)
        got = _together(S, N, t_f, t_b, t_w, cf, cb, x, widen=int(max(t_b.max(), t_f.max())))
        differs += got is None or not np.array_equal(got, ref["start"])
    assert differs > 0


@pytest.mark.parametrize("seed", range(40))
def test_weight_ops_folded_into_the_op_that_follows(seed):
    S, N, t_f, t_b, t_w, cf, cb, x = _problem(seed)
    gen = oracle.zb_simulate(S, N, t_f, t_b, t_w, cf, cb, x=x)
    order = gen["order"]                      # [S][3N], ops as type * N + m, in each stage's own order
    rng = np.random.default_rng(1000 + seed)
    cf2 = rng.integers(0, 300, max(S - 1, 0))
    cb2 = rng.integers(0, 300, max(S - 1, 0))
    ref = oracle.zb_simulate(S, N, t_f, t_b, t_w, cf2, cb2, order=order)
    # a topological order of the forward and backward ops: by their start times under the
    # delays the plan was generated with (an op starts after everything it depends on has started)
    ops = []
    for i in range(S):
        weight_time = 0
        for op in order[i]:
            ty, m = divmod(int(op), N)
            if ty == 2:
                weight_time += int(t_w[i])
            else:
                ops.append((int(gen["start"][i, ty, m]), i, ty, m, weight_time))
                weight_time = 0
    tail = [0] * S
    for i in range(S):
        for op in order[i][::-1]:
            if int(op) // N != 2:
                break
            tail[i] += int(t_w[i])
    ops.sort()
    busy = [0] * S
    ready = [0] * N
    for _, i, ty, m, weight_time in ops:
        fin = max(busy[i] + weight_time, ready[m]) + int((t_f, t_b)[ty][i])
        assert fin == ref["fin"][i, ty, m]
        busy[i] = fin
        ready[m] = fin + (int(cf2[i]) if ty == 0 and i < S - 1 else (int(cb2[i - 1]) if ty == 1 and i > 0 else 0))
    assert max(busy[i] + tail[i] for i in range(S)) == ref["makespan"]
