"""The paper's analytic warm-up planning, written from its definitions -- TEST INFRASTRUCTURE.

Plain Python integers, one function per algorithm, in the paper's notation
(x_i = warm-up forward count of stage i, Delta_i = x_i - x_{i+1}).  Results are
returned both as x and as w = x - 1 (the library's convention: last stage of
plain 1F1B at w = 0).  Only tests, smoke() and bench.py's cpu_baseline leg may
import this module.  Pinned by tests/test_oracle_seed_pins.py.
"""
from __future__ import annotations


def initial_plan(S: int, x_max: int):
    """Algorithm 1 (initial planning), from what it is defined to achieve: stage 0 holds x_max
    warm-up forwards (the memory limit, x_max = floor(M / M^F), passed in), the last stage 1, and
    the x_max - 1 units of slack in between are shared out over the S - 1 links as evenly as
    integers allow, the links nearest stage 0 taking the units left over.  x_i is x_max minus
    the slack of the links above stage i."""
    if S < 1 or x_max < 1:
        raise ValueError("S >= 1 and x_max >= 1 required")
    if S == 1:
        return [x_max]
    share, left_over = divmod(x_max - 1, S - 1)
    slack = [share + 1] * left_over + [share] * (S - 1 - left_over)          # link 0 first
    return [x_max - sum(slack[:i]) for i in range(S)]


def link_slack(N: int, S: int, tau_i: int, tau_next: int, c_fwd_i: int, c_bwd_i: int) -> int:
    """The slack Algorithm 2 gives link i: the smallest Delta >= 2 for which Eq. (1) holds,
    tau_i + 2 c_i <= Delta tau_{i+1}, clipped at N - 2 S.

    Readings (the paper is silent): the two directions of a link may differ, so 2 c_i is
    c_fwd[i] + c_bwd[i]; a zero denominator makes the ratio infinite (the clip decides);
    the clip N - 2S can be below 0, so the slack is floored at 0 (Lemma 1)."""
    clip = N - 2 * S
    if tau_next == 0:
        want = clip
    else:
        load = tau_i + c_fwd_i + c_bwd_i
        want = min(clip, max(-(-load // tau_next), 2))            # ceiling division
    return max(want, 0)


def adapted_plan(S: int, N: int, t_f, t_b, c_fwd, c_bwd):
    """Algorithm 2 (dynamic adaptation): the last stage holds one warm-up forward and every
    stage above it as many more as the slacks of the links below it add up to, x_i = 1 +
    sum of Delta_j for j >= i, capped at N (a stage cannot warm up more forwards than there
    are micro-batches; the slacks are not negative, so capping the sums equals capping every
    step of the listing's recurrence x_i = x_{i+1} + Delta_i)."""
    tau = [int(t_f[i]) + int(t_b[i]) for i in range(S)]
    slack = [link_slack(N, S, tau[i], tau[i + 1], int(c_fwd[i]), int(c_bwd[i])) for i in range(S - 1)]
    return [min(N, 1 + sum(slack[i:])) for i in range(S)]


def absorbed(S: int, t_f, t_b, w, c_fwd, c_bwd):
    """Eq. (1) per link for the schedule w: the delay of link i causes no cascading bubbles
    iff t^F_i + t^B_i + 2 c_i <= Delta_i (t^F_{i+1} + t^B_{i+1}), Delta_i = w_i - w_{i+1}
    (2 c_i read as c_fwd[i] + c_bwd[i])."""
    out = []
    for i in range(S - 1):
        lhs = int(t_f[i]) + int(t_b[i]) + int(c_fwd[i]) + int(c_bwd[i])
        rhs = (int(w[i]) - int(w[i + 1])) * (int(t_f[i + 1]) + int(t_b[i + 1]))
        out.append(lhs <= rhs)
    return out


def to_w(x):
    return [v - 1 for v in x]
