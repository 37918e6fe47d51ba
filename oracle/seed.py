"""The paper's analytic warm-up planning, written out step by step -- TEST INFRASTRUCTURE.

Plain Python integers, one function per algorithm, in the paper's notation
(x_i = warm-up forward count of stage i, Delta_i = x_i - x_{i+1}).  Results are
returned both as x and as w = x - 1 (the library's convention: last stage of
plain 1F1B at w = 0).  Only tests, smoke() and bench.py's cpu_baseline leg may
import this module.  Pinned by tests/test_oracle_seed_pins.py.
"""
from __future__ import annotations


def get_init_warmup_fwds(S: int, x_max: int):
    """Algorithm 1 (initial planning): the first stage holds x_max forwards, the slack
    x_max - 1 is spread over the S - 1 links as evenly as possible, the first
    (x_max - 1) mod (S - 1) links getting one more.  x_max = floor(M / M^F) is passed in."""
    if S < 1 or x_max < 1:
        raise ValueError("S >= 1 and x_max >= 1 required")
    x = [x_max]
    if S == 1:
        return x
    d_avg = (x_max - 1) // (S - 1)
    r = (x_max - 1) % (S - 1)
    for i in range(1, S):
        d = d_avg + 1 if i <= r else d_avg
        x.append(x[i - 1] - d)
    return x


def get_adapted_warmup_fwds(S: int, N: int, t_f, t_b, c_fwd, c_bwd):
    """Algorithm 2 (dynamic adaptation): x_{S-1} = 1 and, from the last link backwards,
    Delta_i = min(N - 2S, max(ceil((t^F_i + t^B_i + 2 c_i) / (t^F_{i+1} + t^B_{i+1})), 2)),
    x_i = x_{i+1} + Delta_i.

    Readings (the paper is silent): the two directions of a link may differ, so 2 c_i is
    c_fwd[i] + c_bwd[i]; a zero denominator makes the ratio infinite (the clip decides);
    the clip N - 2S can be below 0, so Delta_i is floored at 0 (Lemma 1) and x_i is capped
    at N (a stage cannot warm up more forwards than there are micro-batches)."""
    x = [0] * S
    x[S - 1] = 1
    for i in range(S - 2, -1, -1):
        num = int(t_f[i]) + int(t_b[i]) + int(c_fwd[i]) + int(c_bwd[i])
        den = int(t_f[i + 1]) + int(t_b[i + 1])
        clip = N - 2 * S
        if den == 0:
            d = clip
        else:
            d = min(clip, max(-(-num // den), 2))
        d = max(d, 0)
        x[i] = min(x[i + 1] + d, N)
    return x


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
