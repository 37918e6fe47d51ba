#!/usr/bin/env python3
"""Benchmark of the batched pipeline-schedule evaluation on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: adaptra_eval_best -- feasibility pre-pass, max-plus recurrence for every
pair, makespan + per-stage bubbles + flag byte, per-scenario argmin over the feasible
candidates, winner's bubbles, histogram if the configuration asks for one.  Every pair is
resolved once; `--two-calls` times adaptra_eval followed by adaptra_best instead (the same
outputs, the feasible pairs resolved a second time by the search).  `value` counts each
(candidate, scenario) pair once per step.

Prints ONE JSON line (see the fields below).  `roofline` prices the dominant kernel (the
recurrence kernel of adaptra_eval) against the integer-VALU peak, with the kernel's duration
measured by HIP events the library records on its own stream:
  frac              3 int32 operations per resolved op (add the link delay, max with the stage
                    frontier, add the duration) against 256 CUs x 64 lanes x 2.4 GHz.  Not bounded
                    by 1: the kernel's formulation needs 2 operations, and adds issue at twice
                    the rate of the peak's one instruction per SIMD per four cycles.
  frac_formulation  the least time the kernel's own formulation could take on this chip -- per
                    resolved op one add on vector operands (two cycles of a SIMD per wavefront,
                    the measured double rate) and one max (four cycles) -- over the time it
                    takes.  At most 1 by construction.
  valu_busy_min/max share of the SIMDs' cycles in which the vector ALU is occupied by this kernel,
                    from the instruction count of the committed rocprofv3 summary: max prices
                    every instruction at four cycles, min prices one add per resolved op at two
                    (the adds on vector operands, if each of them got the double rate).  null
                    when the summary was measured on other sources than the ones in the tree.
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same pairs.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT32_VALU_PEAK = 256 * 64 * 2.4e9          # CUs x lanes/clk x clock = 39.32e12 int32 lane-ops/s


class HipEvents:
    """Raw hipEvent_t handles (the library records them; torch events cannot be handed over)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed ({rc})")
        return ev

    def elapsed_ms(self, a, b) -> float:
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)

    def destroy(self, ev):
        self.hip.hipEventDestroy(ev)


def kernel_source_sha256() -> str:
    """Hash of the library's sources (csrc/ and include/): rocprofv3 summaries under profiles/
    carry the hash of the sources they were measured on, so that figures taken from them can be
    dropped when the kernels have changed since."""
    import hashlib
    h = hashlib.sha256()
    for folder in (os.path.join(ROOT, "paper_2504_19232_amd", "csrc"), os.path.join(ROOT, "include")):
        for name in sorted(os.listdir(folder)):
            if name.endswith((".hip", ".h")):
                h.update(name.encode())
                h.update(open(os.path.join(folder, name), "rb").read())
    return h.hexdigest()


def from_profile(S: int, config: int) -> dict:
    """Figures that cannot be measured from inside this process, read from the committed
    rocprofv3 summary of the resolve kernel on this workload: HBM bytes per launch (FETCH_SIZE
    and WRITE_SIZE, scaled by a copy of known size) and the vector instructions the kernel
    issues per launch (SQ_INSTS_VALU) with the shader clock cycles that launch took
    (GRBM_GUI_ACTIVE per XCD).  Every value is None when there is no summary or when the summary was measured on
    other sources than the ones in the tree now."""
    out = {"traffic": None, "valu_instructions": None, "cycles": None, "profile_is_current": False}
    path = os.path.join(ROOT, "profiles", f"resolve_scen_lanes_S{S}_config{config}.txt")
    try:
        lines = open(path).read().splitlines()
    except OSError:
        return out
    found = {}
    for line in lines:
        s = line.strip()
        for key in ("source_sha256", "traffic_bytes_per_launch", "valu_instructions_per_launch",
                    "shader_cycles_per_launch"):
            if s.startswith(key) and "=" in s:
                found[key] = s.split("=")[1].strip()
    if found.get("source_sha256") != kernel_source_sha256():
        return out
    out["profile_is_current"] = True
    try:
        out["traffic"] = int(found["traffic_bytes_per_launch"])
        out["valu_instructions"] = float(found["valu_instructions_per_launch"])
        out["cycles"] = float(found["shader_cycles_per_launch"])
    except (KeyError, ValueError):
        pass
    return out


def probe_rates(binding, torch, dev, iters: int = 400) -> dict:
    """Issue rate of every probe mix of the library (vector instructions per second over the
    whole chip), each timed with events on the stream it runs on."""
    scr = torch.zeros(64, dtype=torch.int32, device=dev)
    rates = {}
    for mix, name in enumerate(binding.PROBE_MIXES):
        binding.adaptra_valu_probe(mix, 8192, 20, scr)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        n = binding.adaptra_valu_probe(mix, 8192, iters, scr)
        e1.record()
        torch.cuda.synchronize()
        rates[name] = n / (e0.elapsed_time(e1) * 1e-3)
    return rates


def cpu_baseline(wl, target_seconds: float = 16.0) -> dict:
    """The oracle as it stands, on the host cores, on a seeded sample of this workload's pairs:
    all threads for about `target_seconds`, then one thread on a sixteenth of that sample."""
    from oracle import oracle
    from paper_2504_19232_amd import workloads
    threads = oracle.default_threads()
    pc, ps = workloads.sample_pairs(4242, wl.n_cand, wl.n_scen, 1 << 22)
    n0 = 1 << 14
    t0 = time.perf_counter()
    oracle.eval_workload(wl, pair_cand=pc[:n0], pair_scen=ps[:n0], threads=threads)
    probe = time.perf_counter() - t0
    n = int(min(len(pc), max(n0, n0 * target_seconds / max(probe, 1e-3))))
    t0 = time.perf_counter()
    r = oracle.eval_workload(wl, pair_cand=pc[:n], pair_scen=ps[:n], threads=threads)
    dt = time.perf_counter() - t0
    live = int(((r["flag"] & 2) == 0).sum())
    n1 = max(256, n // (16 * max(threads, 1)))
    t0 = time.perf_counter()
    oracle.eval_workload(wl, pair_cand=pc[:n1], pair_scen=ps[:n1], threads=1)
    dt1 = time.perf_counter() - t0
    return {"value": n / dt, "unit": "evaluations/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} seeded random pairs of the workload ({live} not deadlocked), "
                      f"event-driven simulation incl. bubbles, {dt:.1f} s",
            "resolved_ops_per_s": live * 2.0 * wl.S * wl.M / dt,
            "one_core": {"value": n1 / dt1, "sample_pairs": n1, "seconds": dt1}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload index 0..4 (default 3: S=32, M=128, 2^26 pairs)")
    ap.add_argument("--no-bubble", action="store_true", help="skip adaptra_eval's [S][K][C] bubble output")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--two-calls", action="store_true",
                    help="step = adaptra_eval then adaptra_best (feasible pairs resolved twice) instead of "
                         "adaptra_eval_best")
    ap.add_argument("--no-zb", action="store_true", help="skip the ZeroBubble (F/B/W) side measurement")
    ap.add_argument("--no-sens", action="store_true",
                    help="skip the per-scenario stage time and link sensitivity side measurements")
    ap.add_argument("--kernel-mode", type=int, default=0)
    ap.add_argument("--probe-only", action="store_true",
                    help="run only the instruction issue-rate probes (for a counter profile of them)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy before the timed region (a kernel of "
                         "known traffic, to scale the FETCH_SIZE / WRITE_SIZE counters in a profile)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); nothing here is distributed.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2504_19232_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.load()
    binding.adaptra_set_kernel_mode(args.kernel_mode)
    if args.probe_only:
        rates = probe_rates(binding, torch, torch.device("cuda:0"))
        slots = 256 * 4 * 2.4e9 / 4               # vector issue slots per second at one per SIMD per four cycles
        print(json.dumps({"probe_valu_instructions_per_s": rates,
                          "fraction_of_one_per_four_cycles_at_2.4GHz": {k: v / slots for k, v in rates.items()}}))
        return

    wl = workloads.config(args.config)
    S, M, C, K = wl.S, wl.M, wl.n_cand, wl.n_scen
    w_bound = int(wl.w.max())                      # known to whoever generated the candidates
    prob = binding.Problem.from_workload(wl, w_bound=w_bound)
    dev = prob.device
    ws = binding.alloc_workspace(prob)
    mk = torch.empty((K, C), dtype=torch.int32, device=dev)
    fl = torch.empty((K, C), dtype=torch.uint8, device=dev)
    bub = None if args.no_bubble else torch.empty((S, K, C), dtype=torch.int32, device=dev)
    bidx = torch.empty(K, dtype=torch.int32, device=dev)
    bmk = torch.empty(K, dtype=torch.int32, device=dev)
    bbub = torch.empty((K, S), dtype=torch.int32, device=dev)
    hist = torch.empty((S, wl.hist_bins), dtype=torch.int64, device=dev) if wl.hist_bins else None

    def step():
        if args.two_calls:
            binding.adaptra_eval(prob, mk, bub, fl, want_bubble=bub is not None, workspace=ws)
            binding.adaptra_best(prob, bidx, bmk, bbub, hist, workspace=ws)
        else:       # the same outputs, every pair resolved once
            binding.adaptra_eval_best(prob, mk, bub, fl, bidx, bmk, bbub, hist, want_bubble=bub is not None,
                                      workspace=ws)

    if args.copy_calibration:
        src = torch.zeros(1 << 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # per-step timing of adaptra_eval's recurrence kernel, through events the library records
    evs = HipEvents()
    pairs = [(evs.create(), evs.create()) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        binding.adaptra_set_resolve_events(pairs[i][0], pairs[i][1])
        if args.two_calls:
            binding.adaptra_eval(prob, mk, bub, fl, want_bubble=bub is not None, workspace=ws)
            binding.adaptra_set_resolve_events(None, None)
            binding.adaptra_best(prob, bidx, bmk, bbub, hist, workspace=ws)
        else:
            step()
            binding.adaptra_set_resolve_events(None, None)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_ms = [evs.elapsed_ms(a, b) for a, b in pairs]
    for a, b in pairs:
        evs.destroy(a)
        evs.destroy(b)

    # separate timings of the two entry points (outside the timed region)
    def timed(fn, n=3):
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / n

    t_eval = timed(lambda: binding.adaptra_eval(prob, mk, bub, fl, want_bubble=bub is not None, workspace=ws))
    t_best = timed(lambda: binding.adaptra_best(prob, bidx, bmk, bbub, hist, workspace=ws))

    # sustained issue rates of this GPU for the instructions the kernel is made of (no memory traffic)
    rates = probe_rates(binding, torch, dev)
    measured_peak = rates["add_max"] * 64          # int32 lane-ops/s of independent v_add_u32 / v_max_i32 chains

    def device_ms(fn, n):
        """Average duration of fn() over n back-to-back calls, by events on the stream fn enqueues on."""
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    # the analytic planning kernel (Algorithm 1 / 2 / Eq. (1)): HBM-bound, timed at 2^20 scenarios
    seed_info = None
    if S > 1:
        from paper_2504_19232_amd.workloads import _rng
        Ks = 1 << 20
        g = _rng(77)
        cfs = torch.from_numpy(g.integers(0, 50000, (S - 1, Ks)).astype(np.int32)).to(dev)
        cbs = torch.from_numpy(g.integers(0, 50000, (S - 1, Ks)).astype(np.int32)).to(dev)
        sprob = binding.Problem(M, prob.tensors[0], prob.tensors[1], prob.tensors[2], cfs, cbs)
        w_cur = torch.from_numpy(np.arange(S - 1, -1, -1, dtype=np.int32)).to(dev)
        seed_out = binding.adaptra_seed(sprob, S, w_cur, want_not_absorbed=True)
        t_seed = device_ms(lambda: binding.adaptra_seed(sprob, S, w_cur, out=seed_out), n=20) * 1e-3
        seed_bytes = Ks * (8 * (S - 1) + 4 * S + (S - 1))     # delays read once, w_adapted and the Eq. (1) bytes written
        seed_info = {"scenarios": Ks, "ms": t_seed * 1e3, "algorithmic_GBps": seed_bytes / t_seed / 1e9,
                     "frac_of_hbm_peak": seed_bytes / t_seed / 8e12,
                     "timing": "HIP events around 20 launches of k_seed, outputs preallocated"}
        del seed_out
        del cfs, cbs, sprob
        # how far the paper's own pick (Algorithm 2, one vector per scenario) is from the exhaustive
        # argmin over this workload's candidates: each vector evaluated under its own scenario
        if not args.no_sens:
            _, w_ad, _ = binding.adaptra_seed(prob, want_init=False)
            aprob = binding.Problem(M, prob.tensors[0], prob.tensors[1], w_ad, prob.tensors[3], prob.tensors[4],
                                    prob.tensors[5])
            amk, _, afl = binding.adaptra_eval(aprob, want_bubble=False)
            torch.cuda.synchronize()
            own = torch.arange(K, device=dev)
            a_mk, a_fl = amk[own, own], afl[own, own]
            ok = (a_fl == 1) & (bmk != 2 ** 31 - 1)
            live = ((a_fl & 2) == 0) & (bmk != 2 ** 31 - 1)
            seed_info["algorithm2_vs_exhaustive"] = {
                "within_memory_cap": int((a_fl == 1).sum()), "scenarios": int(K),
                "makespan_ratio_mean_where_within_cap": float((a_mk[ok].double() / bmk[ok].double()).mean()) if ok.any() else None,
                "makespan_ratio_mean_ignoring_cap": float((a_mk[live].double() / bmk[live].double()).mean()) if live.any() else None}
            del aprob, amk, afl

    # ZeroBubble (F / B / W) policy evaluation, first version: timed on configuration 1's
    # candidates and scenarios (S=8, N=32, 2^20 pairs, 3 S N = 768 ops per pair), t_w = t_b / 2
    zb_info = None
    if not args.no_zb:
        wz = workloads.config(1)
        zprob = binding.Problem.from_workload(wz)
        t_w = torch.from_numpy((wz.t_b // 2).astype(np.int32)).to(dev)
        zws = torch.empty(binding.load().adaptra_zb_workspace_bytes(ctypes.byref(zprob.params), zprob.C, zprob.K),
                          dtype=torch.uint8, device=dev)
        binding.adaptra_zb_eval(zprob, t_w, -1, workspace=zws)
        t_zb = timed(lambda: binding.adaptra_zb_eval(zprob, t_w, -1, workspace=zws), n=2)
        t_zbp = timed(lambda: binding.adaptra_zb_eval(zprob, t_w, 0, workspace=zws), n=2)
        zops = zprob.C * zprob.K * 3 * wz.S * wz.M
        # Integer work a started op cannot do without.  Policy: the earliest-action scan over the
        # stages (S - 1 comparisons), the choice among backward / forward / weight op (2), the
        # start (one max), the finish and the arrival it posts (two adds): S + 4.  A fixed plan
        # replayed: max, add, add.
        zb_policy_ops, zb_replay_ops = wz.S + 4, 3
        zb_info = {"workload": f"{wz.name} + W ops: {zprob.C} candidates x {zprob.K} scenarios",
                   "policy_ms": t_zb * 1e3, "policy_evaluations_per_s": zprob.C * zprob.K / t_zb,
                   "policy_resolved_ops_per_s": zops / t_zb,
                   "fixed_plan_ms": t_zbp * 1e3, "fixed_plan_evaluations_per_s": zprob.C * zprob.K / t_zbp,
                   "roofline": {"bound": "alu", "peak": INT32_VALU_PEAK / 1e12, "unit": "Tint32op/s",
                                "policy": {"algorithmic_ops_per_resolved_op": zb_policy_ops,
                                           "achieved": zb_policy_ops * zops / t_zb / 1e12,
                                           "frac": zb_policy_ops * zops / t_zb / INT32_VALU_PEAK},
                                "fixed_plan": {"algorithmic_ops_per_resolved_op": zb_replay_ops,
                                               "achieved": zb_replay_ops * zops / t_zbp / 1e12,
                                               "frac": zb_replay_ops * zops / t_zbp / INT32_VALU_PEAK,
                                               "includes": "the recording launch (one scenario) and the replay under all"}}}
        del zws, zprob

    # computation stragglers (per-scenario stage times) on the same workload, and the link
    # sensitivities of 64 of its candidates (S copies of every scenario per candidate)
    vt_info = sens_info = None
    if not args.no_sens and S > 1:
        tfs, tbs = workloads.straggler_stage_times(99, wl)
        vprob = binding.Problem.from_workload(wl, dev, w_bound, t_f_scen=tfs, t_b_scen=tbs)
        binding.adaptra_eval(vprob, mk, bub, fl, want_bubble=bub is not None, workspace=ws)
        t_vt = timed(lambda: binding.adaptra_eval(vprob, mk, bub, fl, want_bubble=bub is not None, workspace=ws))
        vt_info = {"eval_ms": t_vt * 1e3, "evaluations_per_s": C * K / t_vt, "vs_fixed_stage_times": t_eval / t_vt}
        del vprob
        pick = np.flatnonzero((fl[0].cpu().numpy() & 2) == 0)
        pick = pick[:: max(1, len(pick) // 64)][:64]
        sub = workloads.Workload(**{**wl.__dict__, "w": np.ascontiguousarray(wl.w[:, pick])})
        sprob2 = binding.Problem.from_workload(sub, dev, w_bound)
        sws = torch.empty(binding.load().adaptra_sensitivity_workspace_bytes(ctypes.byref(sprob2.params), sprob2.C, sprob2.K),
                          dtype=torch.uint8, device=dev)
        sens_out = binding.adaptra_sensitivity(sprob2, 1, workspace=sws)
        t_sens = device_ms(lambda: binding.adaptra_sensitivity(sprob2, 1, workspace=sws, out=sens_out), n=10) * 1e-3
        sens_info = {"candidates": int(sprob2.C), "scenarios": int(K), "links": S - 1, "ms": t_sens * 1e3,
                     "evaluations_per_s": sprob2.C * K * S / t_sens,
                     "timing": "HIP events around 10 calls, outputs preallocated"}
        del sws, sprob2, sens_out

    # guided search (neighbourhood descent on batched evaluation) over the same scenarios,
    # from the plain 1F1B schedule; compared with the exhaustive argmin over the workload's candidates
    search_info = None
    if not args.no_sens and S > 1:
        w_init = torch.arange(S - 1, -1, -1, dtype=torch.int32, device=dev)   # plain 1F1B: fits every cap here
        sws = torch.empty(binding.load().adaptra_search_workspace_bytes(ctypes.byref(prob.params), K, 1),
                          dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        sw, smk, rounds, evaluated = binding.adaptra_search(prob, w_init, 1, 500, workspace=sws)
        torch.cuda.synchronize()
        t_search = time.perf_counter() - t0
        found = (bmk != 2 ** 31 - 1) & (smk != 2 ** 31 - 1)
        ratio = (smk[found].double() / bmk[found].double())
        search_info = {"neighbourhood": 1, "start": "plain 1F1B, w_s = S - 1 - s", "rounds": rounds,
                       "pairs_evaluated": evaluated, "ms": t_search * 1e3,
                       "evaluations_per_s": evaluated / t_search,
                       "makespan_vs_exhaustive_over_candidates_mean": float(ratio.mean()) if ratio.numel() else None,
                       "makespan_vs_exhaustive_over_candidates_max": float(ratio.max()) if ratio.numel() else None}
        del sws

    # the online decision (one measured scenario, all candidates): latency of adaptra_best alone
    online_info = None
    if not args.no_sens and S > 1:
        one = binding.Problem(M, prob.tensors[0], prob.tensors[1], prob.tensors[2],
                              prob.tensors[3][:, :1].contiguous(), prob.tensors[4][:, :1].contiguous(),
                              prob.tensors[5], w_bound=w_bound)
        oidx = torch.empty(1, dtype=torch.int32, device=dev)
        omk = torch.empty(1, dtype=torch.int32, device=dev)
        binding.adaptra_best(one, oidx, omk, None, None, want_bubble=False, workspace=ws)
        t_one = timed(lambda: binding.adaptra_best(one, oidx, omk, None, None, want_bubble=False, workspace=ws), n=20)
        online_info = {"candidates": C, "scenarios": 1, "best_ms": t_one * 1e3,
                       "kernel": "candidate lanes, read-ahead form (few scenarios)"}
        del one

    flags = fl[0].cpu().numpy()                    # the flag depends on the candidate only
    n_live = int(((flags & 2) == 0).sum())
    n_feasible = int((flags == 1).sum())
    ops_per_pair = 2 * S * M
    ops_eval = n_live * K * ops_per_pair           # ops resolved by adaptra_eval's kernel per launch
    ops_best = n_feasible * K * ops_per_pair
    hot_S = next((p for p in (2, 4, 8, 16, 32) if S <= p), S)     # the hot kernel's instantiated size
    ms_step = dt / args.steps * 1e3
    kernel_avg_ms = float(np.mean(kernel_ms))
    achieved = 3.0 * ops_eval / (kernel_avg_ms * 1e-3)
    prof = from_profile(hot_S, args.config)
    simds = 256 * 4
    # the kernel's own formulation: per resolved op one add at the double rate (2 SIMD cycles per
    # wavefront instruction) and one max (4 cycles), nothing else
    floor_s = ops_eval / 64 * (2 + 4) / (simds * 2.4e9)
    busy_min = busy_max = None
    if prof["valu_instructions"] and prof["cycles"]:
        busy_max = prof["valu_instructions"] * 4 / (simds * prof["cycles"])
        busy_min = (prof["valu_instructions"] * 4 - ops_eval / 64 * 2) / (simds * prof["cycles"])

    out = {
        "metric": "schedule_evaluations_per_sec",
        "value": C * K / (dt / args.steps),
        "unit": "evaluations/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {wl.name}: S={S}, M={M}, {C} candidates x {K} scenarios "
                               f"= {C * K} pairs; step = "
                               + (f"adaptra_eval (makespan{'' if args.no_bubble else ' + bubbles'} + flags) + adaptra_best"
                                  if args.two_calls else
                                  f"adaptra_eval_best (makespan{'' if args.no_bubble else ' + bubbles'} + flags + "
                                  f"per-scenario argmin + histogram, every pair resolved once)"),
                   "pairs": C * K, "not_deadlocked_candidates": n_live, "feasible_candidates": n_feasible,
                   "w_bound": w_bound, "kernel_mode": args.kernel_mode, "inputs_sha256": wl.sha256()},
        "resolved_ops_per_s": (ops_eval + (ops_best if args.two_calls else 0)) / (dt / args.steps),
        "eval": {"ms": t_eval * 1e3, "evaluations_per_s": C * K / t_eval, "resolved_ops_per_s": ops_eval / t_eval},
        "best": {"ms": t_best * 1e3, "evaluations_per_s": C * K / t_best, "resolved_ops_per_s": ops_best / t_best},
        "roofline": {"bound": "alu", "kernel": f"k_resolve_scen_lanes<{hot_S}, false, false>",
                     "achieved": achieved / 1e12, "peak": INT32_VALU_PEAK / 1e12, "unit": "Tint32op/s",
                     "frac": achieved / INT32_VALU_PEAK, "traffic": prof["traffic"],
                     "frac_formulation": floor_s / (kernel_avg_ms * 1e-3),
                     "valu_busy_min": busy_min, "valu_busy_max": busy_max,
                     "peak_measured": measured_peak / 1e12, "frac_of_measured": achieved / measured_peak,
                     "probe_valu_instructions_per_simd_per_4_cycles": {k: v / (simds * 2.4e9 / 4) for k, v in rates.items()},
                     "kernel_ms": kernel_avg_ms, "resolved_ops_per_launch": ops_eval,
                     "algorithmic_ops_per_resolved_op": 3, "profile_is_current": prof["profile_is_current"]},
    }
    if seed_info:
        out["seed"] = seed_info
    if zb_info:
        out["zb"] = zb_info
    if vt_info:
        out["stage_time_scenarios"] = vt_info
        out["sensitivity"] = sens_info
    if search_info:
        out["search"] = search_info
    if online_info:
        out["online_decision"] = online_info
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
