"""GPU parity: the HIP library, called through its C ABI (ctypes), against the CPU oracle
on the same seeded inputs.  All values are integers, so the bar is bit-exact."""
import sys

import numpy as np
import pytest

from paper_2504_19232_amd import workloads

pytestmark = pytest.mark.gpu

INT32_MAX = 2 ** 31 - 1


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_19232_amd import binding
    binding.load()
    yield binding
    binding.adaptra_set_kernel_mode(0)


def gpu_eval(binding, wl, mode=0, want_bubble=True, w_bound=-1):
    import torch
    binding.adaptra_set_kernel_mode(mode)
    prob = binding.Problem.from_workload(wl, w_bound=w_bound)
    mk, bub, fl = binding.adaptra_eval(prob, want_bubble=want_bubble)
    torch.cuda.synchronize()
    binding.adaptra_set_kernel_mode(0)
    return mk.cpu().numpy(), None if bub is None else bub.cpu().numpy(), fl.cpu().numpy()


def gpu_best(binding, wl, mode=0, w_bound=-1):
    import torch
    binding.adaptra_set_kernel_mode(mode)
    prob = binding.Problem.from_workload(wl, w_bound=w_bound)
    idx, mk, bub, hist = binding.adaptra_best(prob)
    torch.cuda.synchronize()
    binding.adaptra_set_kernel_mode(0)
    return (idx.cpu().numpy(), mk.cpu().numpy(), bub.cpu().numpy(),
            None if hist is None else hist.cpu().numpy().astype(np.uint64))


def check_full(binding, oracle, wl, modes=(0, 1, 2, 3, 4)):
    ref = oracle.eval_workload(wl)
    rbest = oracle.best_from_eval(ref["makespan"], ref["flag"], ref["bubble"])
    rhist = (oracle.hist_from_eval(ref["bubble"], ref["flag"], wl.hist_bins, wl.hist_shift)
             if wl.hist_bins else None)
    for mode in modes:
        say(f"  {wl.name}: eval mode {mode}")
        mk, bub, fl = gpu_eval(binding, wl, mode)
        assert np.array_equal(fl, ref["flag"]), f"flag mismatch mode {mode}"
        assert np.array_equal(mk, ref["makespan"]), f"makespan mismatch mode {mode}"
        assert np.array_equal(bub, ref["bubble"]), f"bubble mismatch mode {mode}"
        say(f"  {wl.name}: best mode {mode}")
        idx, bmk, bbub, hist = gpu_best(binding, wl, mode)
        assert np.array_equal(idx, rbest["best_idx"]), f"best_idx mismatch mode {mode}"
        assert np.array_equal(bmk, rbest["best_makespan"])
        assert np.array_equal(bbub, rbest["best_bubble"])
        if rhist is not None:
            assert np.array_equal(hist, rhist), f"histogram mismatch mode {mode}"
        say(f"  {wl.name}: eval + best in one call, mode {mode}")
        import torch
        binding.adaptra_set_kernel_mode(mode)
        out = binding.adaptra_eval_best(binding.Problem.from_workload(wl))
        torch.cuda.synchronize()
        binding.adaptra_set_kernel_mode(0)
        mk, bub, fl, idx, bmk, bbub, hist = [None if t is None else t.cpu().numpy() for t in out]
        assert np.array_equal(fl, ref["flag"]) and np.array_equal(mk, ref["makespan"])
        assert np.array_equal(bub, ref["bubble"])
        assert np.array_equal(idx, rbest["best_idx"]), f"fused best_idx mismatch mode {mode}"
        assert np.array_equal(bmk, rbest["best_makespan"]) and np.array_equal(bbub, rbest["best_bubble"])
        if rhist is not None:
            assert np.array_equal(hist.astype(np.uint64), rhist), f"fused histogram mismatch mode {mode}"


@pytest.mark.parametrize("index", [0, 1])
def test_config_full_parity(lib, oracle, index):
    wl = workloads.config(index)
    say(f"config {index}: {wl.name}, {wl.n_pairs} pairs")
    check_full(lib, oracle, wl)


RAGGED = [
    # seed, S, M, C, K, kwargs
    (1, 1, 1, 5, 3, {}),
    (2, 1, 7, 70, 65, dict(hist_bins=8, hist_shift=6)),
    (3, 2, 3, 33, 64, {}),
    (4, 3, 5, 100, 7, {}),                      # 3 stages: runs padded in the 4-stage kernel
    (5, 4, 8, 257, 129, dict(hist_bins=16, hist_shift=8)),
    (6, 4, 1, 64, 64, {}),                      # a single micro-batch
    (7, 5, 12, 130, 40, dict(cap=False)),
    (8, 8, 32, 1000, 64, dict(d_max=7, hist_bins=64, hist_shift=10)),
    (9, 8, 100, 300, 100, dict(w_extra=60)),    # deep warm-ups: the largest ring classes
    (10, 8, 9, 200, 64, dict(w_extra=20)),      # w above M-1 everywhere: clamped
    (11, 16, 64, 500, 70, dict(d_max=4)),
    (12, 16, 20, 77, 128, dict(w_extra=3, hist_bins=300, hist_shift=7)),   # histogram too wide for LDS
    (13, 32, 40, 150, 64, dict(d_max=4)),
    (14, 32, 128, 64, 65, dict(d_max=4, c_hi=50000)),
    (15, 64, 70, 40, 30, dict(d_max=2)),
    (16, 2, 300, 50, 64, dict(w_extra=1)),
    (17, 8, 64, 17, 1, dict()),                 # a single scenario
    (18, 8, 200, 64, 64, dict(w_extra=40)),     # ring classes 5-6
    (19, 4, 32768, 6, 3, dict(d_max=2)),        # the largest M: general kernel (K = 3)
    (20, 4, 32768, 5, 64, dict(d_max=2, c_hi=300, t_hi=30)),   # the largest M: on-chip kernels
    (21, 64, 300, 70, 3, dict(d_max=1)),        # the largest S
    (22, 8, 16, 1, 1, dict()),                  # one pair
    (23, 16, 40, 1000, 192, dict(d_max=3, hist_bins=5, hist_shift=11)),   # three full scenario tiles
    (24, 2, 2, 4000, 100, dict(d_max=1)),
    # stage counts between the hot kernel's sizes (padded with zero-time stages)
    (25, 6, 20, 300, 33, dict(hist_bins=32, hist_shift=7)),
    (26, 12, 48, 200, 70, dict(d_max=3, hist_bins=16, hist_shift=9)),
    (27, 17, 30, 50, 64, dict(d_max=3)),
    (28, 24, 64, 100, 65, dict(d_max=3, c_hi=20000)),
    (29, 31, 40, 64, 64, dict(d_max=3, hist_bins=200, hist_shift=8)),
    (30, 33, 40, 20, 10, dict(d_max=2)),        # beyond the hot kernel: general kernel
    (31, 4, 400, 40, 64, dict(w_extra=300)),    # warm-ups deeper than the 128-slot LDS ring: general kernel
    (32, 8, 160, 30, 3, dict(w_extra=120)),     # the same with few scenarios
    # the kernel sizes between the powers of two (12, 24, 48 stages) and pipelines padded into them
    (33, 10, 30, 90, 70, dict(d_max=3, hist_bins=16, hist_shift=9)),
    (34, 20, 50, 80, 66, dict(d_max=3)),
    (35, 24, 128, 64, 64, dict(d_max=4, c_hi=30000)),
    (36, 48, 40, 30, 20, dict(d_max=2)),
    (37, 40, 64, 50, 5, dict(d_max=2)),
    (38, 12, 100, 40, 64, dict(w_extra=70)),    # 12 stages with deep warm-ups
]


@pytest.mark.parametrize("seed,S,M,C,K,kw", RAGGED, ids=[f"S{r[1]}_M{r[2]}_C{r[3]}_K{r[4]}" for r in RAGGED])
def test_ragged_shapes_full_parity(lib, oracle, seed, S, M, C, K, kw):
    wl = workloads.random_workload(seed, S, M, C, K, **kw)
    say(f"ragged {wl.name}")
    check_full(lib, oracle, wl)


def test_no_feasible_candidate(lib, oracle):
    wl = workloads.random_workload(40, 4, 6, 90, 70)
    wl.mem_cap[:] = 0                                   # nobody fits
    check_full(lib, oracle, wl)
    idx, mk, bub, _ = gpu_best(lib, wl)
    assert np.all(idx == -1) and np.all(mk == INT32_MAX) and np.all(bub == INT32_MAX)


def test_zero_times_and_zero_delays(lib, oracle):
    wl = workloads.random_workload(41, 8, 16, 128, 64, cap=False)
    wl.t_f[::2] = 0
    wl.t_b[1::3] = 0
    wl.c_fwd[:] = 0
    wl.c_bwd[::2] = 0
    check_full(lib, oracle, wl)


def _sampled_parity(lib, oracle, index, n_sample, full_scenarios):
    """A full-size configuration through the very call bench.py times -- adaptra_eval_best with
    a w_bound hint, every output preallocated, bubbles on, histogram where the configuration has
    one -- checked against the oracle on
      (a) a seeded sample of n_sample pairs: flag, makespan and all S bubbles, read from the
          GPU's own output arrays;
      (b) whole scenarios (every candidate): evaluation and the search's pick;
    and, at any size, on properties of the complete arrays:
      (c) flags depend on the candidate only; deadlocked pairs carry the sentinels; every live
          bubble plane equals makespan - M (t_f + t_b);
      (d) the search equals a host argmin over the GPU's complete evaluation, the histogram a
          numpy.bincount over it;
      (e) adaptra_eval followed by adaptra_best gives the same arrays as the one call."""
    import torch
    wl = workloads.config(index)
    w_bound = int(wl.w.max())                          # as bench.py passes it
    S, K, C = wl.S, wl.n_scen, wl.n_cand
    say(f"config {index}: {wl.name}: adaptra_eval_best on {wl.n_pairs} pairs, bubbles on, w_bound {w_bound}")
    lib.adaptra_set_kernel_mode(0)
    prob = lib.Problem.from_workload(wl, w_bound=w_bound)
    dev = prob.device
    ws = lib.alloc_workspace(prob)
    d_mk = torch.empty((K, C), dtype=torch.int32, device=dev)
    d_fl = torch.empty((K, C), dtype=torch.uint8, device=dev)
    d_bub = torch.empty((S, K, C), dtype=torch.int32, device=dev)
    d_idx = torch.empty(K, dtype=torch.int32, device=dev)
    d_bmk = torch.empty(K, dtype=torch.int32, device=dev)
    d_bbub = torch.empty((K, S), dtype=torch.int32, device=dev)
    d_hist = torch.empty((S, wl.hist_bins), dtype=torch.int64, device=dev) if wl.hist_bins else None
    lib.adaptra_eval_best(prob, d_mk, d_bub, d_fl, d_idx, d_bmk, d_bbub, d_hist, workspace=ws)
    torch.cuda.synchronize()
    mk, fl = d_mk.cpu().numpy(), d_fl.cpu().numpy()
    idx, bmk, bbub = d_idx.cpu().numpy(), d_bmk.cpu().numpy(), d_bbub.cpu().numpy()
    hist = None if d_hist is None else d_hist.cpu().numpy().astype(np.uint64)
    tau = (wl.t_f + wl.t_b).astype(np.int64)
    # (a) sampled pairs: the GPU's arrays, gathered on the device, against the oracle
    pc, ps = workloads.sample_pairs(900 + index, C, K, n_sample)
    say(f"  (a) oracle on {n_sample} sampled pairs, bubbles included")
    ref = oracle.eval_workload(wl, pair_cand=pc, pair_scen=ps)
    t_pc, t_ps = torch.from_numpy(pc).to(dev), torch.from_numpy(ps).to(dev)
    assert np.array_equal(d_fl[t_ps, t_pc].cpu().numpy(), ref["flag"])
    assert np.array_equal(d_mk[t_ps, t_pc].cpu().numpy(), ref["makespan"])
    for s in range(S):
        assert np.array_equal(d_bub[s][t_ps, t_pc].cpu().numpy(), ref["bubble"][s]), f"bubble plane {s}"
    assert ((ref["flag"] & 2) == 0).sum() > n_sample // 2          # the sample is mostly live pairs
    # (c) the complete arrays
    say("  (c) complete arrays: flags, sentinels, bubble planes")
    assert bool((d_fl == d_fl[0:1]).all())
    dead = (d_fl[0] & 2) != 0
    assert bool((d_mk[:, dead] == INT32_MAX).all())
    t_tau = torch.from_numpy(tau).to(dev)
    for s in range(S):
        want = torch.where(dead[None, :], torch.full_like(d_mk, INT32_MAX), d_mk - int(wl.M * tau[s]))
        assert bool((d_bub[s] == want).all()), f"bubble plane {s} is not makespan - M (t_f + t_b)"
        del want
    del t_tau
    # (d) search == argmin over the GPU's evaluation
    say("  (d) search vs host argmin over the GPU evaluation")
    masked = np.where(fl == 1, mk.astype(np.int64), np.int64(2) ** 40)
    want_idx = masked.argmin(axis=1).astype(np.int32)
    any_ok = (fl == 1).any(axis=1)
    want_idx[~any_ok] = -1
    want_mk = np.where(any_ok, masked.min(axis=1), INT32_MAX).astype(np.int32)
    del masked
    assert np.array_equal(idx, want_idx)
    assert np.array_equal(bmk, want_mk)
    want_bub = np.where(any_ok[:, None], want_mk.astype(np.int64)[:, None] - wl.M * tau[None, :], INT32_MAX)
    assert np.array_equal(bbub.astype(np.int64), want_bub)
    if wl.hist_bins:
        want = np.zeros((wl.S, wl.hist_bins), dtype=np.uint64)
        ok = fl == 1
        for s in range(wl.S):
            b = np.minimum(wl.hist_bins - 1, (mk[ok].astype(np.int64) - wl.M * tau[s]) >> wl.hist_shift)
            want[s] = np.bincount(b, minlength=wl.hist_bins).astype(np.uint64)
        assert np.array_equal(hist, want)
    # (e) the two separate calls write the same arrays
    say("  (e) adaptra_eval + adaptra_best vs the one call")
    e_mk, e_fl = torch.empty_like(d_mk), torch.empty_like(d_fl)
    d_bub2 = torch.empty_like(d_bub)
    lib.adaptra_eval(prob, e_mk, d_bub2, e_fl, workspace=ws)
    b_out = lib.adaptra_best(prob, workspace=ws)
    torch.cuda.synchronize()
    assert bool((e_mk == d_mk).all()) and bool((e_fl == d_fl).all()) and bool((d_bub2 == d_bub).all())
    del d_bub2, e_mk, e_fl
    assert np.array_equal(b_out[0].cpu().numpy(), idx) and np.array_equal(b_out[1].cpu().numpy(), bmk)
    assert np.array_equal(b_out[2].cpu().numpy(), bbub)
    if wl.hist_bins:
        assert np.array_equal(b_out[3].cpu().numpy().astype(np.uint64), hist)
    # (b) whole scenarios through the oracle, search included
    for k in full_scenarios:
        say(f"  (b) oracle on all {C} candidates of scenario {k}")
        cand = np.arange(C, dtype=np.int64)
        ref = oracle.eval_workload(wl, pair_cand=cand, pair_scen=np.full(C, k, dtype=np.int64))
        assert np.array_equal(fl[k], ref["flag"])
        assert np.array_equal(mk[k], ref["makespan"])
        assert np.array_equal(d_bub[:, k, :].cpu().numpy(), ref["bubble"])
        rb = oracle.best_from_eval(ref["makespan"][None, :], ref["flag"][None, :], ref["bubble"][:, None, :])
        assert idx[k] == rb["best_idx"][0] and bmk[k] == rb["best_makespan"][0]
        assert np.array_equal(bbub[k], rb["best_bubble"][0])


def test_config2_sampled_parity(lib, oracle):
    _sampled_parity(lib, oracle, 2, 1 << 20, (0, 131))


def test_config3_sampled_parity(lib, oracle):
    _sampled_parity(lib, oracle, 3, 1 << 20, (0, 517))


def test_config4_sampled_parity(lib, oracle):
    _sampled_parity(lib, oracle, 4, 1 << 20, (37, 63))


NEAR_BOUND = [
    # seed, S, M, C, K, kwargs: 2 M S (max time + max delay) is 99 % of 2^31
    (81, 8, 32, 200, 70, dict(hist_bins=16, hist_shift=24)),
    (82, 4, 1, 70, 64, {}),                       # one micro-batch: the largest times of all
    (83, 16, 2, 90, 65, dict(d_max=1)),
    (84, 32, 64, 64, 64, dict(d_max=4)),
    (85, 5, 300, 40, 33, dict(w_extra=20)),       # padded to 8 stages, deep warm-ups
    (86, 2, 4000, 10, 64, dict(d_max=1)),
]


@pytest.mark.parametrize("seed,S,M,C,K,kw", NEAR_BOUND, ids=[f"S{r[1]}_M{r[2]}_C{r[3]}_K{r[4]}" for r in NEAR_BOUND])
def test_times_near_the_int32_bound(lib, oracle, seed, S, M, C, K, kw):
    """Times and delays so large that the precondition 2 M S (max t + max c) < 2^31 holds with
    1 % to spare: the shifted times of the scenario-lanes kernel and its "no earlier op"
    sentinel of -2^30 are closest to their limits here.  Every kernel mode, element by element."""
    wl = workloads.near_bound_workload(seed, S, M, C, K, **kw)
    bound = 2 * M * S * (int(max(wl.t_f.max(), wl.t_b.max())) + int(max(wl.c_fwd.max(), wl.c_bwd.max())))
    assert 0.98 * 2 ** 31 <= bound < 2 ** 31
    clean = workloads.near_bound_workload(seed, S, M, C, K, **kw)
    np.maximum(clean.w, 0, out=clean.w)                 # the generator plants negative w to test the clamp
    assert lib.adaptra_check_inputs(lib.Problem.from_workload(clean)) == lib.OK
    say(f"near the bound: {wl.name}, 2MS(t+c) = {bound / 2 ** 31:.4f} x 2^31")
    check_full(lib, oracle, wl)


@pytest.mark.parametrize("promise", ["kept", "broken"])
def test_direct_output_of_the_hot_kernel(lib, oracle, promise):
    """With a w_bound hint and chunks of 16 candidates the scenario-lanes kernel writes makespan,
    flags and bubbles itself; the epilogue only redoes tiles that hold candidates left to the
    general kernel.  A quarter of configuration 3 (16 384 candidates x 1024 scenarios, bubbles
    on), once with a true bound and once with a bound some candidates exceed."""
    wl = workloads.config(3)
    wl.w = np.ascontiguousarray(wl.w[:, 8192:8192 + 16384])
    w_max = int(wl.w.max())
    w_bound = w_max if promise == "kept" else 31
    if promise == "broken":
        assert (np.clip(wl.w[0], 0, wl.M - 1) > 31).any()
    say(f"direct output, promise {promise}: w_bound {w_bound}, largest w {w_max}")
    mk, bub, fl = gpu_eval(lib, wl, want_bubble=True, w_bound=w_bound)
    pc, ps = workloads.sample_pairs(78, wl.n_cand, wl.n_scen, 1 << 12)
    if promise == "broken":                              # make sure candidates beyond the bound are sampled
        deep = np.flatnonzero(np.clip(wl.w[0], 0, wl.M - 1) > 31)[:512]
        pc = np.concatenate([pc, deep])
        ps = np.concatenate([ps, np.arange(len(deep)) % wl.n_scen])
    ref = oracle.eval_workload(wl, pair_cand=pc, pair_scen=ps)
    assert np.array_equal(fl[ps, pc], ref["flag"])
    assert np.array_equal(mk[ps, pc], ref["makespan"])
    assert np.array_equal(bub[:, ps, pc], ref["bubble"])
    # everything the oracle did not sample: flags depend on the candidate only, deadlocked pairs
    # carry sentinels, live bubbles are makespan - M (t_f + t_b)
    assert np.array_equal(fl, np.broadcast_to(fl[0], fl.shape))
    dead = (fl[0] & 2) != 0
    assert np.all(mk[:, dead] == INT32_MAX) and np.all(bub[:, :, dead] == INT32_MAX)
    tau = (wl.t_f + wl.t_b).astype(np.int64)
    live = ~dead
    for s in range(0, wl.S, 5):
        assert np.array_equal(bub[s][:, live].astype(np.int64), mk[:, live].astype(np.int64) - wl.M * tau[s])


def test_bubble_output_at_full_size_config3_subset(lib, oracle):
    """Bubble array written by the benchmarked launch shape (S = 32): a slice of configuration 3
    (all scenarios, 2048 candidates) with the bubble output on, sampled against the oracle."""
    wl = workloads.config(3)
    wl.w = np.ascontiguousarray(wl.w[:, 4096:4096 + 2048])
    mk, bub, fl = gpu_eval(lib, wl, want_bubble=True)
    pc, ps = workloads.sample_pairs(77, wl.n_cand, wl.n_scen, 1 << 11)
    ref = oracle.eval_workload(wl, pair_cand=pc, pair_scen=ps)
    assert np.array_equal(fl[ps, pc], ref["flag"])
    assert np.array_equal(mk[ps, pc], ref["makespan"])
    assert np.array_equal(bub[:, ps, pc], ref["bubble"])
    tau = (wl.t_f + wl.t_b).astype(np.int64)
    live = (fl & 2) == 0
    full = mk.astype(np.int64)[None] - wl.M * tau[:, None, None]
    assert np.array_equal(bub.astype(np.int64)[:, live], full[:, live])
    assert np.all(bub[:, ~live] == INT32_MAX)


def test_errors_and_check_inputs(lib):
    import torch
    b = lib
    wl = workloads.random_workload(50, 4, 8, 64, 64)
    prob = b.Problem.from_workload(wl)
    ws = b.alloc_workspace(prob)
    assert b.adaptra_check_inputs(prob, ws) == b.ERANGE      # random_workload plants negative w
    wl.w = np.abs(wl.w)
    prob = b.Problem.from_workload(wl)
    assert b.adaptra_check_inputs(prob, ws) == b.OK
    wl2 = workloads.random_workload(51, 4, 8, 64, 64)
    wl2.w = np.abs(wl2.w)
    wl2.c_fwd[1, 3] = -1
    assert b.adaptra_check_inputs(b.Problem.from_workload(wl2), ws) == b.ERANGE
    wl3 = workloads.random_workload(52, 4, 8, 64, 64)
    wl3.w = np.abs(wl3.w)
    wl3.c_bwd[2, 5] = 2 ** 31 // (2 * 4 * 8)                 # 2 M S (t + c) reaches 2^31
    assert b.adaptra_check_inputs(b.Problem.from_workload(wl3), ws) == b.EOVERFLOW
    # too small / misaligned workspace, bad sizes
    with pytest.raises(b.AdaptraError) as e:
        b.adaptra_eval(prob, workspace=ws[:1024])
    assert e.value.code == b.EWORKSPACE
    with pytest.raises(b.AdaptraError) as e:
        b.adaptra_eval(prob, workspace=ws[1:])
    assert e.value.code == b.EWORKSPACE
    bad = b.Problem.from_workload(wl)
    bad.params.M = 0
    with pytest.raises(b.AdaptraError) as e:
        b.adaptra_eval(bad, workspace=ws)
    assert e.value.code == b.EINVAL
    bad = b.Problem.from_workload(wl)
    bad.params.hist_bins = 4                                  # histogram requested, no buffer
    bad.hist_bins = 0
    with pytest.raises(b.AdaptraError) as e:
        b.adaptra_best(bad, workspace=ws)
    assert e.value.code == b.EINVAL
    torch.cuda.synchronize()


def test_runs_on_a_side_stream_and_is_repeatable(lib, oracle):
    import torch
    b = lib
    wl = workloads.random_workload(60, 8, 24, 512, 64, hist_bins=32, hist_shift=8)
    ref = oracle.eval_workload(wl)
    rbest = oracle.best_from_eval(ref["makespan"], ref["flag"], ref["bubble"])
    prob = b.Problem.from_workload(wl)
    ws = b.alloc_workspace(prob)
    st = torch.cuda.Stream()
    outs = []
    with torch.cuda.stream(st):
        for _ in range(3):
            mk, bub, fl = b.adaptra_eval(prob, workspace=ws)
            idx, bmk, bbub, hist = b.adaptra_best(prob, workspace=ws)
            outs.append((mk, idx, hist))
    st.synchronize()
    for mk, idx, hist in outs:
        assert np.array_equal(mk.cpu().numpy(), ref["makespan"])
        assert np.array_equal(idx.cpu().numpy(), rbest["best_idx"])
    assert torch.equal(outs[0][2], outs[2][2])               # histogram overwritten, not accumulated


@pytest.mark.parametrize("bound", [-1, 3, 10, 17, 63, 1000])
def test_w_bound_promise_kept_or_broken(lib, oracle, bound):
    """The w_bound hint only sizes the on-chip ring; results must not depend on it, even when
    candidates exceed it (those take the general kernel)."""
    import torch
    b = lib
    wl = workloads.random_workload(70, 8, 40, 400, 64, d_max=6, w_extra=4, hist_bins=16, hist_shift=9)
    ref = oracle.eval_workload(wl)
    rbest = oracle.best_from_eval(ref["makespan"], ref["flag"], ref["bubble"])
    rhist = oracle.hist_from_eval(ref["bubble"], ref["flag"], wl.hist_bins, wl.hist_shift)
    prob = b.Problem.from_workload(wl, w_bound=bound)
    mk, bub, fl = b.adaptra_eval(prob)
    idx, bmk, bbub, hist = b.adaptra_best(prob)
    torch.cuda.synchronize()
    assert np.array_equal(fl.cpu().numpy(), ref["flag"])
    assert np.array_equal(mk.cpu().numpy(), ref["makespan"])
    assert np.array_equal(bub.cpu().numpy(), ref["bubble"])
    assert np.array_equal(idx.cpu().numpy(), rbest["best_idx"])
    assert np.array_equal(hist.cpu().numpy().astype(np.uint64), rhist)


@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_analytic_seed_parity(lib, index):
    """Algorithm 1, Algorithm 2 and the Eq. (1) test on the GPU against the step-by-step oracle,
    on the scenario sets of the five configurations."""
    import torch
    from oracle import seed
    b = lib
    wl = workloads.config(index)
    prob = b.Problem.from_workload(wl)
    x_max = wl.S + 3
    w_init, w_ad, _ = b.adaptra_seed(prob, x_max)
    _, _, na = b.adaptra_seed(prob, 1, w_init, want_init=False, want_adapted=False, want_not_absorbed=True)
    torch.cuda.synchronize()
    w_init, w_ad, na = w_init.cpu().numpy(), w_ad.cpu().numpy(), na.cpu().numpy()
    ref_init = seed.to_w(seed.initial_plan(wl.S, x_max))
    assert list(w_init) == ref_init
    ks = range(wl.n_scen) if wl.n_scen <= 64 else range(0, wl.n_scen, 7)
    for k in ks:
        ref = seed.to_w(seed.adapted_plan(wl.S, wl.M, wl.t_f, wl.t_b, wl.c_fwd[:, k], wl.c_bwd[:, k]))
        assert list(w_ad[:, k]) == ref, k
        ok = seed.absorbed(wl.S, wl.t_f, wl.t_b, ref_init, wl.c_fwd[:, k], wl.c_bwd[:, k])
        assert list(na[:, k]) == [0 if v else 1 for v in ok], k


def test_analytic_seed_edge_cases(lib):
    import torch
    from oracle import seed
    b = lib
    for (sd, S, M, K) in [(1, 1, 5, 3), (2, 2, 3, 70), (3, 6, 9, 10), (4, 64, 200, 5), (5, 5, 4000, 300)]:
        wl = workloads.random_workload(sd, S, M, 8, K, c_hi=60000)
        if S > 2:
            wl.t_f[2] = 0
            wl.t_b[2] = 0                      # a zero denominator on link 1
        prob = b.Problem.from_workload(wl)
        for x_max in (1, 2, S, 3 * S + 1):
            w_init, w_ad, _ = b.adaptra_seed(prob, x_max)
            torch.cuda.synchronize()
            assert list(w_init.cpu().numpy()) == seed.to_w(seed.initial_plan(S, x_max))
        w_ad = w_ad.cpu().numpy()
        for k in range(K):
            ref = seed.to_w(seed.adapted_plan(S, M, wl.t_f, wl.t_b, wl.c_fwd[:, k], wl.c_bwd[:, k]))
            assert list(w_ad[:, k]) == ref
    with pytest.raises(b.AdaptraError):
        b.adaptra_seed(prob, 0)                  # x_max must be >= 1 for Algorithm 1


@pytest.mark.parametrize("M,K", [(7, 4000), (9, 4001), (40, 4002), (32768, 12000)])
def test_analytic_seed_ratios_at_their_boundaries(lib, M, K):
    """Algorithm 2's ceiling ratio where an inexact division would show: load = q * tau_next + e
    with e in {-1, 0, 1}, q from 0 to beyond the clip M - 2S, tau_next from 1 to 2^32 - 2 and
    loads up to 2^33 (per-scenario stage times, so that every scenario has a divisor of its own);
    zero divisors; Eq. (1) under slacks of either sign.  K not a multiple of 4 takes the kernel's
    one-scenario-per-thread form, the others its four-per-thread form."""
    import torch
    from oracle import seed as oseed
    S, big = 3, 2 ** 31 - 1
    rng = np.random.default_rng(1000 + M)
    clip = M - 2 * S
    tfs = np.zeros((S, K), np.int64); tbs = np.zeros((S, K), np.int64)
    cf = np.zeros((S - 1, K), np.int64); cb = np.zeros((S - 1, K), np.int64)
    den = np.floor(2.0 ** rng.uniform(0, 32, (S, K))).astype(np.int64).clip(1, 2 * big)
    den[:, rng.random(K) < 0.02] = 0                       # zero divisors (all stages of a scenario)
    den[1, rng.random(K) < 0.02] = 0
    tfs[:] = den // 2; tbs[:] = den - den // 2
    for i in range(S - 1):
        q = np.where(rng.random(K) < 0.5, rng.integers(0, 6, K),
                     np.where(rng.random(K) < 0.5, max(clip, 0) + rng.integers(-2, 3, K), rng.integers(0, max(clip, 4) + 3, K)))
        load = np.maximum(q, 0) * den[i + 1] + rng.integers(-1, 2, K)
        load = load.clip(den[i], den[i] + 2 * big)         # load = tau_i + c_fwd + c_bwd with both delays in int32
        rest = load - den[i]
        cf[i] = rest // 2; cb[i] = rest - rest // 2
    wl = workloads.random_workload(5, S, M, 8, K)
    wl.c_fwd = cf.astype(np.int32); wl.c_bwd = cb.astype(np.int32)
    prob = lib.Problem.from_workload(wl, t_f_scen=tfs.astype(np.int32), t_b_scen=tbs.astype(np.int32))
    for w_cur in ([5, 3, 0], [0, 4, 4], [-big, big, -big]):
        w_dev = torch.tensor(w_cur, dtype=torch.int32, device="cuda:0")
        _, w_ad, na = lib.adaptra_seed(prob, 1, w_current=w_dev, want_init=False, want_not_absorbed=True)
        torch.cuda.synchronize()
        w_ad, na = w_ad.cpu().numpy(), na.cpu().numpy()
        for k in range(K):
            x = oseed.adapted_plan(S, M, tfs[:, k], tbs[:, k], cf[:, k], cb[:, k])
            assert list(w_ad[:, k]) == oseed.to_w(x), k
            ab = oseed.absorbed(S, tfs[:, k], tbs[:, k], w_cur, cf[:, k], cb[:, k])
            assert list(na[:, k]) == [0 if a else 1 for a in ab], k


def test_algorithm2_pick_against_the_exhaustive_search(lib, oracle):
    """Algorithm 2's vectors are valid candidates: evaluating them (diagonal of the
    scenario x scenario grid) can never beat adaptra_best over a candidate set that contains them."""
    import torch
    b = lib
    wl = workloads.config(1)
    wl.mem_cap = None
    prob = b.Problem.from_workload(wl)
    _, w_ad, _ = b.adaptra_seed(prob, 1, want_init=False)
    torch.cuda.synchronize()
    w_all = np.concatenate([wl.w, w_ad.cpu().numpy()], axis=1)
    wl2 = workloads.Workload("cfg1+alg2", wl.S, wl.M, wl.t_f, wl.t_b, None, np.ascontiguousarray(w_all), wl.c_fwd, wl.c_bwd)
    mk, _, fl = gpu_eval(lib, wl2, want_bubble=False)
    idx, bmk, _, _ = gpu_best(lib, wl2)
    C0 = wl.n_cand
    diag = mk[np.arange(wl.n_scen), C0 + np.arange(wl.n_scen)]
    assert np.all(fl[:, C0:] == 1)              # Algorithm 2 never violates Lemma 1
    assert np.all(bmk <= diag)
    ref = oracle.eval_workload(wl2, pair_cand=C0 + np.arange(wl.n_scen), pair_scen=np.arange(wl.n_scen), want_bubble=False)
    assert np.array_equal(diag, ref["makespan"])


def _zb_problem(b, S, N, t_f, t_b, t_w, w, cf, cb):
    import torch
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    prob = b.Problem(N, up(t_f), up(t_b), up(w), up(cf), up(cb))
    return prob, up(t_w)


def test_zb_paper_example_on_gpu(lib):
    """The paper's printed ZeroBubble example through the GPU path: 390 ms without delay; the
    plan generated without delay takes 400 / 440 ms under 10 / 20 ms on link 0 <-> 1; re-planned
    under the delay it loses only the delay itself."""
    import torch
    b = lib
    S, N, t = 4, 12, 10000
    w = np.array([[6], [4], [2], [0]])                       # x = 7 5 3 1
    delays = [0, 10000, 20000]
    cf = np.zeros((S - 1, 3), dtype=np.int32)
    cf[0] = delays
    prob, t_w = _zb_problem(b, S, N, [t] * S, [t] * S, [t] * S, w, cf, cf)
    mk_own, _ = b.adaptra_zb_eval(prob, t_w, -1)
    mk_plan, bub = b.adaptra_zb_eval(prob, t_w, 0)
    torch.cuda.synchronize()
    assert list(mk_plan.cpu().numpy()[:, 0]) == [390000, 400000, 440000]
    assert list(mk_own.cpu().numpy()[:, 0]) == [390000, 400000, 410000]
    assert np.array_equal(bub.cpu().numpy()[:, :, 0], np.array([[30000, 40000, 80000]] * S))


ZB_CASES = [(1, 1, 1, 3, 2), (2, 2, 3, 9, 5), (3, 4, 8, 40, 21), (4, 8, 16, 70, 33), (5, 5, 7, 300, 4),
            (6, 16, 12, 20, 10), (7, 3, 40, 10, 64),
            (8, 32, 10, 6, 70),           # per-wavefront state above the default LDS limit
            (9, 64, 6, 150, 130),         # the largest S; more pairs than resident threads
            (10, 2, 255, 70, 3),          # the most micro-batches the one-word form of the cursors takes
            (11, 3, 256, 30, 4),          # the fewest that need the two-word form
            (12, 2, 300, 20, 6),
            # times in the millions: too large for the (time, stage) words of the earliest-action scan
            (13, 8, 16, 70, 9, 20000), (14, 19, 9, 30, 5, 3000),
            (15, 19, 9, 30, 5, 40),       # 19 stages pad to 24: a stage-index field wider than needed
            # fixed plans are replayed with the scenarios on the lanes from 8 scenarios on, up to 255 micro-batches
            (16, 2, 255, 20, 9), (17, 3, 256, 12, 9), (18, 5, 40, 9, 8), (19, 5, 40, 9, 7),
            (20, 64, 255, 3, 8),          # the largest per-wavefront state of that replay (129 KiB of LDS)
            # up to 16 stages plans are recorded with the stages on the lanes (groups of 8 or 16 lanes) and
            # replayed without weight ops: 11 stages in groups of 16, two tiles of scenarios, several blocks of
            # candidates, an order whose length is no multiple of the replay's 64-entry blocks; 7 stages likewise
            (21, 11, 20, 300, 70), (22, 7, 33, 130, 9), (23, 16, 31, 40, 64),
            (24, 8, 255, 9, 8),           # that recording's largest queues (one wavefront per CU)
            # more stage-lane wavefronts than are resident at once (263 of 85 KiB each): recorded with a lane per
            # candidate and replayed with the weight ops in the order
            (25, 3, 170, 2100, 20)]


@pytest.mark.parametrize("case", ZB_CASES, ids=["S%d_N%d_C%d_K%d" % c[1:5] + ("_x%d" % c[5] if len(c) > 5 else "") for c in ZB_CASES])
def test_zb_parity(lib, oracle, case):
    import torch
    b = lib
    seed_, S, N, C, K = case[:5]
    scale = case[5] if len(case) > 5 else 1
    rng = np.random.default_rng(seed_)
    t_f, t_b, t_w = rng.integers(1, 60, S), rng.integers(1, 90, S), rng.integers(0, 50, S)
    w = np.sort(rng.integers(-1, N + 3, (S, C)), axis=0)[::-1]
    w[:, ::5] = rng.integers(0, N, (S, len(range(0, C, 5))))           # some not monotone
    cf = rng.integers(0, 400, (max(S - 1, 0), K))
    cb = rng.integers(0, 400, (max(S - 1, 0), K))
    t_f, t_b, t_w, cf, cb = t_f * scale, t_b * scale, t_w * scale, cf * scale, cb * scale
    prob, t_w_d = _zb_problem(b, S, N, t_f, t_b, t_w, w, cf, cb)
    x = np.clip(w, 0, N - 1) + 1
    # the oracle sweeps every pair, or -- where that takes too long -- whole scenarios from
    # both ends of the pair range
    ks = np.arange(K) if S * N * C * K < 4_000_000 else np.unique(np.r_[0, K // 2, np.arange(K - 20, K, 3)])
    ref = oracle.zb_batch(S, N, t_f, t_b, t_w, x, cf[:, ks], cb[:, ks])
    mk, bub = b.adaptra_zb_eval(prob, t_w_d, -1)
    torch.cuda.synchronize()
    assert np.array_equal(mk.cpu().numpy()[ks], ref["makespan"])
    assert np.array_equal(bub.cpu().numpy()[:, ks], ref["idle"])
    # fixed plans generated under scenario 1 (or 0), replayed under every scenario
    kp = 1 if K > 1 else 0
    mkp, bubp = b.adaptra_zb_eval(prob, t_w_d, kp)
    torch.cuda.synchronize()
    mkp, bubp = mkp.cpu().numpy(), bubp.cpu().numpy()
    busy = N * (np.asarray(t_f) + np.asarray(t_b) + np.asarray(t_w))
    for c in range(0, C, max(1, C // 12)):
        gen = oracle.zb_simulate(S, N, t_f, t_b, t_w, cf[:, kp], cb[:, kp], x=x[:, c])
        for k in range(0, K, max(1, K // 6)):
            rep = oracle.zb_simulate(S, N, t_f, t_b, t_w, cf[:, k], cb[:, k], order=gen["order"])
            assert mkp[k, c] == rep["makespan"], (c, k)
            assert np.array_equal(bubp[:, k, c], rep["makespan"] - busy), (c, k)


def test_zb_benchmarked_shape(lib, oracle):
    """adaptra_zb_eval on the workload and in the launch shape bench.py times (configuration 1
    with weight ops, 16 384 candidates x 64 scenarios, more work units than resident wavefronts):
    a seeded sample of candidates under four scenarios against the oracle, for the policy and
    for fixed plans generated under scenario 0."""
    import torch
    from paper_2504_19232_amd import workloads
    b = lib
    wl = workloads.config(1)
    prob = b.Problem.from_workload(wl)
    t_w = (wl.t_b // 2).astype(np.int32)
    t_w_d = torch.from_numpy(t_w).cuda()
    S, N = wl.S, wl.M
    rng = np.random.default_rng(77)
    cs = np.unique(np.r_[0, wl.n_cand - 1, rng.integers(0, wl.n_cand, 400)])
    ks = np.array([0, 17, 40, wl.n_scen - 1])
    x = np.clip(wl.w, 0, N - 1) + 1
    ref = oracle.zb_batch(S, N, wl.t_f, wl.t_b, t_w, x[:, cs], wl.c_fwd[:, ks], wl.c_bwd[:, ks])
    mk, bub = b.adaptra_zb_eval(prob, t_w_d, -1)
    torch.cuda.synchronize()
    assert np.array_equal(mk.cpu().numpy()[np.ix_(ks, cs)], ref["makespan"])
    assert np.array_equal(bub.cpu().numpy()[:, ks][:, :, cs], ref["idle"])
    mkp, _ = b.adaptra_zb_eval(prob, t_w_d, 0, want_bubble=False)
    torch.cuda.synchronize()
    mkp = mkp.cpu().numpy()
    assert np.array_equal(mkp[0, cs], ref["makespan"][0])        # a plan replayed under its own scenario
    for c in cs[::40]:
        gen = oracle.zb_simulate(S, N, wl.t_f, wl.t_b, t_w, wl.c_fwd[:, 0], wl.c_bwd[:, 0], x=x[:, c])
        for k in ks[1:]:
            rep = oracle.zb_simulate(S, N, wl.t_f, wl.t_b, t_w, wl.c_fwd[:, k], wl.c_bwd[:, k], order=gen["order"])
            assert mkp[k, c] == rep["makespan"], (c, k)


def test_zb_check_inputs(lib):
    """adaptra_zb_check_inputs: the preconditions of adaptra_zb_eval on the device data --
    forward and backward times of at least 1 us (weight times may be 0), nothing negative,
    3 M S (max time + max delay) below 2^31."""
    b = lib
    S, N, C, K = 4, 8, 20, 6
    rng = np.random.default_rng(5)
    good = dict(t_f=rng.integers(1, 60, S), t_b=rng.integers(1, 90, S), t_w=rng.integers(0, 50, S),
                w=np.sort(rng.integers(0, N, (S, C)), axis=0)[::-1],
                cf=rng.integers(0, 400, (S - 1, K)), cb=rng.integers(0, 400, (S - 1, K)))
    good["t_w"][1] = 0                                     # a stage without weight work is fine

    def code(**change):
        a = {k: np.array(v) for k, v in good.items()}
        for name, (where, value) in change.items():
            a[name][where] = value
        prob, t_w = _zb_problem(b, S, N, a["t_f"], a["t_b"], a["t_w"], a["w"], a["cf"], a["cb"])
        return b.adaptra_zb_check_inputs(prob, t_w)

    assert code() == b.OK
    assert code(t_f=(2, 0)) == b.ERANGE                   # a forward that takes no time
    assert code(t_b=(0, 0)) == b.ERANGE
    assert code(t_w=(3, -1)) == b.ERANGE
    assert code(cf=((1, 2), -5)) == b.ERANGE
    assert code(cb=((0, 0), -1)) == b.ERANGE
    assert code(w=((2, 7), -1)) == b.ERANGE
    limit = 2 ** 31 // (3 * N * S)                         # 3 M S t reaches 2^31 at t = limit + 1 (2^31 has no factor 3)
    top = int(max(good["cf"].max(), good["cb"].max()))
    assert code(t_w=(0, limit - top)) == b.OK              # 3 M S (t + c) just below 2^31
    assert code(t_w=(0, limit - top + 1)) == b.EOVERFLOW
    assert code(t_b=(3, limit + 1)) == b.EOVERFLOW
    assert code(cf=((2, 5), limit + 1)) == b.EOVERFLOW
    # the F/B bound (2 M S) is the weaker one: adaptra_check_inputs accepts what this rejects
    a = {k: np.array(v) for k, v in good.items()}
    a["t_b"][3] = limit + 1
    prob, _ = _zb_problem(b, S, N, a["t_f"], a["t_b"], a["t_w"], a["w"], a["cf"], a["cb"])
    assert b.adaptra_check_inputs(prob) == b.OK


# ----------------------------------------------------------------------------------------
# Per-scenario stage times (computation stragglers) and link sensitivities
STAGE_TIME_CASES = [
    # seed, S, M, C, K, kwargs
    (60, 1, 9, 40, 70, dict(hist_bins=8, hist_shift=8)),
    (61, 2, 12, 100, 64, {}),
    (62, 3, 7, 90, 11, {}),                                    # general kernel only
    (63, 4, 16, 130, 129, dict(hist_bins=32, hist_shift=8)),
    (64, 8, 32, 300, 100, dict(d_max=6, hist_bins=64, hist_shift=10)),
    (65, 8, 90, 100, 64, dict(w_extra=50)),                    # deep warm-ups
    (66, 16, 48, 200, 65, dict(d_max=4)),
    (67, 32, 64, 80, 70, dict(d_max=4, hist_bins=16, hist_shift=12)),
    (68, 64, 80, 30, 5, dict(d_max=2)),
    (69, 8, 24, 50, 3, {}),                                    # few scenarios
    (59, 12, 30, 60, 40, dict(d_max=3, hist_bins=8, hist_shift=10)),   # padded to 16 stages
    (58, 24, 50, 30, 64, dict(d_max=3)),                       # padded to 32 stages
]


def _with_stage_times(binding, wl, tfs, tbs, mode, fn):
    import torch
    binding.adaptra_set_kernel_mode(mode)
    prob = binding.Problem.from_workload(wl, t_f_scen=tfs, t_b_scen=tbs)
    out = fn(prob)
    torch.cuda.synchronize()
    binding.adaptra_set_kernel_mode(0)
    return [None if t is None else t.cpu().numpy() for t in out]


@pytest.mark.parametrize("seed,S,M,C,K,kw", STAGE_TIME_CASES,
                         ids=[f"S{r[1]}_M{r[2]}_C{r[3]}_K{r[4]}" for r in STAGE_TIME_CASES])
def test_per_scenario_stage_times_parity(lib, oracle, seed, S, M, C, K, kw):
    wl = workloads.random_workload(seed, S, M, C, K, **kw)
    tfs, tbs = workloads.straggler_stage_times(seed + 1000, wl)
    assert (tfs != wl.t_f[:, None]).any()
    say(f"stage-time scenarios {wl.name}")
    ref = oracle.eval_scenario_times(S, M, tfs, tbs, wl.mem_cap, wl.w, wl.c_fwd, wl.c_bwd)
    rbest = oracle.best_from_eval(ref["makespan"], ref["flag"], ref["bubble"])
    rhist = oracle.hist_from_eval(ref["bubble"], ref["flag"], wl.hist_bins, wl.hist_shift) if wl.hist_bins else None
    for mode in (0, 1, 2, 3, 4):
        say(f"  eval mode {mode}")
        mk, bub, fl = _with_stage_times(lib, wl, tfs, tbs, mode, lambda p: lib.adaptra_eval(p))
        assert np.array_equal(fl, ref["flag"])
        assert np.array_equal(mk, ref["makespan"]), f"makespan mismatch mode {mode}"
        assert np.array_equal(bub, ref["bubble"]), f"bubble mismatch mode {mode}"
        say(f"  best mode {mode}")
        idx, bmk, bbub, hist = _with_stage_times(lib, wl, tfs, tbs, mode, lambda p: lib.adaptra_best(p))
        assert np.array_equal(idx, rbest["best_idx"]), f"best_idx mismatch mode {mode}"
        assert np.array_equal(bmk, rbest["best_makespan"])
        assert np.array_equal(bbub, rbest["best_bubble"])
        if rhist is not None:
            assert np.array_equal(hist.astype(np.uint64), rhist)


def test_per_scenario_stage_times_checked_and_seeded(lib, oracle):
    """adaptra_check_inputs scans the per-scenario times too, and adaptra_seed (Algorithm 2,
    Eq. (1)) uses them."""
    import torch
    from oracle import seed as oseed
    wl = workloads.random_workload(70, 6, 40, 20, 50)
    np.maximum(wl.w, 0, out=wl.w)                       # the generator plants negative w to test the clamp
    tfs, tbs = workloads.straggler_stage_times(71, wl, p_slow=0.4)
    prob = lib.Problem.from_workload(wl, t_f_scen=tfs, t_b_scen=tbs)
    assert lib.adaptra_check_inputs(prob) == lib.OK
    w_cur = torch.tensor(oseed.to_w(oseed.initial_plan(wl.S, 12)), dtype=torch.int32, device="cuda:0")
    w_init, w_ad, na = lib.adaptra_seed(prob, 12, w_current=w_cur, want_not_absorbed=True)
    torch.cuda.synchronize()
    w_ad, na = w_ad.cpu().numpy(), na.cpu().numpy()
    for k in range(wl.n_scen):
        x = oseed.adapted_plan(wl.S, wl.M, tfs[:, k], tbs[:, k], wl.c_fwd[:, k], wl.c_bwd[:, k])
        assert list(w_ad[:, k]) == oseed.to_w(x), k
        ab = oseed.absorbed(wl.S, tfs[:, k], tbs[:, k], w_cur.cpu().numpy(), wl.c_fwd[:, k], wl.c_bwd[:, k])
        assert list(na[:, k]) == [0 if a else 1 for a in ab], k
    bad = tfs.copy()
    bad[2, 7] = -1
    prob = lib.Problem.from_workload(wl, t_f_scen=bad, t_b_scen=tbs)
    assert lib.adaptra_check_inputs(prob) == lib.ERANGE
    half = lib.Problem.from_workload(wl, t_f_scen=tfs, t_b_scen=None)      # both or neither
    with pytest.raises(lib.AdaptraError) as e:
        lib.adaptra_eval(half)
    assert e.value.code == lib.EINVAL


SENS_CASES = [
    # seed, S, M, C, K, delta, stage times per scenario, kwargs
    (80, 1, 5, 10, 20, 3, False, {}),
    (81, 2, 10, 40, 64, 1, False, {}),
    (82, 3, 9, 30, 17, 25, False, {}),
    (83, 4, 16, 70, 65, 7, True, {}),
    (84, 8, 32, 40, 100, 100, False, dict(d_max=6)),
    (85, 8, 60, 16, 40, 1, True, dict(w_extra=30)),
    (86, 16, 40, 20, 30, 13, False, dict(d_max=3)),
    (87, 32, 64, 6, 70, 50, True, dict(d_max=3)),
    (88, 64, 70, 4, 9, 5, False, dict(d_max=2)),
    (89, 8, 24, 1, 1, 9, False, {}),
]


@pytest.mark.parametrize("seed,S,M,C,K,delta,vt,kw", SENS_CASES,
                         ids=[f"S{r[1]}_M{r[2]}_C{r[3]}_K{r[4]}" for r in SENS_CASES])
def test_sensitivity_parity(lib, oracle, seed, S, M, C, K, delta, vt, kw):
    wl = workloads.random_workload(seed, S, M, C, K, **kw)
    tfs, tbs = workloads.straggler_stage_times(seed + 1000, wl) if vt else (None, None)
    say(f"sensitivity {wl.name} delta {delta} stage-times {vt}")
    ref = oracle.sensitivity(S, M, wl.t_f, wl.t_b, wl.mem_cap, wl.w, wl.c_fwd, wl.c_bwd, delta,
                             t_f_scen=tfs, t_b_scen=tbs)
    assert ref["sens"].shape == (C, S - 1, K)
    for mode in (0, 1, 2, 3, 4):
        say(f"  mode {mode}")
        mk, fl, sens = _with_stage_times(lib, wl, tfs, tbs, mode, lambda p: lib.adaptra_sensitivity(p, delta))
        assert np.array_equal(fl, ref["flag"])
        assert np.array_equal(mk, ref["makespan"]), f"makespan mismatch mode {mode}"
        assert np.array_equal(sens, ref["sens"]), f"sensitivity mismatch mode {mode}"


def test_sensitivity_rejects_bad_arguments(lib):
    wl = workloads.random_workload(90, 4, 8, 5, 6)
    prob = lib.Problem.from_workload(wl)
    with pytest.raises(lib.AdaptraError) as e:
        lib.adaptra_sensitivity(prob, 0)
    assert e.value.code == lib.EINVAL
    import torch
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(lib.AdaptraError) as e:
        lib.adaptra_sensitivity(prob, 1, workspace=small)
    assert e.value.code == lib.EWORKSPACE


def test_sensitivity_full_size_sampled(lib, oracle):
    """Configuration 2's scenarios against a slice of its candidates, at the launch shape of a
    real call; the oracle recomputes sampled (candidate, link, scenario) entries one by one."""
    import torch
    wl = workloads.config(2)
    cand = np.arange(0, wl.n_cand, max(1, wl.n_cand // 64))[:64]
    sub = workloads.Workload(**{**wl.__dict__, "w": np.ascontiguousarray(wl.w[:, cand]), "name": wl.name + "-sens"})
    say(f"sensitivity {sub.name}: {sub.n_cand} candidates x {sub.n_scen} scenarios x {sub.S - 1} links")
    prob = lib.Problem.from_workload(sub)
    mk, fl, sens = lib.adaptra_sensitivity(prob, 10)
    torch.cuda.synchronize()
    mk, fl, sens = mk.cpu().numpy(), fl.cpu().numpy(), sens.cpu().numpy()
    rng = np.random.default_rng(5)
    ks = rng.integers(0, sub.n_scen, 48)
    ref = oracle.sensitivity(sub.S, sub.M, sub.t_f, sub.t_b, sub.mem_cap, sub.w,
                             sub.c_fwd[:, ks], sub.c_bwd[:, ks], 10)
    assert np.array_equal(mk[:, ks], ref["makespan"])
    assert np.array_equal(fl[:, ks], ref["flag"])
    assert np.array_equal(sens[:, :, ks], ref["sens"])
    live = (fl & 2) == 0
    assert (sens[np.broadcast_to(live[:, None, :], sens.shape)] >= 0).all()


# ----------------------------------------------------------------------------------------
# Guided search
SEARCH_CASES = [
    # seed, S, M, K, neighbourhood, max_iters, stage times per scenario, kwargs
    (100, 1, 6, 9, 0, 50, False, {}),
    (101, 2, 60, 7, 0, 50, False, dict(c_hi=60, cap=False)),
    (102, 3, 12, 5, 1, 50, False, {}),                     # general kernel (K < 6)
    (103, 4, 16, 70, 0, 50, False, {}),
    (104, 4, 16, 33, 1, 50, True, {}),
    (105, 8, 32, 64, 0, 50, False, dict(c_hi=3000)),
    (106, 8, 32, 20, 1, 4, False, dict(c_hi=3000)),        # stopped by max_iters
    (107, 16, 40, 12, 0, 50, True, dict(c_hi=2000, cap=False)),
    (108, 5, 20, 1100, 0, 50, False, {}),                  # many scenarios
    (109, 40, 50, 7, 0, 8, False, dict(cap=False)),        # the candidate-lanes kernel's 64-stage size
]


@pytest.mark.parametrize("seed,S,M,K,nb,iters,vt,kw", SEARCH_CASES,
                         ids=[f"S{r[1]}_M{r[2]}_K{r[3]}_nb{r[4]}" for r in SEARCH_CASES])
def test_guided_search_parity(lib, oracle, seed, S, M, K, nb, iters, vt, kw):
    import torch
    from oracle import search as osearch
    wl = workloads.random_workload(seed, S, M, 4, K, **kw)
    tfs, tbs = workloads.straggler_stage_times(seed + 1000, wl) if vt else (None, None)
    start = np.arange(S - 1, -1, -1, dtype=np.int32)        # plain 1F1B
    cap = None if wl.mem_cap is None else np.maximum(wl.mem_cap, start + 1).astype(np.int32)
    wl.mem_cap = cap
    say(f"search {wl.name} neighbourhood {nb}")
    ref = osearch.search(S, M, wl.t_f, wl.t_b, cap, start, wl.c_fwd, wl.c_bwd, neighbourhood=nb,
                         max_iters=iters, t_f_scen=tfs, t_b_scen=tbs)
    for mode in (0, 1, 3, 4):                               # automatic, general kernel, candidate lanes plain / read-ahead
        lib.adaptra_set_kernel_mode(mode)
        prob = lib.Problem.from_workload(wl, t_f_scen=tfs, t_b_scen=tbs)
        w, mk, rounds, evaluated = lib.adaptra_search(prob, torch.from_numpy(start).cuda(), nb, iters)
        lib.adaptra_set_kernel_mode(0)
        assert rounds == ref["rounds"], f"mode {mode}"
        # The GPU path does not evaluate a scenario again once it has come to rest (its pool
        # would be the same in every later round), the oracle keeps evaluating all of them.  A
        # move is a strict improvement, so the scenarios that moved in round r are those whose
        # makespan differs between rounds r - 1 and r of the oracle's trajectory; round r + 1
        # evaluates exactly those.
        hist = np.concatenate([np.full((1, K), INT32_MAX, dtype=np.int64), ref["makespan_history"].astype(np.int64)])
        moved = (hist[1:] != hist[:-1]).sum(axis=1)
        still_moving = [K] + list(moved[:-1]) if S > 1 and M > 1 else [K] * ref["rounds"]
        assert evaluated == sum(still_moving[:ref["rounds"]]) * (len(osearch.moves(S, nb)) + 1)
        assert np.array_equal(mk.cpu().numpy(), ref["makespan"])
        assert np.array_equal(w.cpu().numpy(), ref["w"])


def test_guided_search_arguments(lib):
    import torch
    wl = workloads.random_workload(110, 4, 8, 3, 6)
    prob = lib.Problem.from_workload(wl)
    start = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    for bad in (dict(neighbourhood=2), dict(max_iters=0)):
        with pytest.raises(lib.AdaptraError) as e:
            lib.adaptra_search(prob, start, **bad)
        assert e.value.code == lib.EINVAL
    with pytest.raises(lib.AdaptraError) as e:
        lib.adaptra_search(prob, start, workspace=torch.empty(512, dtype=torch.uint8, device="cuda:0"))
    assert e.value.code == lib.EWORKSPACE


@pytest.mark.parametrize("index", [1, 2])
def test_guided_search_against_exhaustive_argmin(lib, oracle, index):
    """Configurations 1 and 2: the search, started from Algorithm 1's plan under the
    configuration's memory caps, against adaptra_best over the configuration's own candidate
    set.  The search looks at vectors outside that set too, so it may win; what must hold is
    that every point it returns is feasible and priced exactly as the oracle prices it, and
    that it does not lose by much where the candidate set contains the optimum."""
    import torch
    from oracle import seed as oseed
    wl = workloads.config(index)
    S, M, K = wl.S, wl.M, wl.n_scen
    x_max = int(wl.mem_cap[0]) if wl.mem_cap is not None else S
    start = np.array(oseed.to_w(oseed.initial_plan(S, x_max)), dtype=np.int32)
    prob = lib.Problem.from_workload(wl)
    idx, bmk, _, _ = lib.adaptra_best(prob)
    w, mk, rounds, evaluated = lib.adaptra_search(prob, torch.from_numpy(start).cuda(), 1, 200)
    torch.cuda.synchronize()
    w, mk, bmk = w.cpu().numpy(), mk.cpu().numpy().astype(np.int64), bmk.cpu().numpy().astype(np.int64)
    say(f"  config {index}: {rounds} rounds, {evaluated} pairs; search/best makespan ratio "
        f"mean {np.mean(mk / bmk):.4f} max {np.max(mk / bmk):.4f}; search wins {int((mk < bmk).sum())}/{K}")
    ref = oracle.eval_pairs(S, M, wl.t_f, wl.t_b, wl.mem_cap, w, wl.c_fwd, wl.c_bwd,
                            pair_cand=np.arange(K), pair_scen=np.arange(K), want_bubble=False)
    assert np.all(ref["flag"] == 1)
    assert np.array_equal(ref["makespan"].astype(np.int64), mk)
    assert np.max(mk / bmk) < 1.05


# ----------------------------------------------------------------------------------------
def test_eval_and_best_replay_from_a_hip_graph(lib, oracle):
    """The entry points only enqueue kernels (no allocation, no memset node, no host wait), so a
    caller may capture them into a HIP graph.  The graph is replayed several times, with eager
    work and synchronisations of the same library between the replays and with the inputs
    changed in place, and every replay is checked against the oracle."""
    import torch
    wl = workloads.random_workload(120, 8, 24, 300, 70, hist_bins=16, hist_shift=9)
    prob = lib.Problem.from_workload(wl, w_bound=int(np.clip(wl.w, 0, wl.M - 1).max()))
    ws = lib.alloc_workspace(prob)
    dev = prob.device
    mk = torch.empty((prob.K, prob.C), dtype=torch.int32, device=dev)
    bub = torch.empty((prob.S, prob.K, prob.C), dtype=torch.int32, device=dev)
    fl = torch.empty((prob.K, prob.C), dtype=torch.uint8, device=dev)
    bidx = torch.empty(prob.K, dtype=torch.int32, device=dev)
    bmk = torch.empty(prob.K, dtype=torch.int32, device=dev)
    bbub = torch.empty((prob.K, prob.S), dtype=torch.int32, device=dev)
    hist = torch.empty((prob.S, prob.hist_bins), dtype=torch.int64, device=dev)

    def enqueue():
        lib.adaptra_eval(prob, mk, bub, fl, workspace=ws)
        lib.adaptra_best(prob, bidx, bmk, bbub, hist, workspace=ws)

    enqueue()                                   # eager warm-up (sets the kernels' LDS attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            enqueue()
    torch.cuda.synchronize()
    c_fwd_dev = prob.tensors[3]
    for replay in range(4):
        say(f"  replay {replay}")
        if replay:                              # new delays, written in place, and eager work in between
            wl.c_fwd[:] = (wl.c_fwd.astype(np.int64) * (replay + 1) % 4001).astype(np.int32)
            c_fwd_dev.copy_(torch.from_numpy(wl.c_fwd))
            other = workloads.random_workload(121 + replay, 4, 8, 50, 64)
            gpu_eval(lib, other)
        for t in (mk, bub, bmk, bidx):
            t.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.eval_workload(wl)
        rbest = oracle.best_from_eval(ref["makespan"], ref["flag"], ref["bubble"])
        assert np.array_equal(mk.cpu().numpy(), ref["makespan"])
        assert np.array_equal(bub.cpu().numpy(), ref["bubble"])
        assert np.array_equal(fl.cpu().numpy(), ref["flag"])
        assert np.array_equal(bidx.cpu().numpy(), rbest["best_idx"])
        assert np.array_equal(bmk.cpu().numpy(), rbest["best_makespan"])
        assert np.array_equal(bbub.cpu().numpy(), rbest["best_bubble"])
        assert np.array_equal(hist.cpu().numpy().astype(np.uint64),
                              oracle.hist_from_eval(ref["bubble"], ref["flag"], wl.hist_bins, wl.hist_shift))


def test_other_entry_points_replay_from_a_hip_graph(lib):
    """adaptra_eval_best, adaptra_seed and adaptra_sensitivity captured into one HIP graph: every
    replay, after the inputs changed in place, equals what the same calls return eagerly (the
    eager paths are checked against the oracle by the tests above)."""
    import torch
    wl = workloads.random_workload(140, 8, 20, 200, 70, hist_bins=8, hist_shift=10)
    prob = lib.Problem.from_workload(wl, w_bound=int(np.clip(wl.w, 0, wl.M - 1).max()))
    w_cur = torch.from_numpy(np.arange(wl.S - 1, -1, -1, dtype=np.int32)).cuda()

    def enqueue():
        return (lib.adaptra_eval_best(prob), lib.adaptra_seed(prob, x_max=6, w_current=w_cur, want_not_absorbed=True),
                lib.adaptra_sensitivity(prob, 3))

    def flat(out):
        return [t.cpu().numpy().copy() for group in out for t in group if t is not None]

    enqueue()                                   # eager warm-up (sets the kernels' LDS attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            captured = enqueue()
    torch.cuda.synchronize()
    c_bwd_dev = prob.tensors[4]
    for replay in range(3):
        say(f"  replay {replay}")
        if replay:
            wl.c_bwd[:] = (wl.c_bwd.astype(np.int64) * (replay + 3) % 2999).astype(np.int32)
            c_bwd_dev.copy_(torch.from_numpy(wl.c_bwd))
        eager = enqueue()
        torch.cuda.synchronize()
        want = flat(eager)
        for group in captured:
            for t in group:
                if t is not None:
                    t.fill_(0)
        graph.replay()
        torch.cuda.synchronize()
        got = flat(captured)
        assert len(got) == len(want)
        for i, (g, w) in enumerate(zip(got, want)):
            assert np.array_equal(g, w), (replay, i)


def test_zb_replays_from_a_hip_graph(lib, oracle):
    """adaptra_zb_eval draws its work units from a counter in the workspace, reset by a kernel of
    the same call: captured into a HIP graph (policy and fixed plans), every replay starts from
    that reset.  Replayed with the delays changed in place and eager calls in between."""
    import torch
    b = lib
    rng = np.random.default_rng(130)
    S, N, C, K = 8, 16, 150, 33
    t_f, t_b, t_w = rng.integers(1, 60, S), rng.integers(1, 90, S), rng.integers(0, 50, S)
    w = np.sort(rng.integers(0, N, (S, C)), axis=0)[::-1]
    cf = rng.integers(0, 400, (S - 1, K)).astype(np.int32)
    cb = rng.integers(0, 400, (S - 1, K)).astype(np.int32)
    prob, t_w_d = _zb_problem(b, S, N, t_f, t_b, t_w, w, cf, cb)
    x = np.clip(w, 0, N - 1) + 1
    n = int(b.load().adaptra_zb_workspace_bytes(__import__("ctypes").byref(prob.params), prob.C, prob.K))
    ws = torch.empty(n, dtype=torch.uint8, device=prob.device)
    b.adaptra_zb_eval(prob, t_w_d, -1, workspace=ws)          # eager warm-up
    b.adaptra_zb_eval(prob, t_w_d, 2, workspace=ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            mk, bub = b.adaptra_zb_eval(prob, t_w_d, -1, workspace=ws)
            mkp, _ = b.adaptra_zb_eval(prob, t_w_d, 2, want_bubble=False, workspace=ws)
    torch.cuda.synchronize()
    c_fwd_dev = prob.tensors[3]
    for replay in range(3):
        say(f"  replay {replay}")
        if replay:
            cf[:] = (cf.astype(np.int64) * (replay + 2) % 997).astype(np.int32)
            c_fwd_dev.copy_(torch.from_numpy(cf))
            b.adaptra_zb_eval(prob, t_w_d, 0)                 # eager work of the same library in between
        mk.fill_(-7)
        mkp.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.zb_batch(S, N, t_f, t_b, t_w, x, cf, cb)
        assert np.array_equal(mk.cpu().numpy(), ref["makespan"])
        assert np.array_equal(bub.cpu().numpy(), ref["idle"])
        got = mkp.cpu().numpy()
        for c in range(0, C, 13):
            gen = oracle.zb_simulate(S, N, t_f, t_b, t_w, cf[:, 2], cb[:, 2], x=x[:, c])
            for k in (0, 2, K - 1):
                rep = oracle.zb_simulate(S, N, t_f, t_b, t_w, cf[:, k], cb[:, k], order=gen["order"])
                assert got[k, c] == rep["makespan"], (replay, c, k)


def test_many_small_random_problems(lib, oracle):
    """A sweep of small random shapes (every stage count from 1 to 20, M from 1, ragged C and
    K, with and without caps, histograms and per-scenario stage times) in every kernel mode."""
    rng = np.random.default_rng(2025)
    for trial in range(120):
        S = int(rng.integers(1, 21))
        M = int(rng.integers(1, 14))
        C = int(rng.integers(1, 140))
        K = int(rng.integers(1, 80))
        kw = dict(d_max=int(rng.integers(0, 4)), cap=bool(rng.integers(0, 2)))
        if rng.integers(0, 2):
            kw.update(hist_bins=int(rng.integers(1, 40)), hist_shift=int(rng.integers(0, 12)))
        wl = workloads.random_workload(5000 + trial, S, M, C, K, **kw)
        vt = bool(rng.integers(0, 3) == 0)
        tfs, tbs = workloads.straggler_stage_times(6000 + trial, wl, p_slow=0.3) if vt else (None, None)
        if vt:
            ref = oracle.eval_scenario_times(S, M, tfs, tbs, wl.mem_cap, wl.w, wl.c_fwd, wl.c_bwd)
        else:
            ref = oracle.eval_workload(wl)
        rbest = oracle.best_from_eval(ref["makespan"], ref["flag"], ref["bubble"])
        rhist = oracle.hist_from_eval(ref["bubble"], ref["flag"], wl.hist_bins, wl.hist_shift) if wl.hist_bins else None
        for mode in (0, 1, 2, 3, 4):
            tag = f"trial {trial} {wl.name} stage-times {vt} mode {mode}"
            mk, bub, fl = _with_stage_times(lib, wl, tfs, tbs, mode, lambda p: lib.adaptra_eval(p))
            assert np.array_equal(fl, ref["flag"]), tag
            assert np.array_equal(mk, ref["makespan"]), tag
            assert np.array_equal(bub, ref["bubble"]), tag
            idx, bmk, bbub, hist = _with_stage_times(lib, wl, tfs, tbs, mode, lambda p: lib.adaptra_best(p))
            assert np.array_equal(idx, rbest["best_idx"]), tag
            assert np.array_equal(bmk, rbest["best_makespan"]), tag
            assert np.array_equal(bbub, rbest["best_bubble"]), tag
            if rhist is not None:
                assert np.array_equal(hist.astype(np.uint64), rhist), tag


def test_readme_example_runs(lib):
    import torch
    from paper_2504_19232_amd import binding
    wl = workloads.config(1)
    prob = binding.Problem.from_workload(wl)
    mk, bubble, flag, best_idx, best_mk, best_bubble, hist = binding.adaptra_eval_best(prob)
    w_init, w_adapted, _ = binding.adaptra_seed(prob, x_max=8)
    w, makespan, rounds, pairs = binding.adaptra_search(prob, w_init, neighbourhood=1)
    torch.cuda.synchronize()
    assert mk.shape == (wl.n_scen, wl.n_cand) and w.shape == (wl.S, wl.n_scen) and rounds >= 1
    per_scenario = wl.S * (wl.S + 1) + 1                    # the point and its range moves
    assert wl.n_scen * per_scenario <= pairs <= rounds * wl.n_scen * per_scenario
