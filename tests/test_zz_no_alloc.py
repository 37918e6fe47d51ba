"""adaptra_best_static -- the entry point that allocates nothing, its scratch in a fixed device
array inside the library -- against adaptra_best (caller's workspace) through the C ABI.
Bit-exact (integers).  Two calls in a row on the same GPU, the second with a smaller input, so
that what the first call left in the shared array must not leak into the second."""
import sys

import numpy as np
import pytest

from paper_2504_19232_amd import workloads

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _outputs(torch, prob, fill):
    dev = prob.device
    idx = torch.full((prob.K,), fill, dtype=torch.int32, device=dev)
    mk = torch.full((prob.K,), fill, dtype=torch.int32, device=dev)
    bub = torch.full((prob.K, prob.S), fill, dtype=torch.int32, device=dev)
    hist = torch.full((prob.S, prob.hist_bins), fill, dtype=torch.int64, device=dev) if prob.hist_bins else None
    return idx, mk, bub, hist


def _compare(torch, binding, wl, w_bound=-1):
    prob = binding.Problem.from_workload(wl, w_bound=w_bound)
    want = _outputs(torch, prob, -7)
    binding.adaptra_best(prob, *want)
    got = _outputs(torch, prob, -9)
    binding.adaptra_best_static(prob, *got)
    torch.cuda.synchronize()
    for name, g, w in zip(("best_idx", "best_makespan", "best_bubble", "hist"), got, want):
        if w is None:
            continue
        assert np.array_equal(g.cpu().numpy(), w.cpu().numpy()), f"{wl.name}: {name} differs"
    return [None if t is None else t.cpu().numpy() for t in got]


def test_static_entry_point_matches_the_workspace_one_twice_in_a_row():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2504_19232_amd import binding
    binding.load()
    binding.adaptra_set_kernel_mode(0)
    # first call: a slice of configuration 3 (S=32, M=128) with caps and a histogram, scenario-lanes kernel
    big = workloads.config(3)
    big.w = np.ascontiguousarray(big.w[:, :4096])
    big.c_fwd = np.ascontiguousarray(big.c_fwd[:, :256])
    big.c_bwd = np.ascontiguousarray(big.c_bwd[:, :256])
    big.hist_bins, big.hist_shift = 64, 12
    say(f"static entry point, first call: {big.S} stages, {big.M} micro-batches, {big.n_cand} x {big.n_scen}")
    first = _compare(torch, binding, big, w_bound=int(big.w.max()))
    assert (first[0] >= 0).any()
    # second call, smaller in every dimension: fewer stages, candidates, scenarios (candidate-lanes
    # kernel), deep warm-ups so that some candidates go to the general kernel's share of the scratch
    small = workloads.random_workload(71, S=5, M=40, C=300, K=9, w_extra=30, hist_bins=16, hist_shift=7)
    say(f"static entry point, second call: {small.S} stages, {small.M} micro-batches, {small.n_cand} x {small.n_scen}")
    _compare(torch, binding, small)
    # and a third that only the general kernel can take (warm-ups deeper than the LDS ring)
    deep = workloads.random_workload(72, S=4, M=400, C=40, K=64, w_extra=300)
    say(f"static entry point, third call: {deep.S} stages, {deep.M} micro-batches, {deep.n_cand} x {deep.n_scen}")
    _compare(torch, binding, deep)


def test_static_entry_point_limits():
    import torch
    from paper_2504_19232_amd import binding
    wl = workloads.random_workload(73, S=4, M=1025, C=10, K=3)
    prob = binding.Problem.from_workload(wl)
    outs = _outputs(torch, prob, 0)
    with pytest.raises(binding.AdaptraError) as e:
        binding.adaptra_best_static(prob, *outs)
    assert e.value.code == binding.ELIMIT
    torch.cuda.synchronize()
