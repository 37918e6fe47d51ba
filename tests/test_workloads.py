"""Host-side checks of the seeded input generators and of the stored oracle outputs."""
import os

import numpy as np

from paper_2504_19232_amd import workloads

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_shapes_dtypes_and_determinism():
    sizes = [(4, 8, 64, 21), (8, 32, 16384, 64), (16, 64, 1 << 18, 256), (32, 128, 1 << 16, 1024),
             (8, 256, 1 << 20, 64)]
    for i, (S, M, C, K) in enumerate(sizes):
        wl = workloads.config(i)
        assert (wl.S, wl.M, wl.n_cand, wl.n_scen) == (S, M, C, K)
        assert wl.w.shape == (S, C) and wl.w.dtype == np.int32 and wl.w.flags.c_contiguous
        assert wl.c_fwd.shape == (S - 1, K) and wl.c_bwd.shape == (S - 1, K)
        assert wl.t_f.shape == (S,) and wl.t_b.shape == (S,)
        assert wl.t_f.min() > 0 and wl.c_fwd.min() >= 0 and wl.c_bwd.min() >= 0
        assert np.all(wl.w[S - 1] == 0)
        # the int32 precondition of the library: 2 M S (max t + max c) < 2^31
        bound = 2 * M * S * (int(max(wl.t_f.max(), wl.t_b.max())) + int(max(wl.c_fwd.max(), wl.c_bwd.max())))
        assert bound < 2 ** 31
        if i < 3:
            assert workloads.config(i).sha256() == wl.sha256()


def test_stored_input_hashes():
    want = {}
    with open(os.path.join(GOLDEN, "workload_sha256.txt")) as f:
        for line in f:
            i, _, h = line.split()
            want[int(i)] = h
    for i in range(5):
        assert workloads.config(i).sha256() == want[i]


def test_candidate_sets_have_the_documented_structure():
    wl = workloads.config(0)
    d = wl.w - workloads.default_warmup(4)[:, None]
    assert d[:3].min() == 0 and d[:3].max() == 3
    c = np.arange(64)
    for s in range(3):
        assert np.array_equal(d[s], (c // 4 ** s) % 4)
    wl = workloads.config(2)
    fixed = (np.arange(wl.n_cand) % 8) != 0
    w = wl.w.astype(np.int64)
    assert np.all(w[:-1, fixed] >= w[1:, fixed])            # repaired vectors are non-increasing
    d = w - workloads.default_warmup(wl.S)[:, None]
    assert d.min() == 0 and d.max() == 4
    assert not np.all(np.all(w[:-1, ~fixed] >= w[1:, ~fixed], axis=0))   # raw ones mostly are not


def test_cfg0_oracle_outputs_match_stored(oracle):
    wl = workloads.config(0)
    r = oracle.eval_workload(wl, threads=2)
    n = 0
    with open(os.path.join(GOLDEN, "cfg0_oracle.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            v = [int(x) for x in line.split()]
            k, c = v[0], v[1]
            assert r["makespan"][k, c] == v[2] and r["flag"][k, c] == v[3]
            assert list(r["bubble"][:, k, c]) == v[4:]
            n += 1
    assert n == 3 * 64
