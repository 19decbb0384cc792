"""Host-side logic that needs no GPU: the benchmark's one-GPU guard and the
seeded workload generators."""
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert run.returncode != 0
    assert "ONE GPU" in run.stderr and run.stdout.strip() == ""


def test_workloads_are_seeded_and_well_formed():
    from workloads import configs
    for name in ("tiny", "arxiv_small", "rmat12", "reddit_small"):
        a, b = configs.make(name), configs.make(name)
        for k in ("rowptr", "colidx", "val", "X"):
            assert np.array_equal(a[k].numpy(), b[k].numpy()), (name, k)
        rowptr, col = a["rowptr"].numpy(), a["colidx"].numpy()
        w = a["workload"]
        assert rowptr[0] == 0 and rowptr[-1] == col.size and np.all(np.diff(rowptr) >= 0)
        assert col.min() >= 0 and col.max() < w.n
        row = np.repeat(np.arange(w.n), np.diff(rowptr))
        key = row.astype(np.int64) * w.n + col
        assert np.all(np.diff(key) > 0)                       # rows ascending, no duplicate entry
        if w.self_loops:
            assert np.all(np.isin(np.arange(w.n, dtype=np.int64) * (w.n + 1), key))
        if w.norm == "row":                                   # rows sum to one
            sums = np.add.reduceat(a["val"].numpy().astype(np.float64), rowptr[:-1][np.diff(rowptr) > 0])
            assert np.allclose(sums, 1.0, atol=1e-5)
        if w.kind != "rmat":                                  # undirected wiring is symmetric
            assert np.array_equal(np.sort(col.astype(np.int64) * w.n + row), key)


def test_counter_based_rng_is_position_addressable():
    import torch
    from workloads import rng
    whole = rng.uniform(5, 2, 1000, torch.device("cpu"))
    part = rng.uniform(5, 2, 300, torch.device("cpu"), start=200)
    assert torch.equal(whole[200:500], part)
    assert 0.0 <= float(whole.min()) and float(whole.max()) < 1.0
    assert abs(float(whole.mean()) - 0.5) < 0.05
    p = rng.permutation(1, 3, 257, torch.device("cpu"))
    assert sorted(p.tolist()) == list(range(257))
