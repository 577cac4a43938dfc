"""The synthetic input generators: deterministic, distinct coordinates, stated recipe."""
import numpy as np
import torch

import workloads as w
from workloads import rng


def test_rng_is_counter_based_and_split_invariant():
    a = rng.bits64(7, "s", 0, 100)
    b = torch.cat([rng.bits64(7, "s", 0, 37), rng.bits64(7, "s", 37, 63)])
    assert torch.equal(a, b)
    assert not torch.equal(a, rng.bits64(8, "s", 0, 100))
    assert not torch.equal(a, rng.bits64(7, "t", 0, 100))
    u = rng.uniform01(1, "u", 0, 200000)
    assert 0.0 <= float(u.min()) and float(u.max()) < 1.0
    assert abs(float(u.mean()) - 0.5) < 5e-3
    g = rng.normal(1, "g", 0, 200000)
    assert abs(float(g.mean())) < 1e-2 and abs(float(g.std()) - 1.0) < 1e-2
    p = rng.permutation(3, "p", 1000)
    assert sorted(p.tolist()) == list(range(1000))


def test_splitmix64_first_word_matches_integer_arithmetic():
    # the same finaliser evaluated with Python integers
    key = rng.stream_key(5, "x")
    z = (3 * rng._GOLDEN + key) & rng._MASK64
    want = rng._mix_int(z)
    got = int(rng.bits64(5, "x", 3, 1)[0]) & rng._MASK64
    assert got == want


def test_small_configs_are_distinct_and_in_range_and_repeatable():
    for cid in (1, 2, 3, 4, 5):
        a = w.make(cid, small=True)
        b = w.make(cid, small=True)
        for name, X in a.sparse.items():
            key = torch.zeros(X.nnz, dtype=torch.int64)
            for m, d in enumerate(X.dims):
                c = X.coords[m].long()
                assert int(c.min()) >= 0 and int(c.max()) < d
                key = key * d + c
            assert torch.unique(key).numel() == X.nnz
            assert bool((X.vals != 0).all())
            assert all(torch.equal(x, y) for x, y in zip(X.coords, b.sparse[name].coords))
            assert torch.equal(X.vals, b.sparse[name].vals)
        for name, F in a.dense.items():
            assert torch.equal(F, b.dense[name])


def test_zipf_skew_and_dense_mode0():
    c2 = w.make(2, small=True)
    cnt = torch.bincount(c2.sparse["X"].coords[0].long())
    assert cnt.max() > 20 * cnt[cnt > 0].float().median()          # power-law slices
    c3 = w.make(3, small=True)
    X = c3.sparse["X"]
    assert torch.unique(X.coords[0]).numel() == X.dims[0]         # every mode-0 index present
    c4 = w.make(4, small=True)
    U = c4.sparse["U"]
    assert U.nnz == 6 * (60 // 4) * (80 // 4) * (40 // 4)
