"""Seeded random cases for the tuned kernels (order-3 MTTKRP, order-3 and order-4 TTMc) against the
CPU oracle: extents from 2 upwards, a few to tens of thousands of nonzeros, ranks on both sides of
every kernel choice, compact or full output, and plan options drawn from the values each option
takes, so that partitions of one leaf per item, one row per item, one cost unit per batch and every
split of the wavefronts are met.  Each case prints its recipe before it runs."""
import numpy as np
import pytest
import torch

import paper_2401_04836_amd as cst
import workloads as w
from helpers import TOL, compare, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def _pick(rng, values):
    return int(values[int(rng.integers(len(values)))])


def _recipe(seed):
    rng = np.random.default_rng(7000 + seed)
    kind = ("mttkrp3", "ttmc3", "ttmc4")[seed % 3]
    order = 4 if kind == "ttmc4" else 3
    scale = _pick(rng, [0, 1, 2])
    dims = tuple(_pick(rng, ([2, 3, 5], [9, 20, 41], [60, 150, 301])[scale]) for _ in range(order))
    cells = int(np.prod(dims))
    nnz = max(1, min(cells // 3, _pick(rng, ([1, 4, 30], [50, 700, 3000], [9000, 30011])[scale])))
    opts = {}
    if kind == "mttkrp3":
        cid, kw = 2, dict(rank=_pick(rng, [1, 2, 5, 16, 32, 32, 32, 33, 64, 100, 128]))
        for name, values in (("mttkrp_dual", [0, 35, 44, 53, 88]), ("mttkrp_split", [0, 1]), ("mttkrp_hot", [1, 16, 256, 608]),
                             ("mttkrp_chunk", [0, 16, 100])):
            if rng.integers(2):
                opts[name] = _pick(rng, values)
    elif kind == "ttmc3":
        if rng.integers(2):
            ranks = (_pick(rng, [16, 32, 48, 64]), _pick(rng, [16, 32, 48, 64]))
        else:
            ranks = (_pick(rng, [1, 3, 8, 17, 50, 64]), _pick(rng, [1, 2, 8, 33, 64]))
        cid, kw = 5, dict(ranks=ranks)
        for name, values in (("ttmc3_mfma", [0, 1]), ("ttmc3_stream", [0, 1]), ("ttmc3_producers", [2, 3, 4, 6, 8]),
                             ("ttmc3_batch", [1, 16, 2048]), ("ttmc3_itemcost", [0, 2, 50]), ("ttmc3_qn", [1, 2, 4]),
                             ("ttmc3_split", [3, 64, 4096]), ("ttmc3_rowsplit", [1, 3, 64])):
            if rng.integers(2):
                opts[name] = _pick(rng, values)
    else:
        ranks = (16, 16, 16) if rng.integers(2) else (_pick(rng, [1, 4, 16]), _pick(rng, [2, 7, 16]), _pick(rng, [3, 16]))
        cid, kw = 3, dict(ranks=ranks)
        for name, values in (("ttmc4_mfma", [0, 1]), ("ttmc4_split", [1, 5, 256]), ("ttmc4_ksplit", [1, 3, 128])):
            if rng.integers(2):
                opts[name] = _pick(rng, values)
    flags = cst.OUT_COMPACT if rng.integers(2) else 0
    return cid, dims, nnz, kw, opts, flags


@pytest.mark.parametrize("seed", range(240))
def test_random_tuned_case(seed):
    cid, dims, nnz, kw, opts, flags = _recipe(seed)
    print("[case] seed %d: config-%d recipe dims %s nnz %d %s options %s compact %d" % (seed, cid, dims, nnz, kw, opts, flags != 0),
          flush=True)
    wl = w.make(cid, small=True, dims=dims, nnz=nnz, **kw)
    out, pl, _ = run_gpu(wl, flags=flags, options=opts or None)
    print("       " + pl.describe().split("|")[0], flush=True)
    want, S_abs = run_oracle(wl)
    rows = pl.output_rows() if flags else None
    err = compare(out, want, S_abs, rows=rows)
    print("       rel err %.3e" % err, flush=True)
    assert err <= TOL
