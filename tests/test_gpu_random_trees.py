"""Seeded random contraction chains on the GPU against the N-ary reference (Sec. 2.1): tensors of
order 2 to 5 with extents from 1 upwards, 0 to a few thousand nonzeros, one or two dense indices
of any extent, MTTKRP- and TTMc-shaped chains over the CSF levels from the leaves up, factor
layouts in either index order, every fusion the schedule allows or none, and long sums cut into
segments of a random length.  Each case prints its recipe before it runs."""
import numpy as np
import pytest
import torch

import oracle
from oracle import nary
import paper_2401_04836_amd as cst
from helpers import TOL

pytestmark = pytest.mark.gpu

LEVELS = "ijklm"


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    order = int(rng.integers(2, 6))
    dims = tuple(int(rng.choice([1, 2, 3, 5, 9, 17, 40])) for _ in range(order))
    cells = int(np.prod(dims))
    nnz = int(min(cells, rng.choice([0, 1, 2, 7, 60, 700, 4000])))
    flat = rng.choice(cells, size=nnz, replace=False) if nnz else np.zeros(0, dtype=np.int64)
    coords = []
    for d in reversed(dims):
        coords.append((flat % d).astype(np.int32))
        flat = flat // d
    coords.reverse()
    if nnz > 8 and rng.integers(2):                      # one crowded root slice
        coords[0][: nnz // 2] = coords[0][0]
        key = np.zeros(nnz, dtype=np.int64)
        for c, d in zip(coords, dims):
            key = key * d + c
        _, first = np.unique(key, return_index=True)
        coords = [c[first] for c in coords]
        nnz = len(first)
    vals = rng.standard_normal(nnz)
    kind = "mttkrp" if rng.integers(3) else "ttmc"
    n_dense = 1 if kind == "mttkrp" and rng.integers(3) else 2
    if kind == "ttmc":                                   # the reference holds nnz x (product of ranks) doubles at a time
        R = [int(rng.choice([1, 2, 3, 8] if order > 3 else [1, 2, 3, 8, 19])) for _ in range(order - 1)]
        if order > 3 and nnz > 700:
            coords, vals, nnz = [c[:700] for c in coords], vals[:700], 700
    else:
        R = [int(rng.choice([1, 2, 3, 8, 19, 33])) for _ in range(n_dense)]
    return rng, order, dims, coords, vals, kind, R


def _build(rng, order, dims, kind, R):
    """Schedule text, dense operands [(name, letters, array)] in statement order, result letters and extents."""
    lv = LEVELS[:order]
    ops, stmts, extents = [], [], {}
    if kind == "mttkrp":
        dense = "rs"[: len(R)]
        for c, e in zip(dense, R):
            extents[c] = e
        cur, cur_idx = "X", list(lv)
        for step, L in enumerate(range(order - 1, 0, -1)):
            name = "F%d" % L
            letters = [lv[L]] + list(dense)
            if rng.integers(2):
                letters = letters[::-1]
            ops.append((name, "".join(letters), rng.uniform(-1, 1, [dims[L] if c == lv[L] else extents[c] for c in letters])))
            out_dense = list(dense) if rng.integers(2) else list(dense)[::-1]
            out_idx = list(lv[:L]) + out_dense
            res = "M" if L == 1 else "T%d" % step
            loops = list(lv[: L + 1]) + out_dense
            stmts.append("%s[%s] = %s[%s] * %s[%s] | %s" % (res, ",".join(out_idx), cur, ",".join(cur_idx), name,
                                                             ",".join(letters), ",".join(loops)))
            cur, cur_idx = res, out_idx
        return " ; ".join(stmts), ops, "".join(cur_idx), extents
    # TTMc: level L gets its own dense index; the result keeps all of them, innermost level's last
    names = "abcd"
    cur, cur_idx, kept = "X", list(lv), []
    for step, L in enumerate(range(order - 1, 0, -1)):
        d = names[L - 1]
        extents[d] = R[L - 1]
        name = "U%d" % L
        letters = [lv[L], d] if rng.integers(2) else [d, lv[L]]
        ops.append((name, "".join(letters), rng.uniform(-1, 1, [dims[L] if c == lv[L] else extents[c] for c in letters])))
        kept = [d] + kept
        out_idx = list(lv[:L]) + kept
        res = "Y" if L == 1 else "T%d" % step
        loops = list(lv[: L + 1]) + kept
        stmts.append("%s[%s] = %s[%s] * %s[%s] | %s" % (res, ",".join(out_idx), cur, ",".join(cur_idx), name,
                                                         ",".join(letters), ",".join(loops)))
        cur, cur_idx = res, out_idx
    return " ; ".join(stmts), ops, "".join(cur_idx), extents


@pytest.mark.parametrize("seed", range(160))
def test_random_chain(seed):
    rng, order, dims, coords, vals, kind, R = _case(seed)
    text, ops, out_idx, extents = _build(rng, order, dims, kind, R)
    extents[LEVELS[0]] = dims[0]
    fusion = None if rng.integers(3) else [0] * (order - 1)
    options = ["force_generic=1"] if rng.integers(4) else []
    if rng.integers(2):
        options.append("generic_span=%d" % int(rng.choice([1, 3, 16, 200])))
    options = ",".join(options) or None
    print("[case] seed %d: order %d dims %s nnz %d %s ranks %s fusion %s options %s\n       %s"
          % (seed, order, dims, len(vals), kind, R, fusion, options, text), flush=True)
    csf = cst.build_csf([torch.from_numpy(c).cuda() for c in coords], torch.from_numpy(vals).cuda(), dims, list(range(order)))
    csf.check()
    dev = [(n, torch.from_numpy(np.ascontiguousarray(a)).cuda()) for n, _, a in ops]
    pl = cst.plan(text, [("X", csf)] + dev, fusion=fusion, options=options)
    print("       " + pl.describe().split("|")[0], flush=True)
    pl.check()
    out = cst.execute(pl, [t for _, t in dev])
    torch.cuda.synchronize()
    shape = [extents[c] for c in out_idx]
    got = out.cpu().numpy().reshape(shape)
    f = [(a, l) for _, l, a in ops]
    want = nary.contract(coords, vals, LEVELS[:order], f, out_idx, extents)
    S = nary.contract_abs(coords, vals, LEVELS[:order], f, out_idx, extents)
    err = oracle.rel_err(got, want, S)
    print("       rel err %.3e" % err, flush=True)
    assert err <= TOL
