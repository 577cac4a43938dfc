"""Every output mode of the order-3 MTTKRP and TTMc (Sec. 5.2-5.3 run one contraction per mode)
by re-rooting the CSF: output mode at the root, the two other modes in either order below it."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import workloads as w
from helpers import TOL, compare, to_dev
import paper_2401_04836_amd as cst
from paper_2401_04836_amd import schedules as S

pytestmark = pytest.mark.gpu

LEVELS = [p for p in itertools.permutations(range(3))]


def _say(msg):
    print(msg, flush=True)


def _factors(seed, dims, ranks):
    g = torch.Generator().manual_seed(seed)
    return [torch.rand(dims[m], ranks[m], generator=g, dtype=torch.float64) * 2 - 1 for m in range(3)]


@pytest.mark.parametrize("levels", LEVELS)
def test_mttkrp_every_mode_and_level_order(levels):
    wl = w.make(2, small=True)
    X = wl.sparse["X"]
    F = _factors(77, X.dims, (32, 32, 32))
    _say("mttkrp output mode %d, CSF level order %s" % (levels[0], (levels,)))
    dc, dv = to_dev(X)
    csf = cst.build_csf(dc, dv, X.dims, list(levels))
    text, names = S.mttkrp3_for(levels)
    leaf, mid = F[levels[2]].cuda(), F[levels[1]].cuda()
    pl = cst.plan(text, [(names[0], csf), (names[1], leaf), (names[2], mid)])
    out = cst.execute(pl, [leaf, mid]).reshape(pl.n_rows, -1)
    torch.cuda.synchronize()
    c, v = X.numpy()
    other = sorted(levels[1:])
    Fa, Fb = F[other[0]].numpy(), F[other[1]].numpy()
    want = oracle.mttkrp3(c, v, X.dims, Fa, Fb, levels[0])
    S_abs = oracle.mttkrp3_abs(c, v, X.dims, Fa, Fb, levels[0])
    assert compare(out, want, S_abs) <= TOL


@pytest.mark.parametrize("levels", LEVELS)
@pytest.mark.parametrize("ranks", [(8, 5, 11), (16, 32, 48)])
def test_ttmc3_every_mode_and_level_order(levels, ranks):
    wl = w.make(1)
    X = wl.sparse["X"]
    F = _factors(78, X.dims, ranks)
    _say("ttmc output mode %d, CSF level order %s, ranks %s" % (levels[0], (levels,), (ranks,)))
    dc, dv = to_dev(X)
    csf = cst.build_csf(dc, dv, X.dims, list(levels))
    text, names = S.ttmc3_for(levels)
    leaf, mid = F[levels[2]].cuda(), F[levels[1]].cuda()
    pl = cst.plan(text, [(names[0], csf), (names[1], leaf), (names[2], mid)])
    out = cst.execute(pl, [leaf, mid]).reshape(pl.n_rows, mid.shape[1], leaf.shape[1])
    torch.cuda.synchronize()
    c, v = X.numpy()
    other = sorted(levels[1:])
    Fa, Fb = F[other[0]].numpy(), F[other[1]].numpy()
    want = oracle.ttmc3(c, v, X.dims, Fa, Fb, levels[0])            # [root, R_other0, R_other1]
    S_abs = oracle.ttmc3_abs(c, v, X.dims, Fa, Fb, levels[0])
    if levels[1] > levels[2]:                                       # GPU rows are [middle, leaf]
        out = out.permute(0, 2, 1).contiguous()
    assert compare(out, want, S_abs) <= TOL
