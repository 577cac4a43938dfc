"""conststn_execute_static (partial row blocks in the library's static device array, nothing allocated by
the call) against conststn_execute, on two calls in a row, the second with a smaller input."""
import pytest
import torch

import paper_2401_04836_amd as cst
import workloads as w
from paper_2401_04836_amd import schedules as S

pytestmark = pytest.mark.gpu


def _plan(wl):
    dev = "cuda"
    X = wl.sparse["X"]
    csf = cst.build_csf([c.to(dev) for c in X.coords], X.vals.to(dev), X.dims, [0, 1, 2])
    U2, U3 = wl.dense["U2"].to(dev), wl.dense["U3"].to(dev)
    pl = cst.plan(S.TTMC3, [("X", csf), ("U3", U3), ("U2", U2)], flags=cst.OUT_COMPACT)
    return pl, [U3, U2]


def test_execute_static_matches_execute_twice_in_a_row():
    # a power-law tensor whose heaviest slices are cut into several work items (partial row blocks in use),
    # then a smaller one that leaves most of the array's previous contents in place
    cases = [w.make(5, small=True),
             w.make(5, small=True, dims=(3001, 2999, 509), nnz=40_009, ranks=(32, 64))]
    for n, wl in enumerate(cases):
        print("[case] execute_static call %d: %s" % (n, {k: (v.dims, v.nnz) for k, v in wl.sparse.items()}), flush=True)
        pl, facs = _plan(wl)
        assert "family=ttmc3" in pl.describe()
        assert int(pl.describe().split("partial_blocks=")[1].split()[0]) > 0     # the scratch array is in use
        want = cst.execute(pl, facs)
        got = torch.full_like(want, float("nan"))
        free_before = torch.cuda.mem_get_info()[0]
        cst.execute_static(pl, facs, got)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before          # nothing was allocated by the call
        assert torch.equal(got, want)                               # same kernels, same order of additions
        # and once more on the same plan: the array's contents from the first run do not leak into the result
        got2 = torch.full_like(want, float("nan"))
        cst.execute_static(pl, facs, got2)
        torch.cuda.synchronize()
        assert torch.equal(got2, want)


def test_execute_static_rejects_what_it_cannot_take():
    wl = w.make(2, small=True)
    X = wl.sparse["X"]
    csf = cst.build_csf([c.cuda() for c in X.coords], X.vals.cuda(), X.dims, [0, 1, 2])
    B, C = wl.dense["B"].cuda(), wl.dense["C"].cuda()
    pl = cst.plan(S.MTTKRP3, [("X", csf), ("C", C), ("B", B)])
    out = torch.empty(pl.n_rows * pl.row_elems, dtype=torch.float64, device="cuda")
    with pytest.raises(cst.ConststnError) as e:
        cst.execute_static(pl, [C, B], out)
    assert e.value.status_name == "EUNSUPPORTED"
