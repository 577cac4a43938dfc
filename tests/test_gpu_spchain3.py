"""Chain of three sparse tensors with a sparse result (Sec. 5.1, both forms) on the GPU against
the dense-slice reference: the structure of the result must be identical (it is index work), the
values within the tolerance of every other contraction."""

import numpy as np
import pytest
import torch

from oracle import spsp
import oracle
import paper_2401_04836_amd as cst
from helpers import TOL
from workloads.generators import make_lattice_chain, SparseCOO

pytestmark = pytest.mark.gpu

UNRESTRICTED = "T[K,i,v] = I[K,u,v] * C[i,u] | K,i,u,v ; E[K,i,m] = T[K,i,v] * P[m,v] | K,i,m,v"
RESTRICTED = ("T[K,i,v] = I[K,u,v] * C[i,u] | K,i,u,v ; F[K,i,v] = T[K,i,v] * L[K,i] | K,i,v ; "
              "E[K,i,m] = F[K,i,v] * P[m,v] | K,i,m,v")


def _say(msg):
    print(msg, flush=True)


def _csf(t, mode_order):
    return cst.build_csf([c.cuda() for c in t.coords], t.vals.cuda(), t.dims, mode_order)


def _run(I, C, P, L=None, kernel=None, extra=None):
    """Returns (coords of E as three host arrays, values, plan description).  kernel: None = the
    plan's choice, "general" = the form without dense blocks, "block-local" = expect that form."""
    hI, hC, hP = _csf(I, [0, 1, 2]), _csf(C, [1, 0]), _csf(P, [1, 0])
    options = "spchain3_form=2" if kernel == "general" else None
    if extra:
        options = extra if options is None else options + "," + extra
    if L is None:
        pl = cst.plan(UNRESTRICTED, [("I", hI), ("C", hC), ("P", hP)], options=options)
    else:
        hL = _csf(L, [0, 1])
        pl = cst.plan(RESTRICTED, [("I", hI), ("C", hC), ("L", hL), ("P", hP)], options=options)
    desc = pl.describe()
    assert "family=spchain3" in desc, desc
    if kernel is not None:
        assert ("kernel=" + kernel) in desc, desc
    vals = cst.execute(pl, [])
    again = cst.execute(pl, [])
    torch.cuda.synchronize()
    assert torch.equal(vals, again)                       # no atomics: bit-reproducible
    E = pl.output_csf()
    i0, p0, _ = E.export(0)
    i1, p1, _ = E.export(1)
    i2, _, v2 = E.export(2)
    assert v2 is None
    i0, p0, i1, p1, i2 = (t.cpu().numpy() for t in (i0, p0, i1, p1, i2))
    assert pl.n_rows == i2.size and pl.row_elems == 1
    assert p0[0] == 0 and p0[-1] == i1.size and p1[0] == 0 and p1[-1] == i2.size
    assert (np.diff(p0) > 0).all() and (np.diff(p1) > 0).all()          # no empty nodes
    assert (np.diff(i0) > 0).all()
    node_K = np.repeat(i0, np.diff(p0))
    leaf_K = np.repeat(node_K, np.diff(p1))
    leaf_i = np.repeat(i1, np.diff(p1))
    return (leaf_K, leaf_i, i2), vals.cpu().numpy(), desc


def _compare(got_coords, got_vals, ref, dims, all_K):
    """ref: {K: (E, S, N)} from the reference for the K in all_K; every other K must be absent
    from the result when all_K lists every K of the tensor."""
    n_K, n_i, n_u, n_m = dims
    gK, gi, gm = got_coords
    worst = 0.0
    for K in all_K:
        E, S, N = ref[K]
        sel = gK == K
        G = np.zeros((n_i, n_m))
        M = np.zeros((n_i, n_m), dtype=bool)
        G[gi[sel], gm[sel]] = got_vals[sel]
        M[gi[sel], gm[sel]] = True
        assert int(sel.sum()) == int(M.sum())               # no duplicate positions
        np.testing.assert_array_equal(M, N, err_msg="structure of E[%d]" % K)
        # children ascending within every (K,i): CSF order
        order = np.lexsort((gm[sel], gi[sel]))
        assert (order == np.arange(order.size)).all()
        worst = max(worst, oracle.rel_err(G, E, S))
    return worst


def _np(t):
    return ([c.numpy() for c in t.coords], t.vals.numpy())


def _scattered(seed, dims, nnz_I, nnz_C, nnz_P, nnz_L):
    n_K, n_i, n_u, n_m = dims
    g = torch.Generator().manual_seed(seed)

    def rand(shape, nnz, ones=False):
        total = int(np.prod(shape))
        cells = torch.randperm(total, generator=g)[:nnz]
        coords = []
        for d in reversed(shape):
            coords.append((cells % d).to(torch.int32))
            cells = cells // d
        coords.reverse()
        vals = torch.ones(nnz, dtype=torch.float64) if ones else torch.randn(nnz, generator=g, dtype=torch.float64)
        return SparseCOO(tuple(shape), coords, vals)
    return (rand((n_K, n_u, n_u), nnz_I), rand((n_u, n_i), nnz_C), rand((n_u, n_m), nnz_P),
            rand((n_K, n_i), nnz_L, ones=True))


def test_small_lattice_both_forms():
    wl = make_lattice_chain("lat5", 4101, 5, 3, 6, 1.5, 2.0, 1.5, 2.5)
    dims = wl.params["dims"]
    I, C, P, L = (wl.sparse[k] for k in "ICPL")
    _say("5 x 5 lattice: dims %s, nnz I %d C %d P %d L %d" % (dims, I.nnz, C.nnz, P.nnz, L.nnz))
    Ks = range(dims[0])
    ref_u = spsp.chain3(_np(I), _np(C), _np(P), dims, K_values=Ks)
    ref_r = spsp.chain3(_np(I), _np(C), _np(P), dims, _np(L), K_values=Ks)
    coords, vals, desc = _run(I, C, P, kernel="block-local", extra="spchain3_order=0")     # roots in root order
    assert _compare(coords, vals, ref_u, dims, Ks) <= TOL
    for kernel in ("block-local", "general"):
        coords, vals, desc = _run(I, C, P, kernel=kernel)
        err = _compare(coords, vals, ref_u, dims, Ks)
        _say("  unrestricted: %s nnz(E) %d rel err %.3e" % (desc.split("T:")[0], vals.size, err))
        assert err <= TOL
        coords, vals, desc = _run(I, C, P, L, kernel=kernel)
        err = _compare(coords, vals, ref_r, dims, Ks)
        _say("  restricted:   nnz(E) %d rel err %.3e" % (vals.size, err))
        assert err <= TOL


def test_scattered_inputs_ragged_extents_and_missing_indices():
    # no lattice structure: K without a matching u, i absent from C, m absent from P, v absent from P
    dims = (37, 19, 45, 70)
    I, C, P, L = _scattered(4102, dims, 1500, 120, 200, 150)
    L.vals = torch.randn(L.nnz, generator=torch.Generator().manual_seed(5), dtype=torch.float64)   # a weighted filter
    Ks = range(dims[0])
    for form, Lx in (("unrestricted", None), ("restricted", L)):
        coords, vals, _ = _run(I, C, P, Lx)
        ref = spsp.chain3(_np(I), _np(C), _np(P), dims, _np(Lx) if Lx is not None else None, K_values=Ks)
        err = _compare(coords, vals, ref, dims, Ks)
        _say("scattered %s: nnz(E) %d rel err %.3e" % (form, vals.size, err))
        assert err <= TOL


def test_long_lists_span_several_wavefront_passes():
    # > 64 u under one K, > 64 v under one u, > 64 m per (K,i), many slots
    dims = (6, 9, 300, 400)
    I, C, P, L = _scattered(4103, dims, 60000, 900, 9000, 30)
    Ks = range(dims[0])
    coords, vals, desc = _run(I, C, P, kernel="general")          # blocks of 300 x 300 do not fit LDS
    ref = spsp.chain3(_np(I), _np(C), _np(P), dims, K_values=Ks)
    err = _compare(coords, vals, ref, dims, Ks)
    _say("long lists: nnz(E) %d rel err %.3e" % (vals.size, err))
    assert err <= TOL


def test_block_local_with_more_slots_and_entries_than_a_wavefront():
    # K-local blocks with > 64 v slots, > 64 u rows and C rows of > 64 entries, still within LDS
    dims = (5, 7, 70, 40)
    I, C, P, L = _scattered(4106, dims, 9000, 480, 1500, 20)
    Ks = range(dims[0])
    ref = spsp.chain3(_np(I), _np(C), _np(P), dims, K_values=Ks)
    for kernel in ("block-local", "general"):
        coords, vals, _ = _run(I, C, P, kernel=kernel)
        err = _compare(coords, vals, ref, dims, Ks)
        _say("dense blocks, %s: nnz(E) %d rel err %.3e" % (kernel, vals.size, err))
        assert err <= TOL


def test_empty_result_and_empty_operands():
    dims = (8, 5, 12, 9)
    I, C, P, L = _scattered(4104, dims, 40, 10, 15, 10)
    # C's u all outside I's u: shift C's u range away
    C2 = SparseCOO(C.dims, [torch.full_like(C.coords[0], 11), C.coords[1]], C.vals)
    keep = I.coords[1] != 11
    I2 = SparseCOO(I.dims, [c[keep] for c in I.coords], I.vals[keep])
    # distinct coordinates in C2: keep one entry per i
    _, first = np.unique(C2.coords[1].numpy(), return_index=True)
    C2 = SparseCOO(C.dims, [c[first] for c in C2.coords], C2.vals[first])
    coords, vals, _ = _run(I2, C2, P)
    assert vals.size == 0 and coords[0].size == 0
    empty = SparseCOO(I.dims, [torch.empty(0, dtype=torch.int32)] * 3, torch.empty(0, dtype=torch.float64))
    coords, vals, _ = _run(empty, C, P)
    assert vals.size == 0


def test_medium_lattice_sampled_slices():
    wl = make_lattice_chain("lat12", 4105, 12, 3, 10, 2.0, 2.0, 2.0, 3.0)
    dims = wl.params["dims"]
    I, C, P, L = (wl.sparse[k] for k in "ICPL")
    _say("12 x 12 lattice: dims %s, nnz I %d C %d P %d L %d" % (dims, I.nnz, C.nnz, P.nnz, L.nnz))
    Ks = sorted(set(np.random.default_rng(1).integers(0, dims[0], 40).tolist()) | {0, dims[0] - 1})
    for form, Lx in (("unrestricted", None), ("restricted", L)):
        coords, vals, _ = _run(I, C, P, Lx, kernel="block-local")
        ref = spsp.chain3(_np(I), _np(C), _np(P), dims, _np(Lx) if Lx is not None else None, K_values=Ks)
        err = _compare(coords, vals, ref, dims, Ks)
        _say("  %s: nnz(E) %d, %d sampled K, rel err %.3e" % (form, vals.size, len(Ks), err))
        assert err <= TOL


def test_plans_outside_the_family_are_refused():
    wl = make_lattice_chain("lat5", 4101, 5, 3, 6, 1.5, 2.0, 1.5, 2.5)
    I, C, P = (wl.sparse[k] for k in "ICP")
    hI, hC, hP = _csf(I, [0, 1, 2]), _csf(C, [1, 0]), _csf(P, [1, 0])
    # fused on K only (depth 1): not the tuned kernel's schedule.  The generic executor takes it with dense
    # copies of C and P and a DENSE result E[K,i,m]; without them it is refused.
    with pytest.raises(cst.ConststnError):
        cst.plan(UNRESTRICTED, [("I", hI), ("C", hC), ("P", hP)], fusion=[1, 0], options={"generic_densify": 0})
    pl = cst.plan(UNRESTRICTED, [("I", hI), ("C", hC), ("P", hP)], fusion=[1, 0])
    assert "family=generic" in pl.describe() and "dense_copies_of_csf_operands=2" in pl.describe(), pl.describe()
    dims = wl.params["dims"]
    got = cst.execute(pl, []).cpu().numpy().reshape(dims[0], dims[1], dims[3])
    ref = spsp.chain3(_np(I), _np(C), _np(P), dims, K_values=range(dims[0]))
    for K in range(dims[0]):
        E, S_abs, N = ref[K]
        assert not got[K][~N].any()                        # no term, exact zero
        assert oracle.rel_err(got[K], E, S_abs) <= TOL
    with pytest.raises(cst.ConststnError):
        cst.plan(UNRESTRICTED, [("I", hI), ("C", hC), ("P", hP)], flags=cst.OUT_COMPACT)
