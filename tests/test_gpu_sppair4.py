"""Four-index product V[i,j,m,n] = sum_K E[K,i,m] E[K,j,n] (Sec. 5.1) on the GPU against the dense
reference: structure identical, values within tolerance."""
import numpy as np
import pytest
import torch

from oracle import spsp
import oracle
import paper_2401_04836_amd as cst
from paper_2401_04836_amd import schedules as S
from helpers import TOL
from workloads.generators import make_lattice_chain

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _run(Ec, Ev, dims, Fc=None, Fv=None, fdims=None, options=None):
    """E (and optionally a second tensor F) as COO over (K, i, m).  Returns V's coordinates and values."""
    def csf(c, v, d):
        return cst.build_csf([torch.as_tensor(x, dtype=torch.int32).cuda() for x in c],
                             torch.as_tensor(v, dtype=torch.float64).cuda(), d, [1, 0, 2])
    hE = csf(Ec, Ev, dims)
    hF = hE if Fc is None else csf(Fc, Fv, fdims)
    pl = cst.plan(S.SPPAIR4, [("Ea", hE), ("Eb", hF)], options=options)
    desc = pl.describe()
    assert "family=sppair4" in desc, desc
    vals = cst.execute(pl, [])
    again = cst.execute(pl, [])
    torch.cuda.synchronize()
    assert torch.equal(vals, again)
    V = pl.output_csf()
    assert V.order == 4
    lv = [V.export(l) for l in range(4)]
    idx = [t[0].cpu().numpy() for t in lv]
    ptr = [t[1].cpu().numpy() for t in lv[:3]]
    assert lv[3][2] is None and pl.n_rows == idx[3].size
    for l in range(3):
        assert ptr[l][0] == 0 and ptr[l][-1] == idx[l + 1].size and (np.diff(ptr[l]) > 0).all()
    c2 = np.repeat(idx[2], np.diff(ptr[2]))
    n1 = np.repeat(np.arange(idx[1].size), np.diff(ptr[1]))            # pair node of every row
    c1 = np.repeat(idx[1][n1], np.diff(ptr[2]))
    n0 = np.repeat(np.arange(idx[0].size), np.diff(ptr[0]))            # root of every pair
    c0 = np.repeat(idx[0][n0][n1], np.diff(ptr[2]))
    return (c0, c1, c2, idx[3]), vals.cpu().numpy(), desc


def _rand_e(seed, dims, nnz):
    rng = np.random.default_rng(seed)
    cells = rng.choice(int(np.prod(dims)), size=nnz, replace=False)
    return [c.astype(np.int64) for c in np.unravel_index(cells, dims)], rng.standard_normal(nnz)


def test_small_random_whole_tensor():
    dims = (9, 6, 7)
    Ec, Ev = _rand_e(5101, dims, 150)
    (ci, cj, cm, cn), vals, desc = _run(Ec, Ev, dims)
    want, S_abs, N = spsp.pair4(Ec, Ev, dims)
    G = np.zeros_like(want)
    M = np.zeros(want.shape, dtype=bool)
    G[ci, cj, cm, cn] = vals
    M[ci, cj, cm, cn] = True
    assert int(M.sum()) == vals.size
    np.testing.assert_array_equal(M, N)
    key = ((ci.astype(np.int64) * 6 + cj) * 7 + cm) * 7 + cn
    assert (np.diff(key) > 0).all()                                      # CSF order i > j > m > n
    err = oracle.rel_err(G, want, S_abs)
    _say("%s nnz(V) %d rel err %.3e" % (desc.split("|")[0], vals.size, err))
    assert err <= TOL


def test_two_different_tensors_and_missing_indices():
    # Ea and Eb differ; some K stored in one only, some i without any shared K
    da, db = (20, 5, 40), (20, 4, 33)
    Ac, Av = _rand_e(5102, da, 300)
    Bc, Bv = _rand_e(5103, db, 200)
    keep = Bc[0] % 3 != 0                                               # Eb misses every third K
    Bc, Bv = [c[keep] for c in Bc], Bv[keep]
    (ci, cj, cm, cn), vals, _ = _run(Ac, Av, da, Bc, Bv, db)
    A = np.zeros(da); A[tuple(Ac)] = Av
    B = np.zeros(db); B[tuple(Bc)] = Bv
    want = np.einsum("kim,kjn->ijmn", A, B)
    S_abs = np.einsum("kim,kjn->ijmn", np.abs(A), np.abs(B))
    N = np.einsum("kim,kjn->ijmn", (A != 0).astype(float), (B != 0).astype(float)) > 0.5
    G = np.zeros_like(want); M = np.zeros(want.shape, dtype=bool)
    G[ci, cj, cm, cn] = vals
    M[ci, cj, cm, cn] = True
    np.testing.assert_array_equal(M, N)
    assert oracle.rel_err(G, want, S_abs) <= TOL


def test_blocks_larger_than_one_tile_group_and_many_shared_k():
    # > 16 x 8 tiles per (i,j) (m and n up to 200), > 16 shared K (several chunks)
    dims = (70, 3, 200)
    Ec, Ev = _rand_e(5104, dims, 9000)
    (ci, cj, cm, cn), vals, _ = _run(Ec, Ev, dims)
    worst = 0.0
    for i in range(3):
        for j in range(3):
            want, S_abs, N = spsp.pair4_block(Ec, Ev, dims, i, j)
            sel = (ci == i) & (cj == j)
            G = np.zeros_like(want); M = np.zeros(want.shape, dtype=bool)
            G[cm[sel], cn[sel]] = vals[sel]
            M[cm[sel], cn[sel]] = True
            np.testing.assert_array_equal(M, N)
            worst = max(worst, oracle.rel_err(G, want, S_abs))
    _say("large blocks: nnz(V) %d rel err %.3e" % (vals.size, worst))
    assert worst <= TOL


@pytest.mark.parametrize("env", [{"sppair4_rows": 2}, {"sppair4_keep": 2}, {},
                                 {"sppair4_buffers": 1}, {"sppair4_xcd": 0}, {"sppair4_xcd": 1}],
                         ids=["leaf-lists", "nothing-kept", "dense-rows", "one-chunk-buffer", "node-order", "xcd-order"])
@pytest.mark.parametrize("n_m", [200, 300])
def test_every_form_of_the_numeric_pass(env, n_m):
    # the chunk rows copied from dense rows (default, inner dimension <= 256), put together from leaf
    # lists kept by the plan, or found again by every launch; 300 distinct inner indices exceed one
    # 12 x 12 group of tiles and the dense form, and give rows of more than 128 leaves
    dims = (40, 3, n_m)
    Ec, Ev = _rand_e(5110 + n_m, dims, 40 * 3 * n_m * 6 // 10)
    (ci, cj, cm, cn), vals, desc = _run(Ec, Ev, dims, options=env)
    _say("%s: %s" % (env, desc.split("|")[0]))
    dense = "sppair4_rows" not in env and "sppair4_keep" not in env and n_m <= 256
    want_kernel = "nothing kept" if "sppair4_keep" in env else "dense rows" if dense else "leaf lists kept"
    assert "kernel=" + want_kernel in desc, desc
    worst = 0.0
    for i in range(3):
        for j in range(3):
            want, S_abs, N = spsp.pair4_block(Ec, Ev, dims, i, j)
            sel = (ci == i) & (cj == j)
            G = np.zeros_like(want); M = np.zeros(want.shape, dtype=bool)
            G[cm[sel], cn[sel]] = vals[sel]
            M[cm[sel], cn[sel]] = True
            np.testing.assert_array_equal(M, N)
            worst = max(worst, oracle.rel_err(G, want, S_abs))
    assert worst <= TOL


def test_lattice_integrals_from_the_three_index_tensor():
    # E from the reference of the chain on a 5 x 5 lattice, then V = E x E: the pipeline of Sec. 5.1
    wl = make_lattice_chain("lat5", 4101, 5, 3, 6, 1.5, 2.0, 1.5, 2.5)
    n_K, n_i, n_u, n_m = wl.params["dims"]
    as_np = lambda t: ([c.numpy() for c in t.coords], t.vals.numpy())
    ref = spsp.chain3(as_np(wl.sparse["I"]), as_np(wl.sparse["C"]), as_np(wl.sparse["P"]), wl.params["dims"],
                      K_values=range(n_K))
    ek, ei, em, ev = [], [], [], []
    for K, (E, _, N) in ref.items():
        ii, mm = np.nonzero(N)
        ek.append(np.full(ii.size, K)); ei.append(ii); em.append(mm); ev.append(E[ii, mm])
    Ec = [np.concatenate(x) for x in (ek, ei, em)]
    Ev = np.concatenate(ev)
    dims = (n_K, n_i, n_m)
    (ci, cj, cm, cn), vals, desc = _run(Ec, Ev, dims)
    _say("lattice 5 x 5: nnz(E) %d -> %s" % (Ev.size, desc.split("|")[0]))
    worst, total = 0.0, 0
    for i, j in [(0, 0), (0, 1), (3, 17), (12, 12), (24, 20), (7, 8), (24, 0)]:
        want, S_abs, N = spsp.pair4_block(Ec, Ev, dims, i, j)
        sel = (ci == i) & (cj == j)
        G = np.zeros_like(want); M = np.zeros(want.shape, dtype=bool)
        G[cm[sel], cn[sel]] = vals[sel]
        M[cm[sel], cn[sel]] = True
        np.testing.assert_array_equal(M, N, err_msg="structure of V[%d,%d]" % (i, j))
        worst = max(worst, oracle.rel_err(G, want, S_abs))
        total += int(sel.sum())
    _say("  %d sampled elements, rel err %.3e" % (total, worst))
    assert worst <= TOL
    # symmetry of the definition: V[i,j,m,n] = V[j,i,n,m]
    key = ((ci.astype(np.int64) * n_i + cj) * n_m + cm) * n_m + cn
    key_t = ((cj.astype(np.int64) * n_i + ci) * n_m + cn) * n_m + cm
    order = np.argsort(key_t)
    np.testing.assert_array_equal(key_t[order], key)
    np.testing.assert_allclose(vals[order], vals, rtol=0, atol=1e-9)


def test_empty_operand():
    dims = (5, 4, 6)
    (ci, cj, cm, cn), vals, _ = _run([np.zeros(0, dtype=np.int64)] * 3, np.zeros(0), dims)
    assert vals.size == 0
