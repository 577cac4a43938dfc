"""Many small random instances of the sparse x sparse kernels and of the three-tensor network against
the dense references: odd extents, very sparse and nearly dense operands, repeated in one process;
from seed 12 on also with plan options drawn from the values each option takes."""
import numpy as np
import pytest
import torch

from oracle import spsp
import oracle
import paper_2401_04836_amd as cst
from paper_2401_04836_amd import schedules as S
from helpers import TOL, compare, run_gpu, run_oracle
from workloads.generators import make_sptn3_scattered

pytestmark = pytest.mark.gpu


def _options(rng, seed, table):
    """{} for the first twelve seeds; then each option of the table with probability one half."""
    opts = {}
    if seed >= 12:
        for name, values in table:
            if rng.integers(2):
                opts[name] = int(values[int(rng.integers(len(values)))])
    return opts


def _sparse(rng, shape, density):
    total = int(np.prod(shape))
    nnz = max(1, int(round(total * density)))
    cells = rng.choice(total, size=min(nnz, total), replace=False)
    return [c.astype(np.int64) for c in np.unravel_index(cells, shape)], rng.standard_normal(min(nnz, total))


def _csf(c, v, dims, mo):
    return cst.build_csf([torch.as_tensor(x, dtype=torch.int32).cuda() for x in c],
                         torch.as_tensor(v, dtype=torch.float64).cuda(), dims, mo)


def _coords3(E):
    (i0, p0, _), (i1, p1, _), (i2, _, _) = E.export(0), E.export(1), E.export(2)
    i0, p0, i1, p1, i2 = (t.cpu().numpy() for t in (i0, p0, i1, p1, i2))
    nK = np.repeat(i0, np.diff(p0))
    return np.repeat(nK, np.diff(p1)), np.repeat(i1, np.diff(p1)), i2


@pytest.mark.parametrize("seed", range(40))
def test_chain_random(seed):
    rng = np.random.default_rng(7000 + seed)
    n_K, n_i, n_u, n_m = (int(x) for x in rng.integers(1, [12, 9, 40, 50]))
    dI, dC, dP, dL = rng.choice([0.02, 0.1, 0.4, 0.9], size=4)
    opts = _options(rng, seed, (("spchain3_form", [1, 2]), ("spchain3_order", [0, 1]), ("spchain3_local_kb", [1, 4, 30, 78])))
    print("[case] chain seed %d: K,i,u,m = %s densities %s options %s" % (seed, (n_K, n_i, n_u, n_m), (dI, dC, dP, dL), opts), flush=True)
    I = _sparse(rng, (n_K, n_u, n_u), dI)
    C = _sparse(rng, (n_u, n_i), dC)
    P = _sparse(rng, (n_u, n_m), dP)
    L = _sparse(rng, (n_K, n_i), dL)
    dims = (n_K, n_i, n_u, n_m)
    hI, hC, hP, hL = _csf(*I, (n_K, n_u, n_u), [0, 1, 2]), _csf(*C, (n_u, n_i), [1, 0]), \
        _csf(*P, (n_u, n_m), [1, 0]), _csf(*L, (n_K, n_i), [0, 1])
    for text, ops, Lx in ((S.SPCHAIN3, [("I", hI), ("C", hC), ("P", hP)], None),
                          (S.SPCHAIN3_RESTRICTED, [("I", hI), ("C", hC), ("L", hL), ("P", hP)], L)):
        pl = cst.plan(text, ops, options=opts or None)
        vals = cst.execute(pl, []).cpu().numpy()
        gK, gi, gm = _coords3(pl.output_csf())
        ref = spsp.chain3(I, C, P, dims, Lx, K_values=range(n_K))
        G = np.zeros((n_K, n_i, n_m)); M = np.zeros((n_K, n_i, n_m), dtype=bool)
        G[gK, gi, gm] = vals
        M[gK, gi, gm] = True
        assert int(M.sum()) == vals.size
        for K in range(n_K):
            E, Sabs, N = ref[K]
            np.testing.assert_array_equal(M[K], N, err_msg="seed %d K %d" % (seed, K))
            assert oracle.rel_err(G[K], E, Sabs) <= TOL


@pytest.mark.parametrize("seed", range(40))
def test_four_index_random(seed):
    rng = np.random.default_rng(8000 + seed)
    n_K, n_i, n_m = (int(x) for x in rng.integers(1, [40, 7, 45]))
    density = float(rng.choice([0.03, 0.2, 0.7, 1.0]))
    Ec, Ev = _sparse(rng, (n_K, n_i, n_m), density)
    opts = _options(rng, seed, (("sppair4_keep", [1, 2]), ("sppair4_rows", [1, 2]), ("sppair4_buffers", [1, 2]), ("sppair4_xcd", [0, 1, 2])))
    print("[case] four-index seed %d: K,i,m = %s density %s options %s" % (seed, (n_K, n_i, n_m), density, opts), flush=True)
    hE = _csf(Ec, Ev, (n_K, n_i, n_m), [1, 0, 2])
    pl = cst.plan(S.SPPAIR4, [("Ea", hE), ("Eb", hE)], options=opts or None)
    vals = cst.execute(pl, []).cpu().numpy()
    V = pl.output_csf()
    lv = [V.export(l) for l in range(4)]
    idx = [t[0].cpu().numpy() for t in lv]
    ptr = [t[1].cpu().numpy() for t in lv[:3]]
    n1 = np.repeat(np.arange(idx[1].size), np.diff(ptr[1]))
    n0 = np.repeat(np.arange(idx[0].size), np.diff(ptr[0]))
    cm = np.repeat(idx[2], np.diff(ptr[2]))
    cj = np.repeat(idx[1][n1], np.diff(ptr[2]))
    ci = np.repeat(idx[0][n0][n1], np.diff(ptr[2]))
    want, Sabs, N = spsp.pair4(Ec, Ev, (n_K, n_i, n_m))
    G = np.zeros_like(want); M = np.zeros(want.shape, dtype=bool)
    G[ci, cj, cm, idx[3]] = vals
    M[ci, cj, cm, idx[3]] = True
    assert int(M.sum()) == vals.size
    np.testing.assert_array_equal(M, N)
    assert oracle.rel_err(G, want, Sabs) <= TOL


@pytest.mark.parametrize("seed", range(30))
def test_three_tensor_random(seed):
    """Z[i,m] = U[i,j,k] V[j,l] W[k,l,m] with scattered U and W of random extents and fill: the tiled kernel in
    both of its forms, and the baseline kernel."""
    rng = np.random.default_rng(9000 + seed)
    I, J, K, L, M = (int(x) for x in rng.integers(1, [40, 60, 30, 70, 50]))
    nnz_u = max(1, int(I * J * K * float(rng.choice([0.01, 0.1, 0.5]))))
    nnz_w = max(1, int(K * L * M * float(rng.choice([0.01, 0.1, 0.5]))))
    opts = {"sptn3_tiled": int(rng.choice([0, 2, 2]))}
    opts.update(_options(rng, seed + 12, (("sptn3_waves", [1, 2]), ("sptn3_wgs", [1, 50, 8000]), ("sptn3_xcd", [0, 1]))))
    print("[case] three-tensor seed %d: dims %s nnz %d + %d options %s" % (seed, (I, J, K, L, M), nnz_u, nnz_w, opts), flush=True)
    wl = make_sptn3_scattered("rnd%d" % seed, 500 + seed, (I, J, K, L, M), nnz_u, nnz_w)
    out, pl, _ = run_gpu(wl, options=opts)
    print("       " + pl.describe().split("|")[0], flush=True)
    want, S_abs = run_oracle(wl)
    assert compare(out, want, S_abs) <= TOL
