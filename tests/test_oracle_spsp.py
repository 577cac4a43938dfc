"""Pins of the sparse x sparse x sparse reference (oracle/spsp.py) against what Sec. 2.1 and
Sec. 5.1 fix: brute-force loops over the coordinate lists, the N-ary routine with densified
factors, identities, the filter relation between the two forms, and the join structure."""
import itertools

import numpy as np
import pytest

from oracle import nary, spsp


def _rand_sparse(rng, shape, nnz):
    total = int(np.prod(shape))
    cells = rng.choice(total, size=min(nnz, total), replace=False)
    coords = list(np.unravel_index(cells, shape))
    vals = rng.standard_normal(len(cells))
    return [c.astype(np.int64) for c in coords], vals


def _brute(I, C, P, dims, L=None):
    """Every term of the sum visited by nested loops over the stored entries (Fig. 2b style)."""
    n_K, n_i, n_u, n_m = dims
    E = np.zeros((n_K, n_i, n_m))
    S = np.zeros((n_K, n_i, n_m))
    N = np.zeros((n_K, n_i, n_m), dtype=bool)
    Ld = {}
    if L is not None:
        for (k, i), v in zip(zip(*L[0]), L[1]):
            Ld[(int(k), int(i))] = v
    for (K, u, v), x in zip(zip(*I[0]), I[1]):
        for (u2, i), c in zip(zip(*C[0]), C[1]):
            if u2 != u:
                continue
            for (v2, m), p in zip(zip(*P[0]), P[1]):
                if v2 != v:
                    continue
                term = x * c * p
                if L is not None:
                    if (int(K), int(i)) not in Ld:
                        continue
                    term = term * Ld[(int(K), int(i))]
                E[K, i, m] += term
                S[K, i, m] += abs(term)
                N[K, i, m] = True
    return E, S, N


def _stack(res, n_K, n_i, n_m):
    E = np.zeros((n_K, n_i, n_m)); S = np.zeros((n_K, n_i, n_m)); N = np.zeros((n_K, n_i, n_m), dtype=bool)
    for K, (e, s, n) in res.items():
        E[K], S[K], N[K] = e, s, n
    return E, S, N


@pytest.mark.parametrize("seed,dims,with_filter", [(1, (4, 3, 5, 6), False), (2, (3, 5, 4, 2), True),
                                                   (3, (6, 2, 3, 7), True), (4, (2, 6, 6, 3), False)])
def test_chain3_against_brute_force(seed, dims, with_filter):
    rng = np.random.default_rng(seed)
    n_K, n_i, n_u, n_m = dims
    I = _rand_sparse(rng, (n_K, n_u, n_u), 3 * n_K * n_u // 2)
    C = _rand_sparse(rng, (n_u, n_i), n_u * n_i // 2)
    P = _rand_sparse(rng, (n_u, n_m), n_u * n_m // 2)
    L = _rand_sparse(rng, (n_K, n_i), n_K * n_i // 2) if with_filter else None
    E, S, N = _stack(spsp.chain3(I, C, P, dims, L, K_values=range(n_K)), n_K, n_i, n_m)
    Eb, Sb, Nb = _brute(I, C, P, dims, L)
    np.testing.assert_array_equal(N, Nb)
    np.testing.assert_allclose(E, Eb, rtol=0, atol=1e-13 * max(1.0, Sb.max()))
    np.testing.assert_allclose(S, Sb, rtol=1e-13, atol=0)
    assert not E[~N].any() and not S[~N].any()            # no term, exact zero
    assert (S[N] > 0).all()


def test_chain3_against_the_nary_routine_with_densified_factors():
    rng = np.random.default_rng(11)
    dims = (7, 4, 9, 5)
    n_K, n_i, n_u, n_m = dims
    I = _rand_sparse(rng, (n_K, n_u, n_u), 120)
    C = _rand_sparse(rng, (n_u, n_i), 15)
    P = _rand_sparse(rng, (n_u, n_m), 20)
    Cd = np.zeros((n_u, n_i)); Cd[C[0][0], C[0][1]] = C[1]
    Pd = np.zeros((n_u, n_m)); Pd[P[0][0], P[0][1]] = P[1]
    want = nary.contract(I[0], I[1], "Kuv", [(Cd, "ui"), (Pd, "vm")], "Kim", {"K": n_K, "i": n_i, "m": n_m})
    E, S, _ = _stack(spsp.chain3(I, C, P, dims, K_values=range(n_K)), n_K, n_i, n_m)
    np.testing.assert_allclose(E, want, rtol=0, atol=1e-13 * max(1.0, S.max()))


def test_identity_factors_return_the_integral_tensor():
    rng = np.random.default_rng(12)
    n = 6
    I = _rand_sparse(rng, (5, n, n), 60)
    eye = ([np.arange(n), np.arange(n)], np.ones(n))
    E, S, N = _stack(spsp.chain3(I, eye, eye, (5, n, n, n), K_values=range(5)), 5, n, n)
    D = np.zeros((5, n, n)); D[I[0][0], I[0][1], I[0][2]] = I[1]
    np.testing.assert_array_equal(E, D)
    np.testing.assert_array_equal(N, D != 0)


def test_filter_relation_between_the_two_forms():
    rng = np.random.default_rng(13)
    dims = (6, 5, 7, 4)
    n_K, n_i, n_u, n_m = dims
    I = _rand_sparse(rng, (n_K, n_u, n_u), 100)
    C = _rand_sparse(rng, (n_u, n_i), 18)
    P = _rand_sparse(rng, (n_u, n_m), 14)
    L = _rand_sparse(rng, (n_K, n_i), 13)
    L = (L[0], np.ones_like(L[1]))                        # a 0/1 sparse map
    E0, S0, N0 = _stack(spsp.chain3(I, C, P, dims, K_values=range(n_K)), n_K, n_i, n_m)
    E1, S1, N1 = _stack(spsp.chain3(I, C, P, dims, L, K_values=range(n_K)), n_K, n_i, n_m)
    mask = np.zeros((n_K, n_i), dtype=bool); mask[L[0][0], L[0][1]] = True
    np.testing.assert_array_equal(E1, np.where(mask[:, :, None], E0, 0.0))
    np.testing.assert_array_equal(N1, N0 & mask[:, :, None])
    full = ([np.repeat(np.arange(n_K), n_i), np.tile(np.arange(n_i), n_K)], np.ones(n_K * n_i))
    E2, _, N2 = _stack(spsp.chain3(I, C, P, dims, full, K_values=range(n_K)), n_K, n_i, n_m)
    np.testing.assert_array_equal(E2, E0)
    np.testing.assert_array_equal(N2, N0)


def test_default_k_values_are_the_nonempty_ones():
    rng = np.random.default_rng(14)
    I = _rand_sparse(rng, (9, 4, 4), 10)
    C = _rand_sparse(rng, (4, 3), 8)
    P = _rand_sparse(rng, (4, 3), 8)
    res = spsp.chain3(I, C, P, (9, 3, 4, 3))
    assert sorted(res) == sorted(set(int(k) for k in I[0][0]))


def test_pair4_against_brute_force_and_symmetry():
    rng = np.random.default_rng(15)
    n_K, n_i, n_m = 5, 3, 4
    Ec, Ev = _rand_sparse(rng, (n_K, n_i, n_m), 25)
    V, S, N = spsp.pair4(Ec, Ev, (n_K, n_i, n_m))
    Vb = np.zeros((n_i, n_i, n_m, n_m)); Sb = np.zeros_like(Vb); Nb = np.zeros(Vb.shape, dtype=bool)
    ent = list(zip(zip(*Ec), Ev))
    for ((K, i, m), a), ((K2, j, n), b) in itertools.product(ent, ent):
        if K == K2:
            Vb[i, j, m, n] += a * b
            Sb[i, j, m, n] += abs(a * b)
            Nb[i, j, m, n] = True
    np.testing.assert_array_equal(N, Nb)
    np.testing.assert_allclose(V, Vb, rtol=0, atol=1e-13 * max(1.0, Sb.max()))
    np.testing.assert_allclose(S, Sb, rtol=1e-13, atol=0)
    np.testing.assert_allclose(V, V.transpose(1, 0, 3, 2), rtol=0, atol=1e-13 * S.max())


def test_pair4_block_is_a_block_of_pair4():
    rng = np.random.default_rng(16)
    n_K, n_i, n_m = 6, 4, 5
    Ec, Ev = _rand_sparse(rng, (n_K, n_i, n_m), 50)
    V, S, N = spsp.pair4(Ec, Ev, (n_K, n_i, n_m))
    for i in range(n_i):
        for j in range(n_i):
            v, s, n = spsp.pair4_block(Ec, Ev, (n_K, n_i, n_m), i, j)
            np.testing.assert_allclose(v, V[i, j], rtol=0, atol=1e-13 * max(1.0, S.max()))
            np.testing.assert_allclose(s, S[i, j], rtol=1e-13, atol=0)
            np.testing.assert_array_equal(n, N[i, j])


def test_lattice_workload_has_the_stated_shape():
    from workloads.generators import make_lattice_chain
    wl = make_lattice_chain("t", 77, 5, 3, 6, 1.5, 2.0, 1.5, 2.5)
    n_K, n_i, n_u, n_m = wl.params["dims"]
    assert (n_K, n_i, n_u, n_m) == (150, 25, 75, 75)
    I, C, P, L = (wl.sparse[k] for k in "ICPL")
    assert I.dims == (n_K, n_u, n_u) and C.dims == (n_u, n_i) and P.dims == (n_u, n_m) and L.dims == (n_K, n_i)
    for t in (I, C, P, L):
        key = np.zeros(t.nnz, dtype=np.int64)
        for c, d in zip(t.coords, t.dims):
            assert int(c.min()) >= 0 and int(c.max()) < d
            key = key * d + c.numpy().astype(np.int64)
        assert np.unique(key).size == t.nnz                 # distinct coordinates
        assert (t.vals != 0).all()
    assert (L.vals == 1.0).all()
    # cut-off structure: an entry of C joins atoms at most r_mo = 2 apart
    au, ai = C.coords[0].numpy() // 3, C.coords[1].numpy()
    d2 = (au // 5 - ai // 5) ** 2 + (au % 5 - ai % 5) ** 2
    assert d2.max() <= 4
    again = make_lattice_chain("t", 77, 5, 3, 6, 1.5, 2.0, 1.5, 2.5)
    assert all((a == b).all() for a, b in zip(again.sparse["I"].coords, I.coords))
