"""Pins for the CPU oracle: every contraction routine is checked against things
other than itself -- the textbook nested loop over densified tensors (Fig. 2b),
library einsum / matmul special cases (Sec. 2.1: R_ij = T_ik S_kj is a matrix
product), closed forms, linearity, mode-permutation invariance and the unfused
binary sequence (Fig. 3a).  The paper prints no numeric example to pin to."""
import itertools

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(12345)


def rand_coo(dims, nnz, rng=RNG):
    total = int(np.prod(dims))
    flat = rng.choice(total, size=nnz, replace=False)
    coords = np.unravel_index(flat, dims)
    vals = rng.uniform(-1, 1, size=nnz)
    vals[vals == 0] = 0.5
    return [c.astype(np.int32) for c in coords], vals


def densify(coords, vals, dims):
    D = np.zeros(dims)
    for n in range(len(vals)):
        D[tuple(int(c[n]) for c in coords)] = vals[n]
    return D


# ---------- brute force: one loop per index, one statement (Fig. 2b) -------------------------

def brute_ttmc3(D, Fa, Fb, mode):
    N = D.shape
    other = [m for m in range(3) if m != mode]
    Y = np.zeros((N[mode], Fa.shape[1], Fb.shape[1]))
    for c in itertools.product(range(N[0]), range(N[1]), range(N[2])):
        for ra in range(Fa.shape[1]):
            for rb in range(Fb.shape[1]):
                Y[c[mode], ra, rb] += D[c] * Fa[c[other[0]], ra] * Fb[c[other[1]], rb]
    return Y


def brute_mttkrp3(D, Fa, Fb, mode):
    N = D.shape
    other = [m for m in range(3) if m != mode]
    M = np.zeros((N[mode], Fa.shape[1]))
    for c in itertools.product(range(N[0]), range(N[1]), range(N[2])):
        for r in range(Fa.shape[1]):
            M[c[mode], r] += D[c] * Fa[c[other[0]], r] * Fb[c[other[1]], r]
    return M


def brute_ttmc4(D, U1, U2, U3):
    N = D.shape
    Y = np.zeros((N[0], U1.shape[1], U2.shape[1], U3.shape[1]))
    for i, j, k, l in itertools.product(*[range(n) for n in N]):
        if D[i, j, k, l] == 0.0:
            continue                       # adding an exact zero term changes nothing
        for r1 in range(U1.shape[1]):
            for r2 in range(U2.shape[1]):
                for r3 in range(U3.shape[1]):
                    Y[i, r1, r2, r3] += D[i, j, k, l] * U1[j, r1] * U2[k, r2] * U3[l, r3]
    return Y


def brute_sptn3(DU, V, DW):
    Ni, Nj, Nk = DU.shape
    _, L, M = DW.shape
    Z = np.zeros((Ni, M))
    for i in range(Ni):
        for m in range(M):
            s = 0.0
            for j in range(Nj):
                for k in range(Nk):
                    for l in range(L):
                        s += DU[i, j, k] * V[j, l] * DW[k, l, m]
            Z[i, m] = s
    return Z


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("ranks", [(1, 1), (2, 3), (3, 2)])
def test_ttmc3_vs_nested_loop(mode, ranks):
    dims = (4, 5, 3)
    coords, vals = rand_coo(dims, 23)
    other = [m for m in range(3) if m != mode]
    Fa = RNG.uniform(-1, 1, (dims[other[0]], ranks[0]))
    Fb = RNG.uniform(-1, 1, (dims[other[1]], ranks[1]))
    want = brute_ttmc3(densify(coords, vals, dims), Fa, Fb, mode)
    got = oracle.ttmc3(coords, vals, dims, Fa, Fb, mode)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("R", [1, 2, 3])
def test_mttkrp3_vs_nested_loop(mode, R):
    dims = (5, 3, 4)
    coords, vals = rand_coo(dims, 31)
    other = [m for m in range(3) if m != mode]
    Fa = RNG.uniform(-1, 1, (dims[other[0]], R))
    Fb = RNG.uniform(-1, 1, (dims[other[1]], R))
    want = brute_mttkrp3(densify(coords, vals, dims), Fa, Fb, mode)
    got = oracle.mttkrp3(coords, vals, dims, Fa, Fb, mode)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("ranks", [(1, 1, 1), (2, 3, 1), (3, 2, 2)])
def test_ttmc4_vs_nested_loop(ranks):
    dims = (3, 4, 3, 5)
    coords, vals = rand_coo(dims, 41)
    U1 = RNG.uniform(-1, 1, (dims[1], ranks[0]))
    U2 = RNG.uniform(-1, 1, (dims[2], ranks[1]))
    U3 = RNG.uniform(-1, 1, (dims[3], ranks[2]))
    want = brute_ttmc4(densify(coords, vals, dims), U1, U2, U3)
    got = oracle.ttmc4(coords, vals, dims, U1, U2, U3)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_sptn3_vs_nested_loop():
    udims, wdims = (4, 5, 3), (3, 4, 6)
    uc, uv = rand_coo(udims, 27)
    wc, wv = rand_coo(wdims, 19)
    V = RNG.normal(size=(5, 4))
    want = brute_sptn3(densify(uc, uv, udims), V, densify(wc, wv, wdims))
    got = oracle.sptn3(uc, uv, udims, V, wc, wv, wdims)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


# ---------- library routine on densified inputs ---------------------------------------------

def test_all_forms_vs_einsum():
    dims = (7, 6, 8)
    coords, vals = rand_coo(dims, 90)
    D = densify(coords, vals, dims)
    A, B, C = RNG.normal(size=(7, 4)), RNG.normal(size=(6, 4)), RNG.normal(size=(8, 4))
    U = [RNG.normal(size=(7, 3)), RNG.normal(size=(6, 2)), RNG.normal(size=(8, 5))]
    np.testing.assert_allclose(oracle.ttmc3(coords, vals, dims, U[1], U[2], 0),
                               np.einsum("ijk,jy,kz->iyz", D, U[1], U[2]), atol=1e-12)
    np.testing.assert_allclose(oracle.ttmc3(coords, vals, dims, U[0], U[2], 1),
                               np.einsum("ijk,ix,kz->jxz", D, U[0], U[2]), atol=1e-12)
    np.testing.assert_allclose(oracle.ttmc3(coords, vals, dims, U[0], U[1], 2),
                               np.einsum("ijk,ix,jy->kxy", D, U[0], U[1]), atol=1e-12)
    np.testing.assert_allclose(oracle.mttkrp3(coords, vals, dims, B, C, 0),
                               np.einsum("ijk,jr,kr->ir", D, B, C), atol=1e-12)
    np.testing.assert_allclose(oracle.mttkrp3(coords, vals, dims, A, C, 1),
                               np.einsum("ijk,ir,kr->jr", D, A, C), atol=1e-12)
    np.testing.assert_allclose(oracle.mttkrp3(coords, vals, dims, A, B, 2),
                               np.einsum("ijk,ir,jr->kr", D, A, B), atol=1e-12)
    d4 = (5, 6, 4, 7)
    c4, v4 = rand_coo(d4, 120)
    U1, U2, U3 = RNG.normal(size=(6, 3)), RNG.normal(size=(4, 2)), RNG.normal(size=(7, 4))
    np.testing.assert_allclose(oracle.ttmc4(c4, v4, d4, U1, U2, U3),
                               np.einsum("ijkl,jr,ks,lt->irst", densify(c4, v4, d4), U1, U2, U3),
                               atol=1e-12)
    udims, wdims = (6, 7, 5), (5, 8, 9)
    uc, uv = rand_coo(udims, 60)
    wc, wv = rand_coo(wdims, 70)
    V = RNG.normal(size=(7, 8))
    np.testing.assert_allclose(oracle.sptn3(uc, uv, udims, V, wc, wv, wdims),
                               np.einsum("ijk,jl,klm->im", densify(uc, uv, udims), V,
                                         densify(wc, wv, wdims)), atol=1e-11)


def test_order2_case_is_matrix_product():
    """Sec. 2.1: R_ij = T_ik S_kj is a matrix product.  A tensor whose third mode has
    extent 1, with the 1x1 factor [[1]], turns TTMc into sparse-matrix x dense-matrix."""
    dims = (9, 11, 1)
    coords, vals = rand_coo(dims, 40)
    U2 = RNG.normal(size=(11, 5))
    one = np.ones((1, 1))
    Y = oracle.ttmc3(coords, vals, dims, U2, one, 0)
    Xmat = densify(coords, vals, dims)[:, :, 0]
    np.testing.assert_allclose(Y[:, :, 0], Xmat @ U2, atol=1e-13)
    M = oracle.mttkrp3(coords, vals, dims, U2, np.ones((1, 5)), 0)
    np.testing.assert_allclose(M, Xmat @ U2, atol=1e-13)


# ---------- closed forms --------------------------------------------------------------------

def test_single_nonzero_is_scaled_outer_product():
    dims = (5, 6, 7)
    coords = [np.array([3], np.int32), np.array([4], np.int32), np.array([2], np.int32)]
    vals = np.array([-0.75])
    U2, U3 = RNG.normal(size=(6, 3)), RNG.normal(size=(7, 4))
    Y = oracle.ttmc3(coords, vals, dims, U2, U3, 0)
    want = np.zeros((5, 3, 4))
    want[3] = -0.75 * np.outer(U2[4], U3[2])
    np.testing.assert_allclose(Y, want, rtol=4e-16, atol=0)
    B, C = RNG.normal(size=(6, 4)), RNG.normal(size=(7, 4))
    M = oracle.mttkrp3(coords, vals, dims, B, C, 0)
    wantM = np.zeros((5, 4))
    wantM[3] = -0.75 * B[4] * C[2]
    np.testing.assert_allclose(M, wantM, rtol=4e-16, atol=0)


def test_ones_factors_give_slice_sums_and_identity_gives_dense():
    dims = (6, 5, 4)
    coords, vals = rand_coo(dims, 50)
    D = densify(coords, vals, dims)
    Y = oracle.ttmc3(coords, vals, dims, np.ones((5, 1)), np.ones((4, 1)), 0)
    np.testing.assert_allclose(Y[:, 0, 0], D.sum(axis=(1, 2)), atol=1e-13)
    Yd = oracle.ttmc3(coords, vals, dims, np.eye(5), np.eye(4), 0)
    np.testing.assert_array_equal(Yd, D)
    d4 = (3, 4, 5, 2)
    c4, v4 = rand_coo(d4, 30)
    Y4 = oracle.ttmc4(c4, v4, d4, np.eye(4), np.eye(5), np.eye(2))
    np.testing.assert_array_equal(Y4, densify(c4, v4, d4))


def test_mttkrp_rank1_equals_ttmc_rank1():
    dims = (8, 7, 9)
    coords, vals = rand_coo(dims, 100)
    b, c = RNG.normal(size=(7, 1)), RNG.normal(size=(9, 1))
    np.testing.assert_allclose(oracle.mttkrp3(coords, vals, dims, b, c, 0)[:, 0],
                               oracle.ttmc3(coords, vals, dims, b, c, 0)[:, 0, 0], atol=1e-14)


def test_mttkrp_is_diagonal_of_ttmc():
    """M[i,r] = Y[i,r,r] when both use the same factors (batch index = equal rank indices)."""
    dims = (8, 7, 9)
    coords, vals = rand_coo(dims, 120)
    B, C = RNG.normal(size=(7, 4)), RNG.normal(size=(9, 4))
    Y = oracle.ttmc3(coords, vals, dims, B, C, 0)
    M = oracle.mttkrp3(coords, vals, dims, B, C, 0)
    np.testing.assert_allclose(M, np.einsum("irr->ir", Y), atol=1e-13)


# ---------- invariants ----------------------------------------------------------------------

def test_linearity_in_X():
    dims = (6, 7, 5)
    c1, v1 = rand_coo(dims, 60)
    c2, v2 = rand_coo(dims, 45)
    a, b = 1.75, -0.375
    U2, U3 = RNG.normal(size=(7, 3)), RNG.normal(size=(5, 2))
    D = a * densify(c1, v1, dims) + b * densify(c2, v2, dims)
    nz = np.nonzero(D)
    cu = [x.astype(np.int32) for x in nz]
    vu = D[nz]
    lhs = oracle.ttmc3(cu, vu, dims, U2, U3, 0)
    rhs = a * oracle.ttmc3(c1, v1, dims, U2, U3, 0) + b * oracle.ttmc3(c2, v2, dims, U2, U3, 0)
    np.testing.assert_allclose(lhs, rhs, atol=1e-12)
    B, C = RNG.normal(size=(7, 3)), RNG.normal(size=(5, 3))
    lhs = oracle.mttkrp3(cu, vu, dims, B, C, 0)
    rhs = a * oracle.mttkrp3(c1, v1, dims, B, C, 0) + b * oracle.mttkrp3(c2, v2, dims, B, C, 0)
    np.testing.assert_allclose(lhs, rhs, atol=1e-12)


def test_mode_relabelling_invariance():
    """Relabelling the modes of X (and the factors with them) must not change the result:
    mode-2 MTTKRP of X equals mode-0 MTTKRP of X with modes (k,j,i)."""
    dims = (6, 7, 5)
    coords, vals = rand_coo(dims, 80)
    A, B = RNG.normal(size=(6, 3)), RNG.normal(size=(7, 3))
    m2 = oracle.mttkrp3(coords, vals, dims, A, B, 2)
    flipped = [coords[2], coords[1], coords[0]]
    m0 = oracle.mttkrp3(flipped, vals, (5, 7, 6), B, A, 0)
    np.testing.assert_allclose(m2, m0, atol=1e-13)
    U0, U1 = RNG.normal(size=(6, 2)), RNG.normal(size=(7, 4))
    y2 = oracle.ttmc3(coords, vals, dims, U0, U1, 2)                 # [k, x, y]
    y0 = oracle.ttmc3(flipped, vals, (5, 7, 6), U1, U0, 0)           # [k, y, x]
    np.testing.assert_allclose(y2, y0.transpose(0, 2, 1), atol=1e-13)


def test_input_order_independence():
    dims = (9, 8, 7)
    coords, vals = rand_coo(dims, 150)
    p = RNG.permutation(150)
    U2, U3 = RNG.normal(size=(8, 3)), RNG.normal(size=(7, 3))
    a = oracle.ttmc3(coords, vals, dims, U2, U3, 0)
    b = oracle.ttmc3([c[p] for c in coords], vals[p], dims, U2, U3, 0)
    S = oracle.ttmc3_abs(coords, vals, dims, U2, U3, 0)
    assert oracle.rel_err(b, a, S) < 1e-14


def test_fused_equals_unfused_tree():
    """The N-ary sum and the unfused binary sequence with whole intermediates (Fig. 3a)
    agree to rounding (Sec. 2.1 'Contraction tree')."""
    dims = (7, 9, 8)
    coords, vals = rand_coo(dims, 200)
    U2, U3 = RNG.normal(size=(9, 3)), RNG.normal(size=(8, 4))
    S = oracle.ttmc3_abs(coords, vals, dims, U2, U3, 0)
    assert oracle.rel_err(oracle.unfused_ttmc3(coords, vals, dims, U2, U3),
                          oracle.ttmc3(coords, vals, dims, U2, U3, 0), S) < 1e-13
    B, C = RNG.normal(size=(9, 5)), RNG.normal(size=(8, 5))
    S = oracle.mttkrp3_abs(coords, vals, dims, B, C, 0)
    assert oracle.rel_err(oracle.unfused_mttkrp3(coords, vals, dims, B, C),
                          oracle.mttkrp3(coords, vals, dims, B, C, 0), S) < 1e-13
    d4 = (4, 6, 5, 7)
    c4, v4 = rand_coo(d4, 150)
    U1, V2, V3 = RNG.normal(size=(6, 2)), RNG.normal(size=(5, 3)), RNG.normal(size=(7, 2))
    S = oracle.ttmc4_abs(c4, v4, d4, U1, V2, V3)
    assert oracle.rel_err(oracle.unfused_ttmc4(c4, v4, d4, U1, V2, V3),
                          oracle.ttmc4(c4, v4, d4, U1, V2, V3), S) < 1e-13
    udims, wdims = (6, 7, 5), (5, 8, 9)
    uc, uv = rand_coo(udims, 90)
    wc, wv = rand_coo(wdims, 110)
    V = RNG.normal(size=(7, 8))
    S = oracle.sptn3_abs(uc, uv, udims, V, wc, wv, wdims)
    assert oracle.rel_err(oracle.unfused_sptn3(uc, uv, udims, V, wc, wv, wdims),
                          oracle.sptn3(uc, uv, udims, V, wc, wv, wdims), S) < 1e-13


def test_abs_terms_is_sum_of_absolute_terms():
    dims = (4, 3, 5)
    coords, vals = rand_coo(dims, 25)
    U2, U3 = RNG.normal(size=(3, 2)), RNG.normal(size=(5, 2))
    S = oracle.ttmc3_abs(coords, vals, dims, U2, U3, 0)
    want = np.zeros_like(S)
    for n in range(len(vals)):
        i, j, k = (int(c[n]) for c in coords)
        want[i] += np.abs(vals[n] * np.outer(U2[j], U3[k]))
    np.testing.assert_allclose(S, want, atol=1e-14)
    # empty rows: sum|terms| == 0 and the value is exactly 0
    Y = oracle.ttmc3(coords, vals, dims, U2, U3, 0)
    assert np.all(Y[S == 0] == 0.0)


def test_rel_err_metric():
    want = np.array([1.0, 0.0, 2.0])
    S = np.array([4.0, 0.0, 2.0])
    assert oracle.rel_err(want + np.array([4e-10, 0, 0]), want, S) == pytest.approx(1e-10)
    assert oracle.rel_err(np.array([1.0, 1e-300, 2.0]), want, S) == np.inf


def test_bad_inputs_raise():
    dims = (3, 3, 3)
    coords = [np.array([0, 3], np.int32), np.array([0, 1], np.int32), np.array([0, 1], np.int32)]
    with pytest.raises(ValueError):
        oracle.ttmc3(coords, np.ones(2), dims, np.ones((3, 1)), np.ones((3, 1)), 0)


def test_empty_tensor_gives_zero():
    e = [np.zeros(0, np.int32)] * 3
    Y = oracle.ttmc3(e, np.zeros(0), (3, 4, 5), np.ones((4, 2)), np.ones((5, 2)), 0)
    assert Y.shape == (3, 2, 2) and not Y.any()


# ---------- a planted mistake must be caught by the pins above --------------------------------

def test_pins_catch_planted_mistakes():
    dims = (4, 5, 3)
    coords, vals = rand_coo(dims, 23)
    D = densify(coords, vals, dims)
    Fa, Fb = RNG.uniform(-1, 1, (5, 2)), RNG.uniform(-1, 1, (3, 2))
    want = brute_ttmc3(D, Fa, Fb, 0)
    good = oracle.ttmc3(coords, vals, dims, Fa, Fb, 0)
    # transposed rank operands, swapped coordinate modes, dropped nonzero
    bad1 = good.transpose(0, 2, 1)
    bad2 = oracle.ttmc3([coords[0], coords[1], (coords[2] + 1) % 3], vals, dims, Fa, Fb, 0)
    bad3 = oracle.ttmc3([c[:-1] for c in coords], vals[:-1], dims, Fa, Fb, 0)
    for bad in (bad1, bad2, bad3):
        assert np.abs(bad - want).max() > 1e-6
    assert np.abs(good - want).max() < 1e-13
