"""Pins of the N-ary reference (oracle/nary.py): brute-force loops over a densified tiny tensor
(the definition of Sec. 2.1 with nothing skipped), the independent C routines of the oracle for
the orders they cover, and properties the definition fixes."""
import itertools

import numpy as np

import oracle
from oracle import nary


def _tiny(seed, dims, nnz):
    rng = np.random.default_rng(seed)
    cells = rng.choice(int(np.prod(dims)), size=nnz, replace=False)
    coords = list(np.unravel_index(cells, dims))
    vals = rng.standard_normal(nnz)
    return [c.astype(np.int32) for c in coords], vals


def _brute(coords, vals, dims, x_idx, factors, out_idx, extents):
    """Every index combination, dense X, plain Python sums."""
    X = np.zeros(dims)
    X[tuple(coords)] = vals
    letters = sorted(set(x_idx) | set("".join(l for _, l in factors)) | set(out_idx))
    ext = dict(extents)
    for c, d in zip(x_idx, dims):
        ext[c] = d
    for arr, l in factors:
        for c, d in zip(l, arr.shape):
            ext[c] = d
    out = np.zeros([ext[c] for c in out_idx])
    for combo in itertools.product(*[range(ext[c]) for c in letters]):
        at = dict(zip(letters, combo))
        x = X[tuple(at[c] for c in x_idx)]
        if x == 0.0:
            continue
        t = x
        for arr, l in factors:
            t *= arr[tuple(at[c] for c in l)]
        out[tuple(at[c] for c in out_idx)] += t
    return out


def test_brute_force_order3_network_with_dense_only_and_two_letter_factors():
    dims = (3, 4, 2)
    coords, vals = _tiny(1, dims, 9)
    rng = np.random.default_rng(2)
    P = rng.standard_normal((4, 2, 3))          # P[j,k,r]
    D = rng.standard_normal((3, 2))             # D[r,q]: touches no mode of X
    ext = {"i": 3, "q": 2}
    got = nary.contract(coords, vals, "ijk", [(P, "jkr"), (D, "rq")], "qi", ext)
    want = _brute(coords, vals, dims, "ijk", [(P, "jkr"), (D, "rq")], "qi", ext)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-14)


def test_brute_force_order4_ttmc_and_full_contraction():
    dims = (2, 3, 2, 3)
    coords, vals = _tiny(3, dims, 11)
    rng = np.random.default_rng(4)
    U1, U2, U3 = rng.standard_normal((3, 2)), rng.standard_normal((2, 3)), rng.standard_normal((3, 2))
    f = [(U1, "ja"), (U2, "kb"), (U3, "lc")]
    ext = {"i": 2, "a": 2, "b": 3, "c": 2}
    np.testing.assert_allclose(nary.contract(coords, vals, "ijkl", f, "iabc", ext),
                               _brute(coords, vals, dims, "ijkl", f, "iabc", ext), rtol=1e-13, atol=1e-14)
    A = rng.standard_normal((2, 2))
    f2 = [(A, "ir"), (rng.standard_normal((3, 2)), "jr"), (rng.standard_normal((2, 2)), "kr"),
          (rng.standard_normal((3, 2)), "lr")]
    np.testing.assert_allclose(nary.contract(coords, vals, "ijkl", f2, "r", {"r": 2}),
                               _brute(coords, vals, dims, "ijkl", f2, "r", {"r": 2}), rtol=1e-13, atol=1e-14)


def test_agrees_with_c_routines_on_the_orders_they_cover():
    rng = np.random.default_rng(5)
    dims = (17, 13, 11)
    coords, vals = _tiny(6, dims, 400)
    U2, U3 = rng.standard_normal((13, 5)), rng.standard_normal((11, 7))
    got = nary.contract(coords, vals, "ijk", [(U2, "jr"), (U3, "ks")], "irs", {"i": 17, "r": 5, "s": 7})
    np.testing.assert_allclose(got, oracle.ttmc3(coords, vals, dims, U2, U3, 0), rtol=1e-12, atol=1e-13)
    B, C = rng.standard_normal((13, 6)), rng.standard_normal((11, 6))
    got = nary.contract(coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 17, "r": 6})
    np.testing.assert_allclose(got, oracle.mttkrp3(coords, vals, dims, B, C, 0), rtol=1e-12, atol=1e-13)
    A = rng.standard_normal((17, 6))
    got = nary.contract(coords, vals, "ijk", [(A, "ir"), (B, "jr")], "kr", {"k": 11, "r": 6})
    np.testing.assert_allclose(got, oracle.mttkrp3(coords, vals, dims, A, B, 2), rtol=1e-12, atol=1e-13)
    dims4 = (7, 6, 5, 4)
    c4, v4 = _tiny(7, dims4, 300)
    U1, U2, U3 = rng.standard_normal((6, 3)), rng.standard_normal((5, 2)), rng.standard_normal((4, 3))
    got = nary.contract(c4, v4, "ijkl", [(U1, "ja"), (U2, "kb"), (U3, "lc")], "iabc",
                        {"i": 7, "a": 3, "b": 2, "c": 3})
    np.testing.assert_allclose(got, oracle.ttmc4(c4, v4, dims4, U1, U2, U3), rtol=1e-12, atol=1e-13)


def test_chunking_and_output_letter_order_do_not_matter():
    rng = np.random.default_rng(8)
    dims = (9, 8, 7)
    coords, vals = _tiny(9, dims, 300)
    U2, U3 = rng.standard_normal((8, 3)), rng.standard_normal((7, 4))
    a = nary.contract(coords, vals, "ijk", [(U2, "jr"), (U3, "ks")], "irs", {"i": 9, "r": 3, "s": 4})
    b = nary.contract(coords, vals, "ijk", [(U2, "jr"), (U3, "ks")], "sir", {"i": 9, "r": 3, "s": 4})
    np.testing.assert_allclose(a, b.transpose(1, 2, 0), rtol=1e-13, atol=1e-14)
    old = nary._CHUNK
    try:
        nary._CHUNK = 7
        c = nary.contract(coords, vals, "ijk", [(U2, "jr"), (U3, "ks")], "irs", {"i": 9, "r": 3, "s": 4})
    finally:
        nary._CHUNK = old
    np.testing.assert_allclose(a, c, rtol=1e-13, atol=1e-14)


def test_single_nonzero_closed_form_and_abs_scale():
    coords = [np.array([2], dtype=np.int32), np.array([1], dtype=np.int32), np.array([0], dtype=np.int32)]
    vals = np.array([-3.0])
    B, C = np.arange(8.0).reshape(4, 2) - 3, np.arange(6.0).reshape(3, 2) + 1
    got = nary.contract(coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 5, "r": 2})
    want = np.zeros((5, 2))
    want[2] = -3.0 * B[1] * C[0]
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(nary.contract_abs(coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 5, "r": 2}),
                                  np.abs(want))
