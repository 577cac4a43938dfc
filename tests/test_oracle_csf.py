"""Pins for the reference CSF builder: a tree built node by node with Python
dictionaries, the round trip back to coordinates, structural invariants, and
the paper's mode-order example (Sec. 3.2: layout <d1,d2,d0> of A_ipq <=> dp_A =
(2,0,1), reference written A[p,q,i])."""
import itertools

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(777)


def rand_coo(dims, nnz):
    flat = RNG.choice(int(np.prod(dims)), size=nnz, replace=False)
    coords = np.unravel_index(flat, dims)
    return [c.astype(np.int32) for c in coords], RNG.uniform(-1, 1, nnz)


def tree_csf(coords, vals, mode_order):
    """CSF by nested dictionaries: level-l children of a node in ascending index order."""
    order = len(coords)
    root = {}
    for n in range(len(vals)):
        node = root
        for l in range(order):
            key = int(coords[mode_order[l]][n])
            if l == order - 1:
                assert key not in node
                node[key] = vals[n]
            else:
                node = node.setdefault(key, {})
    idx = [[] for _ in range(order)]
    ptr = [[0] for _ in range(order - 1)]
    out_vals = []

    def walk(node, l):
        for key in sorted(node):
            idx[l].append(key)
            if l == order - 1:
                out_vals.append(node[key])
            else:
                walk(node[key], l + 1)
                ptr[l].append(len(idx[l + 1]))
    walk(root, 0)
    return idx, ptr, out_vals


@pytest.mark.parametrize("dims,nnz", [((4, 5, 3), 30), ((3, 2, 4, 3), 40), ((6, 7), 20), ((9,), 5)])
def test_csf_matches_dictionary_tree_for_every_mode_order(dims, nnz):
    coords, vals = rand_coo(dims, nnz)
    for mo in itertools.permutations(range(len(dims))):
        idx, ptr, v, perm = oracle.csf_build(coords, vals, dims, list(mo))
        tidx, tptr, tv = tree_csf(coords, vals, mo)
        for l in range(len(dims)):
            assert idx[l].dtype == np.int32 and idx[l].tolist() == tidx[l]
        for l in range(len(dims) - 1):
            assert ptr[l].dtype == np.int64 and ptr[l].tolist() == tptr[l]
        assert v.tolist() == tv
        # round trip and invariants
        ex = oracle.csf_expand(idx, ptr, len(dims))
        for l, m in enumerate(mo):
            assert (ex[l] == np.asarray(coords[m])[perm]).all()
        for l in range(len(dims) - 1):
            assert ptr[l][0] == 0 and ptr[l][-1] == len(idx[l + 1])
            assert (np.diff(ptr[l]) >= 1).all()
            for p in range(len(idx[l])):
                ch = idx[l + 1][ptr[l][p]:ptr[l][p + 1]]
                assert (np.diff(ch) > 0).all()
        assert len(idx[-1]) == nnz


def test_mode_order_is_inverse_of_dp_example():
    """Sec. 3.2 example: A_ipq stored <d1,d2,d0> (dp_A0=2, dp_A1=0, dp_A2=1) is read A[p,q,i]:
    level 0 holds p values, level 1 q values, leaves i values."""
    coords = [np.array([5, 6], np.int32), np.array([0, 1], np.int32), np.array([3, 2], np.int32)]
    dp = [2, 0, 1]
    mode_order = [dp.index(l) for l in range(3)]
    assert mode_order == [1, 2, 0]
    idx, ptr, v, _ = oracle.csf_build(coords, np.array([1.0, 2.0]), (7, 2, 4), mode_order)
    assert idx[0].tolist() == [0, 1] and idx[1].tolist() == [3, 2] and idx[2].tolist() == [5, 6]
    assert v.tolist() == [1.0, 2.0]


def test_duplicates_and_range_rejected_and_empty_ok():
    c = [np.array([1, 1], np.int32), np.array([2, 2], np.int32)]
    with pytest.raises(ValueError):
        oracle.csf_build(c, np.ones(2), (3, 3), [0, 1])
    c = [np.array([1, 3], np.int32), np.array([2, 2], np.int32)]
    with pytest.raises(ValueError):
        oracle.csf_build(c, np.ones(2), (3, 3), [0, 1])
    e = [np.zeros(0, np.int32)] * 3
    idx, ptr, v, _ = oracle.csf_build(e, np.zeros(0), (3, 3, 3), [2, 0, 1])
    assert [len(a) for a in idx] == [0, 0, 0] and [p.tolist() for p in ptr] == [[0], [0]]
