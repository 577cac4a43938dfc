"""Reference CSF construction -- TEST INFRASTRUCTURE ONLY.

CSF (Sec. 2.1, "CSF representation") stores a sparse tensor as a tree fixed by a
permutation of its modes: the nodes of level l hold the index values, in the
l-th mode of the permutation, of the distinct coordinate prefixes of length l+1;
leaves carry the values.  The paper gives no array layout (its figure is a
picture), so the layout below is this project's reading:

  level l (0 = outermost):  idx[l]  int32[nodes_l]   index value of each node
                            ptr[l]  int64[nodes_l+1] children of node p are the
                                    nodes ptr[l][p] .. ptr[l][p+1]-1 of level l+1
                                    (absent for the last level)
  vals fp64[nnz] aligned with the last level; no explicit root node;
  children of one parent are in strictly ascending index order.

Built the slow obvious way: sort the coordinate tuples lexicographically in
mode_order (numpy lexsort), then one scan that opens a new node at level l
whenever the prefix of length l+1 changes.
"""
import numpy as np


def csf_build(coords, vals, dims, mode_order):
    """Returns (idx list, ptr list, vals, perm) for the CSF with levels mode_order.

    Raises ValueError on an out-of-range or duplicated coordinate (the nonzero
    structure is a set, Sec. 2.1 "Sparse tensors")."""
    order = len(dims)
    if sorted(mode_order) != list(range(order)):
        raise ValueError("mode_order is not a permutation")
    cs = [np.asarray(c, dtype=np.int64) for c in coords]
    nnz = len(cs[0]) if order else 0
    for m in range(order):
        if nnz and (cs[m].min() < 0 or cs[m].max() >= dims[m]):
            raise ValueError("coordinate out of range in mode %d" % m)
    lv = [cs[m] for m in mode_order]                   # level l coordinates
    # np.lexsort sorts by the LAST key first: pass innermost level first
    perm = np.lexsort(tuple(lv[l] for l in reversed(range(order)))) if nnz else np.zeros(0, np.int64)
    s = [x[perm] for x in lv]
    # new[l][n]: the prefix of length l+1 of sorted tuple n differs from tuple n-1
    new = []
    diff_any = np.zeros(nnz, dtype=bool)
    for l in range(order):
        d = np.ones(nnz, dtype=bool)
        if nnz:
            d[1:] = s[l][1:] != s[l][:-1]
        diff_any = diff_any | d
        new.append(diff_any.copy())
    if nnz and not new[order - 1].all():
        raise ValueError("duplicate coordinate")
    idx, ptr = [], []
    for l in range(order):
        pos = np.flatnonzero(new[l])
        idx.append(s[l][pos].astype(np.int32))
        if l < order - 1:
            # child index of the first child of each node = number of level-(l+1)
            # nodes opened before it
            cnt = np.cumsum(new[l + 1]) - new[l + 1]          # exclusive count
            p = np.empty(len(pos) + 1, dtype=np.int64)
            p[:-1] = cnt[pos]
            p[-1] = int(new[l + 1].sum())
            ptr.append(p)
    v = np.asarray(vals, dtype=np.float64)[perm]
    return idx, ptr, v, perm


def csf_expand(idx, ptr, order):
    """Inverse of csf_build: the sorted coordinate list, one int64 array per level."""
    nnz = len(idx[order - 1])
    out = [None] * order
    out[order - 1] = idx[order - 1].astype(np.int64)
    # owner[l][n]: node of level l above leaf n
    child_owner = np.arange(nnz, dtype=np.int64)
    for l in reversed(range(order - 1)):
        counts = np.diff(ptr[l])
        node_of_child = np.repeat(np.arange(len(idx[l]), dtype=np.int64), counts)
        child_owner = node_of_child[child_owner]
        out[l] = idx[l].astype(np.int64)[child_owner]
    return out
