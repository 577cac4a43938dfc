"""N-ary contraction of one sparse tensor with dense tensors -- TEST INFRASTRUCTURE ONLY.

The definition of Sec. 2.1 written out: the result element at the output indices is the sum,
over all remaining indices, of X's element times one element of every dense tensor; X
contributes only at its nonzeros.  No tree, no fusion, no intermediate: every nonzero's whole
product is formed and added to its output element (fp64).  `numpy.einsum` multiplies the
gathered factor entries of a chunk of nonzeros; `numpy.add.at` adds them up.

Used as the reference for contraction trees the C oracle has no routine for (other orders,
other trees over the same network); pinned in the CPU tests against the C routines and against
brute-force loops.
"""
import numpy as np

_CHUNK = 1 << 14


def contract(coords, vals, x_idx, factors, out_idx, extents):
    """out[out_idx] = sum_{other indices} X[x_idx] * prod_t F_t[idx_t].

    coords   one integer array per mode of X (COO, distinct coordinates)
    vals     values of the nonzeros
    x_idx    one letter per mode of X, e.g. "ijk"
    factors  list of (array, letters); letters may name modes of X and dense indices
    out_idx  letters of the result, X-mode letters and dense letters in any order
    extents  dict letter -> extent, for every letter of out_idx
    Returns a dense fp64 array of shape [extents[c] for c in out_idx]."""
    coords = [np.asarray(c, dtype=np.int64) for c in coords]
    vals = np.asarray(vals, dtype=np.float64)
    nnz = vals.shape[0]
    assert len(x_idx) == len(coords) and len(set(x_idx)) == len(x_idx)
    assert "n" not in x_idx and all("n" not in l for _, l in factors) and "n" not in out_idx
    out = np.zeros([int(extents[c]) for c in out_idx], dtype=np.float64)
    sparse_out = [c for c in out_idx if c in x_idx]
    dense_out = [c for c in out_idx if c not in x_idx]
    # result of one chunk: axis n, then the dense output letters
    chunk_sub = "n" + "".join(dense_out)
    for lo in range(0, nnz, _CHUNK):
        hi = min(nnz, lo + _CHUNK)
        operands, subs = [vals[lo:hi]], ["n"]
        for arr, letters in factors:
            arr = np.asarray(arr, dtype=np.float64)
            assert arr.ndim == len(letters)
            sp = [a for a, c in enumerate(letters) if c in x_idx]
            if sp:
                # entries of this factor at the chunk's coordinates: gather along its sparse axes
                moved = np.moveaxis(arr, sp, list(range(len(sp))))
                picked = moved[tuple(coords[x_idx.index(letters[a])][lo:hi] for a in sp)]
                operands.append(picked)
                subs.append("n" + "".join(c for c in letters if c not in x_idx))
            else:
                operands.append(arr)
                subs.append(letters)
        part = np.einsum(",".join(subs) + "->" + chunk_sub, *operands)
        if sparse_out:
            # scatter-add every nonzero's block to its output position
            view = out.transpose([out_idx.index(c) for c in sparse_out + dense_out])   # sparse axes first
            np.add.at(view, tuple(coords[x_idx.index(c)][lo:hi] for c in sparse_out), part)
        else:
            view = out.transpose([out_idx.index(c) for c in dense_out])
            view += part.sum(axis=0)
    return out


def contract_abs(coords, vals, x_idx, factors, out_idx, extents):
    """Sum of the absolute values of the terms (the scale of the error bound)."""
    return contract(coords, np.abs(np.asarray(vals, dtype=np.float64)), x_idx,
                    [(np.abs(np.asarray(a, dtype=np.float64)), l) for a, l in factors], out_idx, extents)
