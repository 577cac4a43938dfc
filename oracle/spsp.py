"""Products of several SPARSE tensors with a sparse result -- TEST INFRASTRUCTURE ONLY.

The three-index integral transformation of Sec. 5.1,
        E[K,i,m] = sum_{u,v} I[K,u,v] * C[u,i] * P[v,m]                    (unrestricted form)
        E[K,i,m] = sum_{u,v} I[K,u,v] * C[u,i] * P[v,m] * L[K,i]           (restricted form)
written out from the definition of Sec. 2.1: every tensor is zero outside its stored nonzeros, so
for one K the sum over u and v is the matrix product  C^T . I_K . P  of the densified operands
(numpy matmul, fp64).  The structure of the result is the join of Sec. 2.1: (K,i,m) is a
structural nonzero when at least one term exists, i.e. some u, v have I[K,u,v], C[u,i], P[v,m]
(and L[K,i]) all stored; computed with the same products over 0/1 matrices.

No CSF, no fusion, no sparse workspace: one dense slice per K.  Pinned in the CPU tests against
brute-force loops over the coordinate lists and against the N-ary routine of nary.py.
"""
import numpy as np


def _dense2(coo_coords, coo_vals, shape):
    d = np.zeros(shape, dtype=np.float64)
    d[np.asarray(coo_coords[0], dtype=np.int64), np.asarray(coo_coords[1], dtype=np.int64)] = coo_vals
    return d


def _pattern2(coo_coords, shape):
    d = np.zeros(shape, dtype=np.float64)
    d[np.asarray(coo_coords[0], dtype=np.int64), np.asarray(coo_coords[1], dtype=np.int64)] = 1.0
    return d


def chain3(I, C, P, dims, L=None, K_values=None):
    """E for the K in K_values (default: every K that holds a nonzero of I).

    I = (coords[3], vals) over (K,u,v); C = (coords[2], vals) over (u,i); P over (v,m);
    L (optional) over (K,i); dims = (n_K, n_i, n_u, n_m) with u and v sharing the extent n_u.
    Returns {K: (E_K, S_K, N_K)}: values, sum of |terms|, and the 0/1 structure, each n_i x n_m."""
    n_K, n_i, n_u, n_m = (int(d) for d in dims)
    (ik, iu, iv), ival = [np.asarray(c, dtype=np.int64) for c in I[0]], np.asarray(I[1], dtype=np.float64)
    Cd = _dense2(C[0], np.asarray(C[1], dtype=np.float64), (n_u, n_i))
    Pd = _dense2(P[0], np.asarray(P[1], dtype=np.float64), (n_u, n_m))
    Cp, Pp = _pattern2(C[0], (n_u, n_i)), _pattern2(P[0], (n_u, n_m))
    Ld = Lp = None
    if L is not None:
        Ld = _dense2(L[0], np.asarray(L[1], dtype=np.float64), (n_K, n_i))
        Lp = _pattern2(L[0], (n_K, n_i))
    order = np.argsort(ik, kind="stable")
    ik, iu, iv, ival = ik[order], iu[order], iv[order], ival[order]
    if K_values is None:
        K_values = np.unique(ik)
    out = {}
    for K in K_values:
        K = int(K)
        lo, hi = np.searchsorted(ik, K), np.searchsorted(ik, K + 1)
        IK = np.zeros((n_u, n_u), dtype=np.float64)
        IK[iu[lo:hi], iv[lo:hi]] = ival[lo:hi]
        IKp = np.zeros((n_u, n_u), dtype=np.float64)
        IKp[iu[lo:hi], iv[lo:hi]] = 1.0
        E = Cd.T @ IK @ Pd
        S = np.abs(Cd).T @ np.abs(IK) @ np.abs(Pd)
        N = (Cp.T @ IKp @ Pp) > 0.5                      # counts of terms: small integers, exact in fp64
        if L is not None:
            E = E * Ld[K][:, None]
            S = S * np.abs(Ld[K])[:, None]
            N = N & (Lp[K] > 0.5)[:, None]
        out[K] = (E, S, N)
    return out


def pair4(E_coords, E_vals, dims):
    """V[i,j,m,n] = sum_K E[K,i,m] * E[K,j,n]  (Sec. 5.1, the four-index integrals), dense.

    E over (K,i,m); dims = (n_K, n_i, n_m).  Returns (V, S, N) of shape n_i x n_j x n_m x n_n:
    with E_K flattened to a vector over (i,m), V is the sum over K of outer products."""
    n_K, n_i, n_m = (int(d) for d in dims)
    ek, ei, em = [np.asarray(c, dtype=np.int64) for c in E_coords]
    Ed = np.zeros((n_K, n_i * n_m), dtype=np.float64)
    Ed[ek, ei * n_m + em] = np.asarray(E_vals, dtype=np.float64)
    Ep = np.zeros((n_K, n_i * n_m), dtype=np.float64)
    Ep[ek, ei * n_m + em] = 1.0

    def shape4(G):                                       # [(i,m),(j,n)] -> [i,j,m,n]
        return G.reshape(n_i, n_m, n_i, n_m).transpose(0, 2, 1, 3)
    return shape4(Ed.T @ Ed), shape4(np.abs(Ed).T @ np.abs(Ed)), shape4((Ep.T @ Ep) > 0.5)


def pair4_block(E_coords, E_vals, dims, i, j):
    """One (i,j) block of V = E x E (Sec. 5.1, four-index integrals): V[i,j,:,:] = E_i^T . E_j with
    E_i the n_K x n_m matrix of the entries E[K,i,m].  Returns (V_ij, S_ij, N_ij), each n_m x n_m."""
    n_K, n_i, n_m = (int(d) for d in dims)
    ek, ei, em = [np.asarray(c, dtype=np.int64) for c in E_coords]
    ev = np.asarray(E_vals, dtype=np.float64)

    def slab(x):
        sel = ei == x
        D = np.zeros((n_K, n_m), dtype=np.float64)
        Pm = np.zeros((n_K, n_m), dtype=np.float64)
        D[ek[sel], em[sel]] = ev[sel]
        Pm[ek[sel], em[sel]] = 1.0
        return D, Pm
    Di, Pi = slab(i)
    Dj, Pj = slab(j)
    return Di.T @ Dj, np.abs(Di).T @ np.abs(Dj), (Pi.T @ Pj) > 0.5
