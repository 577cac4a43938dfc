"""Unfused binary-contraction sequences with full intermediates -- TEST INFRASTRUCTURE ONLY.

Each routine evaluates the contraction tree one binary contraction at a time,
materialising every intermediate tensor whole, as in the unfused code of
Fig. 3a (Sec. 2.2).  Intermediates are kept dense, so these are for small
tensors only; the tests use them to check that the direct (N-ary) oracle and
the tree agree (exploiting associativity and distributivity changes the order
of the sums, not their value: Sec. 2.1, "Contraction tree").
"""
import numpy as np


def _scatter(shape, index_arrays, values):
    T = np.zeros(shape, dtype=np.float64)
    np.add.at(T, tuple(index_arrays), values)
    return T


def unfused_ttmc3(coords, vals, dims, U2, U3):
    """T[i,j,s] = X[i,j,k] U3[k,s];  Y[i,r,s] = T[i,j,s] U2[j,r]   (mode-0 TTMc)."""
    i, j, k = [np.asarray(c, dtype=np.int64) for c in coords]
    R3 = U3.shape[1]
    T = np.zeros((dims[0], dims[1], R3), dtype=np.float64)
    np.add.at(T, (i, j), np.asarray(vals)[:, None] * U3[k, :])
    Y = np.zeros((dims[0], U2.shape[1], R3), dtype=np.float64)
    for jj in range(dims[1]):                     # Y[i,r,s] += U2[j,r] * T[i,j,s]
        Y += U2[jj][None, :, None] * T[:, jj, None, :]
    return Y


def unfused_mttkrp3(coords, vals, dims, B, C):
    """T[i,j,r] = X[i,j,k] C[k,r];  M[i,r] = T[i,j,r] B[j,r]   (mode-0 MTTKRP, r a batch index)."""
    i, j, k = [np.asarray(c, dtype=np.int64) for c in coords]
    R = C.shape[1]
    T = np.zeros((dims[0], dims[1], R), dtype=np.float64)
    np.add.at(T, (i, j), np.asarray(vals)[:, None] * C[k, :])
    M = np.zeros((dims[0], R), dtype=np.float64)
    for jj in range(dims[1]):
        M += T[:, jj, :] * B[jj][None, :]
    return M


def unfused_ttmc4(coords, vals, dims, U1, U2, U3):
    """T1[i,j,k,t] = X U3;  T2[i,j,s,t] = T1 U2;  Y[i,r,s,t] = T2 U1."""
    i, j, k, l = [np.asarray(c, dtype=np.int64) for c in coords]
    R1, R2, R3 = U1.shape[1], U2.shape[1], U3.shape[1]
    T1 = np.zeros((dims[0], dims[1], dims[2], R3), dtype=np.float64)
    np.add.at(T1, (i, j, k), np.asarray(vals)[:, None] * U3[l, :])
    T2 = np.zeros((dims[0], dims[1], R2, R3), dtype=np.float64)
    for kk in range(dims[2]):
        T2 += U2[kk][None, None, :, None] * T1[:, :, kk, None, :]
    Y = np.zeros((dims[0], R1, R2, R3), dtype=np.float64)
    for jj in range(dims[1]):
        Y += U1[jj][None, :, None, None] * T2[:, jj, None, :, :]
    return Y


def unfused_sptn3(ucoords, uvals, udims, V, wcoords, wvals, wdims):
    """T[i,k,l] = U[i,j,k] V[j,l];  Z[i,m] = T[i,k,l] W[k,l,m], T held whole."""
    ui, uj, uk = [np.asarray(c, dtype=np.int64) for c in ucoords]
    wk, wl, wm = [np.asarray(c, dtype=np.int64) for c in wcoords]
    L = V.shape[1]
    T = np.zeros((udims[0], udims[2], L), dtype=np.float64)
    np.add.at(T, (ui, uk), np.asarray(uvals)[:, None] * V[uj, :])
    Z = np.zeros((udims[0], wdims[2]), dtype=np.float64)
    contrib = T[:, wk, wl] * np.asarray(wvals)[None, :]          # Ni x nnzW
    for i in range(udims[0]):
        np.add.at(Z[i], wm, contrib[i])
    return Z
