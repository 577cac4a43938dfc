"""Generators: coordinates, values and dense factors for the workload families.

Mode distributions are given as specs:
    ("uniform", N)        every index equally likely
    ("zipf", N, s)        P(rank r) ~ r**-s, r = 1..N, rank -> index through a
                          seeded permutation ("Zipf over shuffled indices")
Coordinates are made distinct by top-up rounds: draw a batch, keep the first
occurrence of every coordinate tuple (in draw order), draw the deficit again
from fresh counters, until exactly nnz distinct tuples exist.  Values are drawn
afterwards, indexed by final position.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np
import torch

from . import rng


@dataclass
class SparseCOO:
    """Order-n sparse tensor in coordinate form (structure of arrays)."""
    dims: Tuple[int, ...]
    coords: List[torch.Tensor]          # order x int32[nnz]
    vals: torch.Tensor                  # fp64[nnz]

    @property
    def order(self):
        return len(self.dims)

    @property
    def nnz(self):
        return int(self.vals.numel())

    def to(self, device):
        return SparseCOO(self.dims, [c.to(device) for c in self.coords], self.vals.to(device))

    def numpy(self):
        return [c.cpu().numpy() for c in self.coords], self.vals.cpu().numpy()


@dataclass
class Workload:
    """One problem instance: its kind, sparse operands, dense factors and sizes."""
    kind: str                            # "ttmc3" | "ttmc4" | "mttkrp3" | "sptn3"
    name: str
    sparse: Dict[str, SparseCOO]
    dense: Dict[str, torch.Tensor]
    params: Dict[str, object] = field(default_factory=dict)


def zipf_cdf(n, s):
    """Cumulative probabilities of P(r) ~ r**-s over ranks 1..n, as fp64 (host numpy)."""
    w = np.arange(1, n + 1, dtype=np.float64) ** (-float(s))
    c = np.cumsum(w)
    c /= c[-1]
    c[-1] = 1.0
    return torch.from_numpy(c)


def _draw_mode(seed, stream, start, count, spec, device, cache):
    kind = spec[0]
    n = int(spec[1])
    if kind == "uniform":
        return rng.uniform_int(seed, stream, start, count, n, device)
    if kind == "zipf":
        key = (stream, "zipf")
        if key not in cache:
            cache[key] = (zipf_cdf(n, spec[2]).to(device),
                          rng.permutation(seed, stream + "/perm", n, device))
        cdf, perm = cache[key]
        u = rng.uniform01(seed, stream, start, count, device)
        rank = torch.clamp(torch.searchsorted(cdf, u, right=True), max=n - 1)
        return perm[rank]
    raise ValueError("unknown mode spec %r" % (spec,))


def _keep_first(keys):
    """Indices (ascending) of the first occurrence of every distinct key."""
    order = torch.sort(keys, stable=True)
    sk, perm = order.values, order.indices
    first = torch.ones_like(sk, dtype=torch.bool)
    first[1:] = sk[1:] != sk[:-1]
    return torch.sort(perm[first]).values


def distinct_coords(seed, name, specs, nnz, device="cpu", forced_first=None):
    """nnz distinct coordinate tuples; returns order x int32[nnz] in draw order.

    forced_first = (mode, count): the first `count` draws take index 0..count-1
    in that mode (so that every index of the mode is present).
    """
    dims = [int(s[1]) for s in specs]
    total = 1
    for d in dims:
        total *= d
    if total >= 1 << 62:
        raise ValueError("coordinate key does not fit 62 bits")
    if nnz > total:
        raise ValueError("more nonzeros than cells")
    strides = []
    acc = 1
    for d in reversed(dims):
        strides.append(acc)
        acc *= d
    strides = strides[::-1]
    cache = {}
    kept = torch.empty(0, dtype=torch.int64, device=device)
    start = 0
    while kept.numel() < nnz:
        need = nnz - kept.numel()
        batch = need + need // 3 + 1024
        key = torch.zeros(batch, dtype=torch.int64, device=device)
        for m, spec in enumerate(specs):
            c = _draw_mode(seed, "%s/mode%d" % (name, m), start, batch, spec, device, cache)
            if forced_first is not None and forced_first[0] == m and start < forced_first[1]:
                k = min(forced_first[1] - start, batch)
                c[:k] = torch.arange(start, start + k, dtype=torch.int64, device=device)
            key += c * strides[m]
        start += batch
        allk = torch.cat([kept, key])
        kept = allk[_keep_first(allk)]
    kept = kept[:nnz]
    out = []
    for m in range(len(dims)):
        out.append(((kept // strides[m]) % dims[m]).to(torch.int32))
    return out


def block_sparse_coords(seed, name, dims, nblocks, n_selected, device="cpu"):
    """Block-sparse structure: an nblocks^order grid of equal blocks, n_selected of
    them (sampled without replacement) dense inside.  COO order: selected blocks in
    selection order, row-major inside a block."""
    order = len(dims)
    bs = [d // nb for d, nb in zip(dims, nblocks)]
    for d, nb, b in zip(dims, nblocks, bs):
        if b * nb != d:
            raise ValueError("extent not divisible by block count")
    grid = 1
    for nb in nblocks:
        grid *= nb
    sel = rng.permutation(seed, name + "/blocks", grid, device)[:n_selected]
    vol = 1
    for b in bs:
        vol *= b
    nnz = n_selected * vol
    e = torch.arange(nnz, dtype=torch.int64, device=device)
    blk = sel[e // vol]
    r = e % vol
    coords = [None] * order
    for m in reversed(range(order)):
        inner = r % bs[m]
        r = r // bs[m]
        bcoord = blk % nblocks[m]
        blk = blk // nblocks[m]
        coords[m] = (bcoord * bs[m] + inner).to(torch.int32)
    return coords


def sparse_values(seed, name, nnz, dist, device="cpu"):
    """Nonzero values: 'u01' U(0,1) with 0 excluded, 'u11' U(-1,1), 'n01' N(0,1)."""
    if dist == "u01":
        v = 1.0 - rng.uniform01(seed, name + "/vals", 0, nnz, device)      # (0,1]
    elif dist == "u11":
        v = 2.0 * rng.uniform01(seed, name + "/vals", 0, nnz, device) - 1.0
    elif dist == "n01":
        v = rng.normal(seed, name + "/vals", 0, nnz, device)
    else:
        raise ValueError(dist)
    # stored values are structural nonzeros; never emit an exact 0.0
    return torch.where(v == 0.0, torch.full_like(v, 2.0 ** -60), v)


def dense_factor(seed, name, rows, cols, dist, device="cpu"):
    """Row-major dense rows x cols fp64 factor."""
    n = rows * cols
    if dist == "u11":
        v = 2.0 * rng.uniform01(seed, name + "/dense", 0, n, device) - 1.0
    elif dist == "n01":
        v = rng.normal(seed, name + "/dense", 0, n, device)
    elif dist == "u01":
        v = rng.uniform01(seed, name + "/dense", 0, n, device)
    else:
        raise ValueError(dist)
    return v.reshape(rows, cols).contiguous()


def make_ttmc3(name, seed, specs, nnz, ranks, val_dist, fac_dist, device="cpu", compact=False):
    """Y[i,r2,r3] = X[i,j,k] U2[j,r2] U3[k,r3]  (Sec. 5.3, first TTMc)."""
    dims = tuple(int(s[1]) for s in specs)
    coords = distinct_coords(seed, name + "/X", specs, nnz, device)
    X = SparseCOO(dims, coords, sparse_values(seed, name + "/X", nnz, val_dist, device))
    U2 = dense_factor(seed, name + "/U2", dims[1], ranks[0], fac_dist, device)
    U3 = dense_factor(seed, name + "/U3", dims[2], ranks[1], fac_dist, device)
    return Workload("ttmc3", name, {"X": X}, {"U2": U2, "U3": U3},
                    {"ranks": tuple(ranks), "compact": bool(compact), "seed": seed})


def make_ttmc4(name, seed, specs, nnz, ranks, val_dist, fac_dist, device="cpu", dense_mode0=True):
    """Y[i,r1,r2,r3] = X[i,j,k,l] U1[j,r1] U2[k,r2] U3[l,r3] (order-4 form of Sec. 5.3)."""
    dims = tuple(int(s[1]) for s in specs)
    forced = (0, min(dims[0], nnz)) if dense_mode0 else None
    coords = distinct_coords(seed, name + "/X", specs, nnz, device, forced_first=forced)
    X = SparseCOO(dims, coords, sparse_values(seed, name + "/X", nnz, val_dist, device))
    U1 = dense_factor(seed, name + "/U1", dims[1], ranks[0], fac_dist, device)
    U2 = dense_factor(seed, name + "/U2", dims[2], ranks[1], fac_dist, device)
    U3 = dense_factor(seed, name + "/U3", dims[3], ranks[2], fac_dist, device)
    return Workload("ttmc4", name, {"X": X}, {"U1": U1, "U2": U2, "U3": U3},
                    {"ranks": tuple(ranks), "seed": seed})


def make_mttkrp3(name, seed, specs, nnz, rank, val_dist, fac_dist, device="cpu"):
    """M0[i,r] = X[i,j,k] B[j,r] C[k,r] and M2[k,r] = X[i,j,k] A[i,r] B[j,r] (Sec. 5.2)."""
    dims = tuple(int(s[1]) for s in specs)
    coords = distinct_coords(seed, name + "/X", specs, nnz, device)
    X = SparseCOO(dims, coords, sparse_values(seed, name + "/X", nnz, val_dist, device))
    A = dense_factor(seed, name + "/A", dims[0], rank, fac_dist, device)
    B = dense_factor(seed, name + "/B", dims[1], rank, fac_dist, device)
    C = dense_factor(seed, name + "/C", dims[2], rank, fac_dist, device)
    return Workload("mttkrp3", name, {"X": X}, {"A": A, "B": B, "C": C},
                    {"rank": int(rank), "seed": seed})


def make_sptn3(name, seed, dims_ijklm, nblocks, n_sel_u, n_sel_w, device="cpu"):
    """Z[i,m] = U[i,j,k] V[j,l] W[k,l,m] (Sec. 1), U and W block-sparse, V dense."""
    I, J, K, L, M = dims_ijklm
    nb = nblocks
    cu = block_sparse_coords(seed, name + "/U", (I, J, K), (nb, nb, nb), n_sel_u, device)
    cw = block_sparse_coords(seed, name + "/W", (K, L, M), (nb, nb, nb), n_sel_w, device)
    U = SparseCOO((I, J, K), cu, sparse_values(seed, name + "/U", cu[0].numel(), "n01", device))
    W = SparseCOO((K, L, M), cw, sparse_values(seed, name + "/W", cw[0].numel(), "n01", device))
    V = dense_factor(seed, name + "/V", J, L, "n01", device)
    return Workload("sptn3", name, {"U": U, "W": W}, {"V": V},
                    {"dims": tuple(dims_ijklm), "seed": seed})


def make_sptn3_scattered(name, seed, dims_ijklm, nnz_u, nnz_w, device="cpu"):
    """Same network as make_sptn3 with U and W scattered (uniform distinct coordinates, no block
    structure): the fibers of neighbouring slices share few indices."""
    I, J, K, L, M = dims_ijklm
    cu = distinct_coords(seed, name + "/U", [("uniform", I), ("uniform", J), ("uniform", K)], nnz_u, device)
    cw = distinct_coords(seed, name + "/W", [("uniform", K), ("uniform", L), ("uniform", M)], nnz_w, device)
    U = SparseCOO((I, J, K), cu, sparse_values(seed, name + "/U", cu[0].numel(), "n01", device))
    W = SparseCOO((K, L, M), cw, sparse_values(seed, name + "/W", cw[0].numel(), "n01", device))
    V = dense_factor(seed, name + "/V", J, L, "n01", device)
    return Workload("sptn3", name, {"U": U, "W": W}, {"V": V},
                    {"dims": tuple(dims_ijklm), "seed": seed})


def _disc_offsets(radius):
    """Integer offsets (dx, dy) with dx^2 + dy^2 <= radius^2, in row-major order."""
    r = int(radius)
    return [(dx, dy) for dx in range(-r, r + 1) for dy in range(-r, r + 1) if dx * dx + dy * dy <= radius * radius]


def _atom_pairs(side, radius, device):
    """All ordered atom pairs (a, b) of a side x side lattice within `radius` (no wrap-around)."""
    atoms = torch.arange(side * side, dtype=torch.int64, device=device)
    ax, ay = atoms // side, atoms % side
    pa, pb = [], []
    for dx, dy in _disc_offsets(radius):
        bx, by = ax + dx, ay + dy
        ok = (bx >= 0) & (bx < side) & (by >= 0) & (by < side)
        pa.append(atoms[ok])
        pb.append((bx * side + by)[ok])
    return torch.cat(pa), torch.cat(pb)


def _thin(seed, stream, count, keep, device):
    """Seeded keep/drop decision per position."""
    if keep >= 1.0:
        return torch.ones(count, dtype=torch.bool, device=device)
    return rng.uniform01(seed, stream, 0, count, device) < keep


def _expand_pairs(pa, pb, na, nb):
    """Atom pairs -> function pairs: every one of `na` functions on a with every one of `nb` on b."""
    n = pa.numel()
    fa = torch.arange(na, device=pa.device).repeat_interleave(nb).repeat(n)
    fb = torch.arange(nb, device=pa.device).repeat(na).repeat(n)
    return (pa.repeat_interleave(na * nb) * na + fa), (pb.repeat_interleave(na * nb) * nb + fb)


def make_lattice_chain(name, seed, side, n_ao, n_df, r_int, r_mo, r_pao, r_filter,
                       keep_int=0.7, keep_mo=0.85, keep_pao=0.85, device="cpu"):
    """E[K,i,m] = I[K,u,v] C[u,i] P[v,m] (x L[K,i]): the sparse three-index integral transformation
    of Sec. 5.1 on synthetic sparse maps.  Atoms sit on a side x side square lattice; every atom
    carries one localized orbital (index i), n_ao atomic orbitals (u, v), n_ao projected atomic
    orbitals (m) and n_df fitting functions (K).  An entry is structurally nonzero when the atoms
    of its indices lie within a cut-off radius of each other (lattice units), thinned at random:
        I[K,u,v]  K-u, K-v and u-v within r_int, kept with probability keep_int
        C[u,i]    within r_mo,  kept with probability keep_mo
        P[v,m]    within r_pao, kept with probability keep_pao
        L[K,i]    within r_filter, all ones (the K -> i sparse map used as a filter)
    Values N(0,1).  Stands in for the quantum-chemistry inputs of Sec. 5.1, which are not public."""
    atoms = side * side
    n_i, n_u, n_m, n_K = atoms, atoms * n_ao, atoms * n_ao, atoms * n_df
    # I: atom triples (aK, au, av), pairwise within r_int
    ka, ua = _atom_pairs(side, r_int, device)               # (aK, au)
    trip_k, trip_u, trip_v = [], [], []
    kx, ky = ka // side, ka % side
    ux, uy = ua // side, ua % side
    for dx, dy in _disc_offsets(r_int):
        vx, vy = kx + dx, ky + dy
        ok = (vx >= 0) & (vx < side) & (vy >= 0) & (vy < side)
        ok &= ((vx - ux) ** 2 + (vy - uy) ** 2) <= r_int * r_int
        trip_k.append(ka[ok]); trip_u.append(ua[ok]); trip_v.append((vx * side + vy)[ok])
    tk, tu, tv = torch.cat(trip_k), torch.cat(trip_u), torch.cat(trip_v)
    nt = tk.numel()
    per = n_df * n_ao * n_ao
    f = torch.arange(per, device=device)
    fK, fu, fv = f // (n_ao * n_ao), (f // n_ao) % n_ao, f % n_ao
    cK = (tk.repeat_interleave(per) * n_df + fK.repeat(nt))
    cu = (tu.repeat_interleave(per) * n_ao + fu.repeat(nt))
    cv = (tv.repeat_interleave(per) * n_ao + fv.repeat(nt))
    keep = _thin(seed, name + "/I/keep", cK.numel(), keep_int, device)
    ci = [cK[keep].to(torch.int32), cu[keep].to(torch.int32), cv[keep].to(torch.int32)]
    I = SparseCOO((n_K, n_u, n_u), ci, sparse_values(seed, name + "/I", ci[0].numel(), "n01", device))

    def pair_tensor(tag, radius, na, nb, keep_p, dims, ones=False):
        pa, pb = _atom_pairs(side, radius, device)
        ca, cb = _expand_pairs(pa, pb, na, nb)
        k = _thin(seed, name + "/" + tag + "/keep", ca.numel(), keep_p, device)
        cc = [ca[k].to(torch.int32), cb[k].to(torch.int32)]
        vals = (torch.ones(cc[0].numel(), dtype=torch.float64, device=device) if ones
                else sparse_values(seed, name + "/" + tag, cc[0].numel(), "n01", device))
        return SparseCOO(dims, cc, vals)

    C = pair_tensor("C", r_mo, n_ao, 1, keep_mo, (n_u, n_i))
    P = pair_tensor("P", r_pao, n_ao, n_ao, keep_pao, (n_u, n_m))
    L = pair_tensor("L", r_filter, n_df, 1, 1.0, (n_K, n_i), ones=True)
    return Workload("spchain3", name, {"I": I, "C": C, "P": P, "L": L}, {},
                    {"dims": (n_K, n_i, n_u, n_m), "side": side, "seed": seed})
