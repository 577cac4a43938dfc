"""The five benchmark configurations and reduced copies of each, plus configuration 6: the
sparse three-index integral transformation of Sec. 5.1 on lattice sparse maps (a stand-in for
the quantum-chemistry inputs, which are not public), and configuration 7: the four-index product
V = E x E of the same section on a smaller lattice.

CONFIGS[c] are the full sizes; SMALL[c] keep the same recipe (distribution
family, skew, rank) at sizes a CPU loop finishes in seconds, chosen so that
slices, fibers and tiles are ragged (not multiples of any kernel tile).
Seeds: BASE_SEED + config number.
"""
from .generators import make_ttmc3, make_ttmc4, make_mttkrp3, make_sptn3, make_lattice_chain

BASE_SEED = 20240104


def _c1(device, **kw):
    n = kw.get("n", 200)
    return make_ttmc3("c1", BASE_SEED + 1,
                      [("uniform", n), ("uniform", n), ("uniform", n)],
                      kw.get("nnz", 8000), kw.get("ranks", (8, 8)), "u11", "u11", device)


def _c2(device, **kw):
    dims = kw.get("dims", (12000, 9000, 29000))
    return make_mttkrp3("c2", BASE_SEED + 2,
                        [("zipf", dims[0], 1.1), ("zipf", dims[1], 1.1), ("zipf", dims[2], 1.1)],
                        kw.get("nnz", 76_000_000), kw.get("rank", 32), "u01", "u11", device)


def _c3(device, **kw):
    dims = kw.get("dims", (1000, 50000, 50000, 2000))
    return make_ttmc4("c3", BASE_SEED + 3,
                      [("uniform", dims[0]), ("zipf", dims[1], 1.05), ("zipf", dims[2], 1.05),
                       ("zipf", dims[3], 1.05)],
                      kw.get("nnz", 40_000_000), kw.get("ranks", (16, 16, 16)), "n01", "n01", device)


def _c4(device, **kw):
    dims = kw.get("dims", (2000, 2000, 400, 2000, 400))
    nb = kw.get("nblocks", 20)
    grid = nb ** 3
    return make_sptn3("c4", BASE_SEED + 4, dims, nb,
                      kw.get("n_sel_u", round(0.08 * grid)), kw.get("n_sel_w", round(0.10 * grid)),
                      device)


def _c5(device, **kw):
    dims = kw.get("dims", (2_000_000, 2_000_000, 25_000))
    return make_ttmc3("c5", BASE_SEED + 5,
                      [("zipf", dims[0], 1.3), ("zipf", dims[1], 1.3), ("uniform", dims[2])],
                      kw.get("nnz", 140_000_000), kw.get("ranks", (64, 64)), "u11", "u11", device,
                      compact=True)


def _c6(device, **kw):
    # 32 x 32 atoms, 3 orbitals and 14 fitting functions per atom: I 14336 x 3072 x 3072 with ~8 M
    # nonzeros, result E with ~53 M (unrestricted) / ~40 M (restricted) structural nonzeros
    return make_lattice_chain("c6", BASE_SEED + 6, kw.get("side", 32), kw.get("n_ao", 3), kw.get("n_df", 14),
                              kw.get("r_int", 2.0), kw.get("r_mo", 2.0), kw.get("r_pao", 2.0),
                              kw.get("r_filter", 3.0), device=device)


def _c7(device, **kw):
    # the four-index product V = E x E of Sec. 5.1 on a 12 x 12 lattice (E: 1440 x 144 x 432 with ~4 M
    # structural nonzeros, made from these inputs by the three-index transformation; V: ~224 M)
    wl = make_lattice_chain("c7", BASE_SEED + 7, kw.get("side", 12), kw.get("n_ao", 3), kw.get("n_df", 10),
                            kw.get("r_int", 2.0), kw.get("r_mo", 2.0), kw.get("r_pao", 2.0),
                            kw.get("r_filter", 3.0), device=device)
    wl.kind = "sppair4"
    return wl


CONFIGS = {1: _c1, 2: _c2, 3: _c3, 4: _c4, 5: _c5, 6: _c6, 7: _c7}

# reduced copies: same recipe, sizes for CPU-second oracle runs
SMALL = {
    1: dict(),                                                       # C1 is already small
    2: dict(dims=(1203, 907, 2903), nnz=150_001, rank=32),
    3: dict(dims=(37, 1511, 1499, 211), nnz=60_007, ranks=(16, 16, 16)),
    4: dict(dims=(60, 80, 40, 60, 40), nblocks=4, n_sel_u=6, n_sel_w=7),
    5: dict(dims=(20_011, 19_997, 2503), nnz=200_003, ranks=(64, 64)),
    6: dict(side=5, n_df=6, r_int=1.5, r_pao=1.5, r_filter=2.5),
    7: dict(side=5, n_df=6, r_int=1.5, r_pao=1.5, r_filter=2.5),
}


def make(cid, device="cpu", small=False, **overrides):
    """Build configuration `cid` (1..7); small=True gives the reduced copy."""
    kw = dict(SMALL[cid]) if small else {}
    kw.update(overrides)
    return CONFIGS[cid](device, **kw)
