"""Full-size parity (configurations 2-5 at the sizes the benchmark times): CSF arrays
bit-exact against an independent sort-based build, and outputs against the CPU oracle: whole
for the order-4 TTMc (every slice is cut into many work items) and the three-tensor network; for
the 47 GB output of the skewed order-3 TTMc sampled light slices whole, one row and one column of
the block of EVERY slice above 60 000 leaves, and the heaviest slice (15.8 M leaves) whole."""
import numpy as np
import pytest
import torch

import oracle
import paper_2401_04836_amd as cst
import workloads as w
from paper_2401_04836_amd import schedules as S
from helpers import TOL

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


def reference_levels(coords, vals, dims, mode_order):
    """Level arrays from a torch sort + run detection (test infrastructure, GPU tensors)."""
    order = len(dims)
    key = torch.zeros_like(coords[0], dtype=torch.int64)
    for m in mode_order:
        key = key * int(dims[m]) + coords[m].long()
    skey, perm = torch.sort(key, stable=True)
    lv = [coords[m][perm] for m in mode_order]
    idx, ptr = [], []
    strides = []
    acc = 1
    for m in reversed(mode_order):
        strides.append(acc)
        acc *= int(dims[m])
    strides = strides[::-1]                       # stride of level l inside the key
    heads = []
    for l in range(order):
        pref = skey // strides[l]
        h = torch.ones_like(pref, dtype=torch.bool)
        h[1:] = pref[1:] != pref[:-1]
        heads.append(h)
        idx.append(lv[l][h])
    for l in range(order - 1):
        below = torch.cumsum(heads[l + 1].long(), 0) - heads[l + 1].long()    # exclusive rank
        p = torch.cat([below[heads[l]], heads[l + 1].sum().reshape(1)])
        ptr.append(p)
    return idx, ptr, vals[perm]


def check_csf_full(csf, coords, vals, dims, mode_order):
    idx, ptr, v = reference_levels(coords, vals, dims, mode_order)
    for l in range(len(dims)):
        gi, gp, gv = csf.export(l)
        assert torch.equal(gi, idx[l]), "idx level %d" % l
        if l < len(dims) - 1:
            assert torch.equal(gp, ptr[l]), "ptr level %d" % l
        else:
            assert torch.equal(gv.view(torch.int64), v.view(torch.int64)), "vals"


def slice_sizes(csf):
    """Leaves under every root node."""
    below = None
    for l in reversed(range(csf.order - 1)):
        p = csf.export(l)[1]
        below = p if below is None else below[p]
    return below[1:] - below[:-1]


def pick_slices(sizes, n_light=24, seed=0):
    """Ordinals of sampled root slices: the heaviest, a few mid-size, random light ones."""
    g = torch.Generator().manual_seed(seed)
    order = torch.argsort(sizes.cpu(), descending=True)
    n = order.numel()
    picks = set(order[:2].tolist())
    picks.update(order[[n // 100, n // 20, n // 4, n // 2, n - 1]].tolist())
    picks.update(order[torch.randint(0, n, (n_light,), generator=g)].tolist())
    # slices made of a few work items (sizes just above the split length)
    sz = sizes.cpu()
    for target in (5_000, 9_000, 20_000, 50_000):
        picks.add(int(torch.argmin((sz - target).abs())))
    return sorted(picks)


def subset(coo_coords, coo_vals, mode, root_values):
    """COO entries whose `mode` index is in root_values, with that index renumbered 0..len-1."""
    rv = torch.as_tensor(root_values, device=coo_coords[0].device, dtype=torch.int64)
    lut = torch.full((int(coo_coords[mode].max()) + 2,), -1, dtype=torch.int64, device=rv.device)
    lut[rv] = torch.arange(rv.numel(), device=rv.device)
    new = lut[coo_coords[mode].long()]
    keep = new >= 0
    cs = [c[keep].cpu().numpy() for c in coo_coords]
    cs[mode] = new[keep].to(torch.int32).cpu().numpy()
    return cs, coo_vals[keep].cpu().numpy()


def test_config2_mttkrp_full_size_both_modes():
    _say("config 2 full size: generate")
    wl = w.make(2, device="cuda")
    X = wl.sparse["X"]
    A, B, C = wl.dense["A"], wl.dense["B"], wl.dense["C"]
    cn = [c.cpu().numpy() for c in X.coords]
    vn = X.vals.cpu().numpy()
    for mode, mo, sched, facs, names in (
            (0, [0, 1, 2], S.MTTKRP3, (C, B), ("C", "B")),
            (2, [2, 1, 0], "T[k,j,r] = X[k,j,i] * A[i,r] | k,j,i,r ; M[k,r] = T[k,j,r] * B[j,r] | k,j,r",
             (A, B), ("A", "B"))):
        _say("config 2 mode %d: CSF %s" % (mode, mo))
        csf = cst.build_csf(X.coords, X.vals, X.dims, mo)
        check_csf_full(csf, X.coords, X.vals, X.dims, mo)
        pl = cst.plan(sched, [("X", csf), (names[0], facs[0]), (names[1], facs[1])])
        out = cst.execute(pl, list(facs)).reshape(pl.n_rows, -1)
        torch.cuda.synchronize()
        _say("config 2 mode %d: oracle over all %d nonzeros" % (mode, X.nnz))
        others = [m for m in range(3) if m != mode]
        Fa, Fb = ([A, B, C][others[0]].cpu().numpy(), [A, B, C][others[1]].cpu().numpy())
        want = oracle.mttkrp3(cn, vn, X.dims, Fa, Fb, mode)
        S_abs = oracle.mttkrp3_abs(cn, vn, X.dims, Fa, Fb, mode)
        err = oracle.rel_err(out.cpu().numpy(), want, S_abs)
        _say("  rel err %.3e" % err)
        assert err <= TOL
        pl.check()                                          # the plan's tables at full size
        # the same contraction on the generic executor with the leaf-level producer inlined (segments of 512
        # leaves, the heaviest slices added by a workgroup)
        gen = cst.plan(sched, [("X", csf), (names[0], facs[0]), (names[1], facs[1])], options="force_generic=1")
        assert "inlined_producers=1" in gen.describe(), gen.describe()
        gen.check()
        out = cst.execute(gen, list(facs)).reshape(gen.n_rows, -1)
        torch.cuda.synchronize()
        err = oracle.rel_err(out.cpu().numpy(), want, S_abs)
        _say("  generic executor, fused pair: rel err %.3e" % err)
        assert err <= TOL
        del pl, gen, csf, out


def test_config2_mttkrp_other_modes_on_the_mode0_csf():
    """Modes 1 and 2 without re-rooting the CSF (Sec. 5.3 runs every mode): results indexed by the
    middle and by the leaf level, added into a dense array."""
    _say("config 2 full size, one CSF for every mode: generate")
    wl = w.make(2, device="cuda")
    X = wl.sparse["X"]
    A, B, C = wl.dense["A"], wl.dense["B"], wl.dense["C"]
    cn = [c.cpu().numpy() for c in X.coords]
    vn = X.vals.cpu().numpy()
    csf = cst.build_csf(X.coords, X.vals, X.dims, [0, 1, 2])
    for mode, sched, ops in (
            (1, "T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; M[j,r] = T[i,j,r] * A[i,r] | i,j,r", (("C", C), ("A", A))),
            (2, "T[i,j,r] = A[i,r] * B[j,r] | i,j,r ; M[k,r] = X[i,j,k] * T[i,j,r] | i,j,k,r", (("A", A), ("B", B)))):
        for options in (None, "reroot=0"):
            pl = cst.plan(sched, [("X", csf)] + list(ops), options=options)
            _say("config 2 mode %d on CSF [0,1,2]: %s" % (mode, pl.describe().split("|")[0]))
            assert ("family=generic" in pl.describe()) == (options is not None)
            facs = [t for _, t in ops]
            out = cst.execute(pl, facs)
            torch.cuda.synchronize()
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0.record()
            out = cst.execute(pl, facs)
            t1.record()
            torch.cuda.synchronize()
            _say("  %.2f ms per contraction" % t0.elapsed_time(t1))
            out = out.reshape(X.dims[mode], -1)
            others = [m for m in range(3) if m != mode]
            Fa, Fb = ([A, B, C][others[0]].cpu().numpy(), [A, B, C][others[1]].cpu().numpy())
            want = oracle.mttkrp3(cn, vn, X.dims, Fa, Fb, mode)
            S_abs = oracle.mttkrp3_abs(cn, vn, X.dims, Fa, Fb, mode)
            err = oracle.rel_err(out.cpu().numpy(), want, S_abs)
            _say("  rel err %.3e" % err)
            assert err <= TOL
            del pl, out


def test_config5_ttmc3_full_size_compact():
    _say("config 5 full size: generate")
    wl = w.make(5, device="cuda")
    X = wl.sparse["X"]
    U2, U3 = wl.dense["U2"], wl.dense["U3"]
    csf = cst.build_csf(X.coords, X.vals, X.dims, [0, 1, 2])
    _say("config 5: CSF check")
    check_csf_full(csf, X.coords, X.vals, X.dims, [0, 1, 2])
    pl = cst.plan(S.TTMC3, [("X", csf), ("U3", U3), ("U2", U2)], flags=cst.OUT_COMPACT)
    csf.check()
    pl.check()                                              # rows, K-steps, batches and partial blocks at full size
    out = cst.execute(pl, [U3, U2]).reshape(pl.n_rows, 64, 64)
    torch.cuda.synchronize()
    rows = pl.output_rows()
    sizes = slice_sizes(csf)
    assert int(sizes.sum()) == X.nnz and rows.numel() == pl.n_rows
    picks = pick_slices(sizes)
    U2n, U3n = U2.cpu().numpy(), U3.cpu().numpy()
    light = [p for p in picks if int(sizes[p]) <= 60_000]
    heavy = [p for p in picks if int(sizes[p]) > 60_000]
    _say("config 5: %d whole slices (up to %d leaves), %d heavy slices by elements (up to %d leaves)"
         % (len(light), max(int(sizes[p]) for p in light), len(heavy), max([int(sizes[p]) for p in heavy] + [0])))
    cs, vs = subset(X.coords, X.vals, 0, rows[light].long())
    dims = (len(light), X.dims[1], X.dims[2])
    want = oracle.ttmc3(cs, vs, dims, U2n, U3n, 0)
    S_abs = oracle.ttmc3_abs(cs, vs, dims, U2n, U3n, 0)
    err = oracle.rel_err(out[light].cpu().numpy(), want, S_abs)
    _say("  whole slices rel err %.3e" % err)
    assert err <= TOL
    # EVERY slice above 60 000 leaves (the slices cut into many work items, where partial row blocks are
    # added by the fix-up pass): one whole row and one whole column of its 64 x 64 block, and four corners
    heavy = torch.nonzero(sizes > 60_000).flatten().tolist()
    _say("config 5: %d slices above 60 000 leaves (%d leaves in all), a row and a column of every block"
         % (len(heavy), int(sizes[heavy].sum())))
    cs, vs = subset(X.coords, X.vals, 0, rows[heavy].long())
    dims = (len(heavy), X.dims[1], X.dims[2])
    got = out[heavy].cpu().numpy()
    for r2 in (17,):
        want = oracle.ttmc3(cs, vs, dims, U2n[:, [r2]], U3n, 0)[:, 0, :]
        S_abs = oracle.ttmc3_abs(cs, vs, dims, U2n[:, [r2]], U3n, 0)[:, 0, :]
        err = oracle.rel_err(got[:, r2, :], want, S_abs)
        _say("  heavy slices, row %d of every block: rel err %.3e" % (r2, err))
        assert err <= TOL
    for r3 in (42,):
        want = oracle.ttmc3(cs, vs, dims, U2n, U3n[:, [r3]], 0)[:, :, 0]
        S_abs = oracle.ttmc3_abs(cs, vs, dims, U2n, U3n[:, [r3]], 0)[:, :, 0]
        err = oracle.rel_err(got[:, :, r3], want, S_abs)
        _say("  heavy slices, column %d of every block: rel err %.3e" % (r3, err))
        assert err <= TOL
    for r2, r3 in ((0, 0), (63, 63), (0, 63), (63, 0)):
        want = oracle.ttmc3(cs, vs, dims, U2n[:, [r2]], U3n[:, [r3]], 0)[:, 0, 0]
        S_abs = oracle.ttmc3_abs(cs, vs, dims, U2n[:, [r2]], U3n[:, [r3]], 0)[:, 0, 0]
        assert oracle.rel_err(got[:, r2, r3], want, S_abs) <= TOL
    # the heaviest slice whole: its nonzeros are dealt to 64 pseudo-slices so that the oracle's row-parallel
    # loop uses every core, and the 64 partial blocks are added here (the order of addition is free)
    top = int(torch.argmax(sizes))
    sel = X.coords[0] == rows[top]
    cj, ck, v = (t[sel].cpu().numpy() for t in (X.coords[1], X.coords[2], X.vals))
    _say("config 5: the heaviest slice whole (%d leaves)" % v.size)
    part = (np.arange(v.size) % 64).astype(np.int32)
    want = oracle.ttmc3([part, cj, ck], v, (64, X.dims[1], X.dims[2]), U2n, U3n, 0).sum(0)
    S_abs = oracle.ttmc3_abs([part, cj, ck], v, (64, X.dims[1], X.dims[2]), U2n, U3n, 0).sum(0)
    err = oracle.rel_err(out[top].cpu().numpy(), want, S_abs)
    _say("  heaviest slice, all 4096 elements: rel err %.3e" % err)
    assert err <= TOL
    # callers that may not allocate: this plan's partial row blocks do not fit the static scratch array
    with pytest.raises(cst.ConststnError) as e:
        cst.execute_static(pl, [U3, U2], out.reshape(-1))
    assert e.value.status_name == "EUNSUPPORTED"


def test_config3_ttmc4_full_size():
    _say("config 3 full size: generate")
    wl = w.make(3, device="cuda")
    X = wl.sparse["X"]
    U1, U2, U3 = (wl.dense[k] for k in ("U1", "U2", "U3"))
    csf = cst.build_csf(X.coords, X.vals, X.dims, [0, 1, 2, 3])
    _say("config 3: CSF check")
    check_csf_full(csf, X.coords, X.vals, X.dims, [0, 1, 2, 3])
    pl = cst.plan(S.TTMC4, [("X", csf), ("U3", U3), ("U2", U2), ("U1", U1)])
    out = cst.execute(pl, [U3, U2, U1]).reshape(pl.n_rows, 16, 16, 16)
    torch.cuda.synchronize()
    # every slice of this tensor is cut into a dozen work items or more: the whole output is compared
    _say("config 3: oracle on all %d slices (%s)" % (pl.n_rows, pl.describe().split("|")[0]))
    cs, vs = X.numpy()
    Un = [u.cpu().numpy() for u in (U1, U2, U3)]
    want = oracle.ttmc4(cs, vs, X.dims, *Un)
    S_abs = oracle.ttmc4_abs(cs, vs, X.dims, *Un)
    err = oracle.rel_err(out.cpu().numpy(), want, S_abs)
    _say("  rel err %.3e over %d elements" % (err, want.size))
    assert err <= TOL
    del pl, out, want, S_abs
    # the order-4 MTTKRP on the same CSF: three statements fused on the whole prefix, one generic kernel with
    # scalar intermediates (leaf segments, every level's running sum); sampled slices against the N-ary sum
    from oracle import nary
    R = 32
    g = torch.Generator().manual_seed(77)
    B, C, D = (torch.rand(X.dims[m], R, generator=g, dtype=torch.float64) * 2 - 1 for m in (1, 2, 3))
    text = ("T1[i,j,k,r] = X[i,j,k,l] * D[l,r] | i,j,k,l,r ; T2[i,j,r] = T1[i,j,k,r] * C[k,r] | i,j,k,r ; "
            "M[i,r] = T2[i,j,r] * B[j,r] | i,j,r")
    dev = [t.cuda() for t in (D, C, B)]
    pl = cst.plan(text, [("X", csf), ("D", dev[0]), ("C", dev[1]), ("B", dev[2])])
    assert "kernels=1 inlined_producers=2" in pl.describe(), pl.describe()
    pl.check()
    out = cst.execute(pl, dev).reshape(pl.n_rows, R)
    torch.cuda.synchronize()
    picks = pick_slices(slice_sizes(csf), n_light=16, seed=3)
    roots = csf.export(0)[0][picks].long()
    sub_c, sub_v = subset(X.coords, X.vals, 0, roots.tolist())
    _say("config 3: order-4 MTTKRP in one kernel, %d sampled slices with %d nonzeros" % (len(picks), sub_v.size))
    f = [(B.numpy(), "jr"), (C.numpy(), "kr"), (D.numpy(), "lr")]
    ext = {"i": len(picks), "r": R}
    want = nary.contract(sub_c, sub_v, "ijkl", f, "ir", ext)
    S_abs = nary.contract_abs(sub_c, sub_v, "ijkl", f, "ir", ext)
    err = oracle.rel_err(out[roots.to(out.device)].cpu().numpy(), want, S_abs)
    _say("  rel err %.3e" % err)
    assert err <= TOL


def test_config4_three_tensor_network_full_size():
    _say("config 4 full size: generate")
    wl = w.make(4, device="cuda")
    U, W, V = wl.sparse["U"], wl.sparse["W"], wl.dense["V"]
    ucsf = cst.build_csf(U.coords, U.vals, U.dims, [0, 2, 1])
    wcsf = cst.build_csf(W.coords, W.vals, W.dims, [0, 1, 2])
    _say("config 4: CSF checks")
    check_csf_full(ucsf, U.coords, U.vals, U.dims, [0, 2, 1])
    check_csf_full(wcsf, W.coords, W.vals, W.dims, [0, 1, 2])
    pl = cst.plan(S.SPTN3, [("U", ucsf), ("V", V), ("W", wcsf)])
    out = cst.execute(pl, [V]).reshape(pl.n_rows, W.dims[2])
    torch.cuda.synchronize()
    _say("config 4: oracle on all %d output rows" % U.dims[0])
    cs, vs = U.numpy()
    wc, wv = W.numpy()
    args = (cs, vs, U.dims, V.cpu().numpy(), wc, wv, W.dims)
    want = oracle.sptn3(*args)
    S_abs = oracle.sptn3_abs(*args)
    err = oracle.rel_err(out.cpu().numpy(), want, S_abs)
    _say("  rel err %.3e over %d elements" % (err, want.size))
    assert err <= TOL


def test_config6_sparse_chain_full_size_sampled_slices():
    """The sparse chain of Sec. 5.1 at the size the benchmark times (32 x 32 lattice), both forms:
    structure and values of sampled slices K against the dense-slice reference."""
    from oracle import spsp
    from paper_2401_04836_amd import schedules as S
    _say("config 6 full size: generate")
    wl = w.make(6, device="cuda")
    dims = wl.params["dims"]
    I, C, P, L = (wl.sparse[k] for k in "ICPL")
    as_np = lambda t: ([c.cpu().numpy() for c in t.coords], t.vals.cpu().numpy())
    nI, nC, nP, nL = as_np(I), as_np(C), as_np(P), as_np(L)
    hI = cst.build_csf(I.coords, I.vals, I.dims, [0, 1, 2])
    hC = cst.build_csf(C.coords, C.vals, C.dims, [1, 0])
    hP = cst.build_csf(P.coords, P.vals, P.dims, [1, 0])
    hL = cst.build_csf(L.coords, L.vals, L.dims, [0, 1])
    Ks = [0, 517, 7001, 9999, dims[0] - 1]
    for form, text, ops, Lx in (("unrestricted", S.SPCHAIN3, [("I", hI), ("C", hC), ("P", hP)], None),
                                ("restricted", S.SPCHAIN3_RESTRICTED, [("I", hI), ("C", hC), ("L", hL), ("P", hP)], nL)):
        pl = cst.plan(text, ops)
        _say("config 6 %s: %s" % (form, pl.describe().split("|")[0]))
        assert "kernel=block-local" in pl.describe()
        vals = cst.execute(pl, [])
        torch.cuda.synchronize()
        E = pl.output_csf()
        i0, p0, _ = E.export(0)
        i1, p1, _ = E.export(1)
        i2, _, _ = E.export(2)
        ref = spsp.chain3(nI, nC, nP, dims, Lx, K_values=Ks)
        worst = 0.0
        for K in Ks:
            want, S_abs, N = ref[K]
            r = int(torch.searchsorted(i0, torch.tensor([K], device=i0.device, dtype=i0.dtype))[0])
            G = np.zeros_like(want)
            M = np.zeros(want.shape, dtype=bool)
            if r < i0.numel() and int(i0[r]) == K:
                na, nb = int(p0[r]), int(p0[r + 1])
                qa, qb = int(p1[na]), int(p1[nb])
                counts = (p1[na + 1:nb + 1] - p1[na:nb]).cpu().numpy()
                ii = np.repeat(i1[na:nb].cpu().numpy(), counts)
                mm = i2[qa:qb].cpu().numpy()
                G[ii, mm] = vals[qa:qb].cpu().numpy()
                M[ii, mm] = True
            np.testing.assert_array_equal(M, N, err_msg="structure of E[%d]" % K)
            worst = max(worst, oracle.rel_err(G, want, S_abs))
        _say("  %d result nonzeros, sampled K %s, rel err %.3e" % (pl.n_rows, Ks, worst))
        assert worst <= TOL
        del pl, vals


def test_config7_four_index_product_full_size_sampled_blocks():
    """The four-index product of Sec. 5.1 at the size the benchmark times (12 x 12 lattice, E with 4 M
    nonzeros, V with 224 M): E comes from the dense-slice reference of the chain, the GPU multiplies it
    with itself, and sampled (i,j) blocks are compared in structure and value with the reference."""
    from oracle import spsp
    from paper_2401_04836_amd import schedules as S
    _say("config 7 full size: generate")
    wl = w.make(7, device="cpu")
    n_K, n_i, n_u, n_m = wl.params["dims"]
    as_np = lambda t: ([c.numpy() for c in t.coords], t.vals.numpy())
    _say("config 7: reference E, %d slices" % n_K)
    ek, ei, em, ev = [], [], [], []
    for K0 in range(0, n_K, 96):                                   # a block of slices at a time keeps memory flat
        ref = spsp.chain3(as_np(wl.sparse["I"]), as_np(wl.sparse["C"]), as_np(wl.sparse["P"]), wl.params["dims"],
                          K_values=range(K0, min(K0 + 96, n_K)))
        for K, (E, _, N) in ref.items():
            ii, mm = np.nonzero(N)
            ek.append(np.full(ii.size, K, dtype=np.int64)); ei.append(ii); em.append(mm); ev.append(E[ii, mm])
    Ec = [np.concatenate(x) for x in (ek, ei, em)]
    Ev = np.concatenate(ev)
    dims = (n_K, n_i, n_m)
    _say("config 7: E has %d structural nonzeros" % Ev.size)
    hE = cst.build_csf([torch.as_tensor(c, dtype=torch.int32).cuda() for c in Ec], torch.as_tensor(Ev).cuda(), dims, [1, 0, 2])
    pl = cst.plan(S.SPPAIR4, [("Ea", hE), ("Eb", hE)])
    _say("config 7: %s" % pl.describe().split("|")[0])
    assert "kernel=dense rows" in pl.describe()
    vals = cst.execute(pl, [])
    torch.cuda.synchronize()
    V = pl.output_csf()
    (i0, p0, _), (i1, p1, _), (i2, p2, _), (i3, _, _) = (V.export(l) for l in range(4))
    assert pl.n_rows == i3.numel() == vals.numel()
    i0c, p0c, i1c, p1c = i0.cpu().numpy(), p0.cpu().numpy(), i1.cpu().numpy(), p1.cpu().numpy()
    p2c = p2.cpu().numpy()
    worst = 0.0
    samples = [(0, 0), (0, 1), (17, 29), (71, 72), (100, 3), (n_i - 1, n_i - 1), (60, 61), (5, 140)]
    for (i, j) in samples:
        want, S_abs, N = spsp.pair4_block(Ec, Ev, dims, i, j)
        G = np.zeros_like(want)
        M = np.zeros(want.shape, dtype=bool)
        r = int(np.searchsorted(i0c, i))
        if r < i0c.size and i0c[r] == i:
            a, b = int(p0c[r]), int(p0c[r + 1])
            x = a + int(np.searchsorted(i1c[a:b], j))
            if x < b and i1c[x] == j:                              # the pair is stored
                ra, rb = int(p1c[x]), int(p1c[x + 1])
                qa, qb = int(p2c[ra]), int(p2c[rb])
                mm = np.repeat(i2[ra:rb].cpu().numpy(), np.diff(p2c[ra:rb + 1]))
                nn = i3[qa:qb].cpu().numpy()
                G[mm, nn] = vals[qa:qb].cpu().numpy()
                M[mm, nn] = True
        np.testing.assert_array_equal(M, N, err_msg="structure of V[%d,%d]" % (i, j))
        worst = max(worst, oracle.rel_err(G, want, S_abs))
    _say("  %d result nonzeros, sampled pairs %s, rel err %.3e" % (pl.n_rows, samples, worst))
    assert worst <= TOL
