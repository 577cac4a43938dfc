#!/usr/bin/env python3
"""Benchmark of the fused sparse contraction path on one MI355X.

A step is one pass of the fused contraction over one synthetic batch with the CSF already
resident in HBM.  With no --config the five configurations run one after the other in one
process (5, 2, 3, 4, 1), followed by the two sparse-result networks of Sec. 5.1 (6: the three-index
transformation, 7: the four-index product) and, as record 8, the order-4 MTTKRP on configuration 3's
tensor; the headline (value, ms_per_step, roofline,
cpu_baseline) is that of configuration 5, the largest that fits one GPU (order-3 TTMc, 140 M
nonzeros, ranks 64 x 64, 47 GB of output), and "configs" holds the same record for every
configuration.  For
configuration 2 a step is the mode-0 MTTKRP (CSF i>j>k) followed by the mode-2 MTTKRP (CSF
k>j>i).  The CSF build (sort + pointer construction + partition) is timed separately and
reported under "csf_build".  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402

PLAN_OPTIONS = None          # tuning options handed to every plan (--generic, --plan-options)
HBM_PEAK_GBS = 8000.0
FP64_PEAK_TFLOPS = 78.6
CSRC = os.path.join(ROOT, "paper_2401_04836_amd", "csrc")
KERNEL_SOURCES = {"mttkrp3": ["kernels_mttkrp3.hip", "partition.hip"],
                  "ttmc3": ["kernels_ttmc3.hip", "partition.hip"],
                  "ttmc4": ["kernels_ttmc4.hip", "partition.hip"],
                  "sptn3": ["kernels_sptn3.hip", "partition.hip"],
                  "spchain3": ["kernels_spchain3.hip"], "sppair4": ["kernels_sppair4.hip"]}
KERNEL_NAMES = {"mttkrp3": "mttkrp3_r32_dual_kernel<4,4> (hot and cold sub-tensor as two teams of wavefronts in one launch)",
                "ttmc3": "ttmc3_stream_kernel<4,2,4>", "ttmc4": "ttmc4_mfma_kernel<1>", "sptn3": "sptn3_owned_kernel",
                "spchain3": "spchain3_local_kernel", "sppair4": "sppair4_kernel",
                "generic": "generic executor (generic_fused_kernel + generic_segsum kernels, or one kernel per statement)"}
# what bounds the dominant kernel of each family: the order-3 forms stream far more bytes than they
# compute (HBM); the order-4 TTMc and the three-tensor network are dense contractions per fiber
# (fp64 matrix cores)
BOUND = {"mttkrp3": "hbm", "ttmc3": "hbm", "ttmc4": "mfma", "sptn3": "mfma", "spchain3": "hbm", "sppair4": "mfma"}


def measured_traffic(family, config):
    """HBM bytes per launch from the rocprofv3 counter runs recorded under profiles/, or None when
    the counters were taken on another workload or the kernel sources have changed since."""
    import hashlib
    try:
        table = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
        entry = table[family]
        if entry.get("config") != config:
            return None
        h = hashlib.sha256()
        for f in KERNEL_SOURCES[family]:
            h.update(open(os.path.join(CSRC, f), "rb").read())
        if h.hexdigest()[:16] != entry["source_sha"]:
            return None
        return entry["traffic_bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


# seconds and algorithmic bytes of the CSF builds alone of the configuration being set up (the builders
# that time them fill it in; "csf_build" of the record then carries a roofline of its own)
CSF_ONLY = {}


def build_mttkrp(cst, S, wl, dev):
    X = wl.sparse["X"]
    coords = [c.to(dev) for c in X.coords]
    vals = X.vals.to(dev)
    A, B, C = (wl.dense[k].to(dev) for k in ("A", "B", "C"))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    csf0 = cst.build_csf(coords, vals, X.dims, [0, 1, 2])
    csf2 = cst.build_csf(coords, vals, X.dims, [2, 1, 0])
    torch.cuda.synchronize()
    CSF_ONLY["seconds"] = time.perf_counter() - t0
    # bytes a build has to move: the coordinate lists and values in, the level arrays out
    CSF_ONLY["bytes"] = sum((4 * X.order + 8) * X.nnz + 12 * sum(c.nodes(l) for l in range(X.order)) for c in (csf0, csf2))
    pl0 = cst.plan(S.MTTKRP3, [("X", csf0), ("C", C), ("B", B)], options=PLAN_OPTIONS)
    pl2 = cst.plan("T[k,j,r] = X[k,j,i] * A[i,r] | k,j,i,r ; M[k,r] = T[k,j,r] * B[j,r] | k,j,r",
                   [("X", csf2), ("A", A), ("B", B)], options=PLAN_OPTIONS)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    R = B.shape[1]
    launches = []
    for csf, pl, facs in ((csf0, pl0, [C, B]), (csf2, pl2, [A, B])):
        nodes = [csf.nodes(l) for l in range(3)]
        out = torch.empty(pl.n_rows * pl.row_elems, dtype=torch.float64, device=dev)
        # algorithmic HBM bytes of one launch: every CSF entry once (index 4 B + value or child
        # pointer 8 B), both factor matrices once, the output once
        alg_bytes = 12 * (nodes[2] + nodes[1] + nodes[0]) + 8 * R * (facs[0].shape[0] + facs[1].shape[0]) \
            + 8 * pl.n_rows * pl.row_elems
        flops = 2 * R * (nodes[2] + nodes[1])
        launches.append(dict(plan=pl, factors=facs, out=out, nodes=nodes, bytes=alg_bytes, flops=flops))
    return launches, build_s, 2 * X.nnz


def build_mttkrp_all_modes(cst, S, wl, dev):
    """One CP-ALS sweep's worth of MTTKRPs (Sec. 5.2 times all three): a CSF rooted at every mode."""
    X = wl.sparse["X"]
    coords = [c.to(dev) for c in X.coords]
    vals = X.vals.to(dev)
    F = [wl.dense[k].to(dev) for k in ("A", "B", "C")]
    R = F[0].shape[1]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    launches = []
    for levels in ([0, 1, 2], [1, 0, 2], [2, 1, 0]):
        csf = cst.build_csf(coords, vals, X.dims, levels)
        text, names = S.mttkrp3_for(levels)
        facs = [F[levels[2]], F[levels[1]]]
        pl = cst.plan(text, [("X", csf), (names[1], facs[0]), (names[2], facs[1])], options=PLAN_OPTIONS)
        nodes = [csf.nodes(l) for l in range(3)]
        out = torch.empty(pl.n_rows * pl.row_elems, dtype=torch.float64, device=dev)
        alg_bytes = 12 * sum(nodes) + 8 * R * (facs[0].shape[0] + facs[1].shape[0]) + 8 * pl.n_rows * pl.row_elems
        launches.append(dict(plan=pl, factors=facs, out=out, nodes=nodes, bytes=alg_bytes,
                             flops=2 * R * (nodes[2] + nodes[1]), keep=csf))
    torch.cuda.synchronize()
    return launches, time.perf_counter() - t0, 3 * X.nnz


def build_chain(cst, S, wl, dev, compact):
    X = wl.sparse["X"]
    coords = [c.to(dev) for c in X.coords]
    vals = X.vals.to(dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    csf = cst.build_csf(coords, vals, X.dims, list(range(X.order)))
    torch.cuda.synchronize()
    CSF_ONLY["seconds"] = time.perf_counter() - t0
    CSF_ONLY["bytes"] = (4 * X.order + 8) * X.nnz + 12 * sum(csf.nodes(l) for l in range(X.order))
    flags = cst.OUT_COMPACT if compact else 0
    if wl.kind == "ttmc3":
        U2, U3 = wl.dense["U2"].to(dev), wl.dense["U3"].to(dev)
        pl = cst.plan(S.TTMC3, [("X", csf), ("U3", U3), ("U2", U2)], flags=flags, options=PLAN_OPTIONS)
        facs = [U3, U2]
    else:
        U1, U2, U3 = (wl.dense[k].to(dev) for k in ("U1", "U2", "U3"))
        pl = cst.plan(S.TTMC4, [("X", csf), ("U3", U3), ("U2", U2), ("U1", U1)], flags=flags, options=PLAN_OPTIONS)
        facs = [U3, U2, U1]
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    nodes = [csf.nodes(l) for l in range(X.order)]
    out = torch.empty(pl.n_rows * pl.row_elems, dtype=torch.float64, device=dev)
    alg_bytes = 12 * sum(nodes) + 8 * sum(f.numel() for f in facs) + 8 * pl.n_rows * pl.row_elems
    ranks = [f.shape[1] for f in facs]             # innermost level first
    flops, width = 0, 1
    for lvl, r in zip(reversed(range(1, X.order)), ranks):
        width *= r
        flops += 2 * width * nodes[lvl]
    return [dict(plan=pl, factors=facs, out=out, nodes=nodes, bytes=alg_bytes, flops=flops)], build_s, X.nnz


def build_mttkrp4(cst, S, wl, dev):
    """Order-4 MTTKRP of rank 32 on an order-4 workload's tensor (the second operation of Sec. 5.3 at
    the next order up): three statements fused on the whole prefix, which the generic executor runs as
    one kernel with scalar intermediates."""
    X = wl.sparse["X"]
    csf = cst.build_csf([c.to(dev) for c in X.coords], X.vals.to(dev), X.dims, list(range(X.order)))
    R = 32
    g = torch.Generator().manual_seed(20240104)
    B, C, D = (torch.rand(X.dims[m], R, generator=g, dtype=torch.float64).to(dev) for m in (1, 2, 3))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    text = ("T1[i,j,k,r] = X[i,j,k,l] * D[l,r] | i,j,k,l,r ; T2[i,j,r] = T1[i,j,k,r] * C[k,r] | i,j,k,r ; "
            "M[i,r] = T2[i,j,r] * B[j,r] | i,j,r")
    pl = cst.plan(text, [("X", csf), ("D", D), ("C", C), ("B", B)], options=PLAN_OPTIONS)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    nodes = [csf.nodes(l) for l in range(X.order)]
    out = torch.empty(pl.n_rows * pl.row_elems, dtype=torch.float64, device=dev)
    alg_bytes = 12 * sum(nodes) + 8 * R * sum(X.dims)
    flops = 2 * R * sum(nodes[1:])
    return [dict(plan=pl, factors=[D, C, B], out=out, nodes=nodes, bytes=alg_bytes, flops=flops, keep=csf)], build_s, X.nnz


def build_sptn(cst, S, wl, dev):
    U, W = wl.sparse["U"], wl.sparse["W"]
    uc, uv = [c.to(dev) for c in U.coords], U.vals.to(dev)
    wc, wv = [c.to(dev) for c in W.coords], W.vals.to(dev)
    V = wl.dense["V"].to(dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ucsf = cst.build_csf(uc, uv, U.dims, [0, 2, 1])
    wcsf = cst.build_csf(wc, wv, W.dims, [0, 1, 2])
    pl = cst.plan(S.SPTN3, [("U", ucsf), ("V", V), ("W", wcsf)], options=PLAN_OPTIONS)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    out = torch.empty(pl.n_rows * pl.row_elems, dtype=torch.float64, device=dev)
    un = [ucsf.nodes(l) for l in range(3)]
    wn = [wcsf.nodes(l) for l in range(3)]
    alg_bytes = 12 * (sum(un) + sum(wn)) + 8 * V.numel() + 8 * out.numel()
    L = V.shape[1]
    # producer: 2L flop per U nonzero; consumer: per (i,k) fiber, 2 flop per W nonzero under k
    w_per_k = W.nnz / max(wn[0], 1)
    flops = 2 * L * un[2] + 2 * w_per_k * un[1]
    return [dict(plan=pl, factors=[V], out=out, nodes=un, bytes=alg_bytes, flops=flops)], build_s, U.nnz + W.nnz


def build_spchain(cst, S, wl, dev, restricted):
    I, C, P, L = (wl.sparse[k] for k in "ICPL")
    on = lambda t: ([c.to(dev) for c in t.coords], t.vals.to(dev))
    (ic, iv), (cc, cv), (pc, pv), (lc, lv) = on(I), on(C), on(P), on(L)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    hI = cst.build_csf(ic, iv, I.dims, [0, 1, 2])
    hC = cst.build_csf(cc, cv, C.dims, [1, 0])
    hP = cst.build_csf(pc, pv, P.dims, [1, 0])
    ops = [("I", hI), ("C", hC), ("P", hP)]
    if restricted:
        hL = cst.build_csf(lc, lv, L.dims, [0, 1])
        ops = [("I", hI), ("C", hC), ("L", hL), ("P", hP)]
    pl = cst.plan(S.SPCHAIN3_RESTRICTED if restricted else S.SPCHAIN3, ops, options=PLAN_OPTIONS)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    E = pl.output_csf()
    en = [E.nodes(l) for l in range(3)]
    nodes = [hI.nodes(l) for l in range(3)]
    out = torch.empty(pl.n_rows, dtype=torch.float64, device=dev)
    # algorithmic HBM bytes: I once (slot 2 B + value 8 B per leaf, index + pointer per upper node), C and P
    # once, the structure of E once (4 B per leaf, 12 B + operand references per upper node), its values once
    alg_bytes = 10 * nodes[2] + 12 * (nodes[1] + nodes[0]) + 12 * (C.nnz + P.nnz) + 4 * en[2] + 28 * en[1] + 8 * en[2]
    nnz_in = I.nnz + C.nnz + P.nnz + (L.nnz if restricted else 0)
    return [dict(plan=pl, factors=[], out=out, nodes=nodes, bytes=alg_bytes, flops=0, keep=ops)], build_s, nnz_in


def build_sppair(cst, S, wl, dev):
    """E by the three-index transformation (on the GPU, outside the timed step), then the plan of V = E x E."""
    I, C, P = (wl.sparse[k] for k in "ICP")
    on = lambda t: ([c.to(dev) for c in t.coords], t.vals.to(dev))
    (ic, iv), (cc, cv), (pc, pv) = on(I), on(C), on(P)
    hI = cst.build_csf(ic, iv, I.dims, [0, 1, 2])
    hC = cst.build_csf(cc, cv, C.dims, [1, 0])
    hP = cst.build_csf(pc, pv, P.dims, [1, 0])
    chain = cst.plan(S.SPCHAIN3, [("I", hI), ("C", hC), ("P", hP)])
    ev = cst.execute(chain, [])
    E = chain.output_csf()
    (i0, p0, _), (i1, p1, _), (i2, _, _) = E.export(0), E.export(1), E.export(2)
    node_K = torch.repeat_interleave(i0, p0[1:] - p0[:-1])
    eK = torch.repeat_interleave(node_K, p1[1:] - p1[:-1]).contiguous()
    ei = torch.repeat_interleave(i1, p1[1:] - p1[:-1]).contiguous()
    em = i2.clone()
    n_K, n_i, _, n_m = wl.params["dims"]
    wl.params["E"] = ([eK, ei, em], ev, (n_K, n_i, n_m))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    hE = cst.build_csf([eK, ei, em], ev, (n_K, n_i, n_m), [1, 0, 2])
    pl = cst.plan(S.SPPAIR4, [("Ea", hE), ("Eb", hE)], options=PLAN_OPTIONS)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    V = pl.output_csf()
    vn = [V.nodes(l) for l in range(4)]
    out = torch.empty(pl.n_rows, dtype=torch.float64, device=dev)
    nodes = [hE.nodes(l) for l in range(3)]
    # dense-block model of the contraction: per stored (i,j), shared K x (m of i) x (n of j) multiply-adds
    ki = torch.zeros(n_i, n_K, dtype=torch.float32, device=dev)
    ki[ei.long(), eK.long()] = 1.0
    shared = ki @ ki.T                                                # K stored under both i and j
    mi = torch.zeros(n_i, n_m, dtype=torch.float32, device=dev)
    mi[ei.long(), em.long()] = 1.0
    width = mi.sum(1)
    flops = float(2.0 * (shared * width[:, None] * width[None, :]).sum())
    alg_bytes = 2 * 12 * sum(nodes) + 12 * vn[3] + 12 * (vn[2] + vn[1] + vn[0])
    return [dict(plan=pl, factors=[], out=out, nodes=nodes, bytes=alg_bytes, flops=flops, keep=(hE, chain))], build_s, 2 * ev.numel()


def cpu_baseline_mttkrp4(wl, factors, budget_nnz):
    """The N-ary reference (numpy) on the first nonzeros of the order-4 tensor; factors = [D, C, B]."""
    from oracle import nary
    X = wl.sparse["X"]
    n = int(min(X.nnz, max(1000, budget_nnz // 400)))
    c = [x[:n].cpu().numpy() for x in X.coords]
    v = X.vals[:n].cpu().numpy()
    D, C, B = (f.cpu().numpy() for f in factors)
    t0 = time.perf_counter()
    nary.contract(c, v, "ijkl", [(B, "jr"), (C, "kr"), (D, "lr")], "ir", {"i": X.dims[0], "r": B.shape[1]})
    dt = time.perf_counter() - t0
    # numpy's einsum (no BLAS in this product) and add.at run on the calling thread
    return dict(value=n / dt, unit="nnz/s", cores=1, kind="oracle",
                sample="N-ary sum over the first %d nonzeros (input order), %.2f s" % (n, dt))


def cpu_baseline(wl, budget_nnz):
    """The CPU oracle, as it stands, on a bounded sample (first nonzeros) of the same workload."""
    import oracle
    if wl.kind == "mttkrp3":
        X = wl.sparse["X"]
        n = min(X.nnz, budget_nnz)
        c = [x[:n].cpu().numpy() for x in X.coords]
        v = X.vals[:n].cpu().numpy()
        B, C = wl.dense["B"].cpu().numpy(), wl.dense["C"].cpu().numpy()
        A = wl.dense["A"].cpu().numpy()
        oracle.lib()
        t0 = time.perf_counter()
        oracle.mttkrp3(c, v, X.dims, B, C, 0)
        oracle.mttkrp3(c, v, X.dims, A, B, 2)
        dt = time.perf_counter() - t0
        return dict(value=2 * n / dt, unit="nnz/s", cores=oracle.num_threads(), kind="oracle",
                    sample="mode-0 and mode-2 MTTKRP of the first %d nonzeros (input order), %.2f s"
                           % (n, dt))
    if wl.kind == "ttmc3":
        X = wl.sparse["X"]
        R2, R3 = wl.params["ranks"]
        n = min(X.nnz, max(1000, budget_nnz * 32 // (R2 * R3)))
        c = [x[:n].cpu().numpy() for x in X.coords]
        v = X.vals[:n].cpu().numpy()
        # restrict to the rows touched so the dense output of the sample stays small
        import numpy as np
        rows, inv = np.unique(c[0], return_inverse=True)
        c[0] = inv.astype(np.int32)
        t0 = time.perf_counter()
        oracle.ttmc3(c, v, (len(rows), X.dims[1], X.dims[2]), wl.dense["U2"].cpu().numpy(),
                     wl.dense["U3"].cpu().numpy(), 0)
        dt = time.perf_counter() - t0
        return dict(value=n / dt, unit="nnz/s", cores=oracle.num_threads(), kind="oracle",
                    sample="TTMc of the first %d nonzeros (rows renumbered), %.2f s" % (n, dt))
    if wl.kind == "ttmc4":
        X = wl.sparse["X"]
        n = min(X.nnz, max(1000, budget_nnz // 128))
        c = [x[:n].cpu().numpy() for x in X.coords]
        v = X.vals[:n].cpu().numpy()
        t0 = time.perf_counter()
        oracle.ttmc4(c, v, X.dims, *(wl.dense[k].cpu().numpy() for k in ("U1", "U2", "U3")))
        dt = time.perf_counter() - t0
        return dict(value=n / dt, unit="nnz/s", cores=oracle.num_threads(), kind="oracle",
                    sample="order-4 TTMc of the first %d nonzeros, %.2f s" % (n, dt))
    if wl.kind == "sptn3":
        import numpy as np
        U, W = wl.sparse["U"], wl.sparse["W"]
        ui = U.coords[0].cpu().numpy()
        # slices are taken whole (the consumer works per slice): as many leading i as hold the budget
        order = np.argsort(ui, kind="stable")
        n = int(min(U.nnz, max(1000, budget_nnz // 5)))
        n_rows = int(ui[order[n - 1]]) + 1
        sel = order[:int(np.searchsorted(ui[order], n_rows))]
        c = [x.cpu().numpy()[sel] for x in U.coords]
        v = U.vals.cpu().numpy()[sel]
        wc = [x.cpu().numpy() for x in W.coords]
        oracle.lib()
        t0 = time.perf_counter()
        oracle.sptn3(c, v, (n_rows, U.dims[1], U.dims[2]), wl.dense["V"].cpu().numpy(), wc, W.vals.cpu().numpy(), W.dims)
        dt = time.perf_counter() - t0
        share = len(v) / U.nnz
        return dict(value=(len(v) + share * W.nnz) / dt, unit="nnz/s", cores=oracle.num_threads(), kind="oracle",
                    sample="the first %d slices i of U (%d nonzeros) against all of V and W, counted with the same "
                           "share of W's nonzeros, %.2f s" % (n_rows, len(v), dt))
    if wl.kind == "sppair4":
        from oracle import spsp
        (ek, ei, em), ev, dims = wl.params["E"]
        Ec = [x.cpu().numpy() for x in (ek, ei, em)]
        Ev = ev.cpu().numpy()
        n_i = dims[1]
        pairs = [(int(a), int(b)) for a, b in zip(torch.linspace(0, n_i - 1, 24), torch.linspace(n_i - 1, 0, 24))]
        pairs += [(a, a) for a, _ in pairs]
        t0 = time.perf_counter()
        for a, b in pairs:
            spsp.pair4_block(Ec, Ev, dims, a, b)
        dt = time.perf_counter() - t0
        per_pair = 2 * len(Ev) / (n_i * n_i)                    # input nonzeros an (i,j) block accounts for
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
        except ImportError:
            cores = 1
        return dict(value=per_pair * len(pairs) / dt, unit="nnz/s", cores=cores, kind="oracle",
                    sample="%d of the %d (i,j) blocks, dense slab products, %.2f s; nonzeros counted as 2 nnz(E) spread "
                           "evenly over the blocks" % (len(pairs), n_i * n_i, dt))
    if wl.kind == "spchain3":
        from oracle import spsp
        I, C, P, L = (wl.sparse[k] for k in "ICPL")
        as_np = lambda t: ([c.cpu().numpy() for c in t.coords], t.vals.cpu().numpy())
        n_K = wl.params["dims"][0]
        ks = sorted(set(int(k) for k in torch.linspace(0, n_K - 1, 128 if n_K > 1000 else n_K)))
        Inp = as_np(I)
        in_sample = int(sum((Inp[0][0] == k).sum() for k in ks))
        t0 = time.perf_counter()
        spsp.chain3(Inp, as_np(C), as_np(P), wl.params["dims"], as_np(L) if wl.params.get("restricted") else None,
                    K_values=ks)
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
        except ImportError:
            cores = 1
        return dict(value=in_sample / dt, unit="nnz/s", cores=cores, kind="oracle",
                    sample="%d of the %d slices K (evenly spaced), %d nonzeros of I, dense slice products, %.2f s"
                           % (len(ks), n_K, in_sample, dt))
    return None


def one_thread():
    """Context manager: the oracle's OpenMP team cut to one thread (the paper's regime, Sec. 5)."""
    import contextlib
    import ctypes

    @contextlib.contextmanager
    def cm():
        import oracle
        oracle.lib()
        omp = ctypes.CDLL("libgomp.so.1")
        before = oracle.num_threads()
        omp.omp_set_num_threads(1)
        try:
            yield
        finally:
            omp.omp_set_num_threads(before)
    return cm()


def measured_peaks(cst):
    """What this GPU delivers on a plain copy, a plain fill and a loop of fp64 matrix instructions."""
    try:
        return {"copy_GBps": cst.measure_peak(cst.PEAK_COPY, 1 << 31, 5),
                "write_GBps": cst.measure_peak(cst.PEAK_WRITE, 1 << 32, 5),
                "mfma_f64_TFLOPs": cst.measure_peak(cst.PEAK_MFMA_F64, 4096, 3),
                "clock_MHz_under_mfma_f64": cst.measure_peak(cst.PEAK_MFMA_CLOCK, 4096, 2),
                "clock_MHz_light_load": cst.measure_peak(cst.PEAK_VALU_CLOCK, 200000, 2),
                "what": "2 GiB device copy (bytes read + written), 4 GiB fill, 8 independent v_mfma_f64_16x16x4 chains "
                        "with four wavefronts per SIMD; nominal 8000 GB/s and 78.6 TFLOP/s"}
    except cst.ConststnError as e:
        return {"error": str(e)}


def run_config(cst, S, dev, args, cid, cpu_budget):
    """Generate configuration `cid`, build its CSFs and plans, time args.steps steps; returns the record."""
    t0 = time.perf_counter()
    wl = workloads.make(cid, device=dev, small=args.small)
    torch.cuda.synchronize()
    CSF_ONLY.clear()
    log("generated config %d (%s) in %.1f s: %s" % (
        cid, wl.kind, time.perf_counter() - t0, {k: (v.dims, v.nnz) for k, v in wl.sparse.items()}))

    if wl.kind == "mttkrp3" and args.all_modes:
        launches, build_s, nnz_per_step = build_mttkrp_all_modes(cst, S, wl, dev)
        name = "C2 MTTKRP order-3 %s nnz=%d rank=%d, modes 0, 1 and 2" % (
            "x".join(map(str, wl.sparse["X"].dims)), wl.sparse["X"].nnz, wl.params["rank"])
    elif wl.kind == "mttkrp3":
        launches, build_s, nnz_per_step = build_mttkrp(cst, S, wl, dev)
        name = "C2 MTTKRP order-3 %s nnz=%d rank=%d, modes 0 and 2" % (
            "x".join(map(str, wl.sparse["X"].dims)), wl.sparse["X"].nnz, wl.params["rank"])
    elif wl.kind == "ttmc4" and args.mttkrp4:
        launches, build_s, nnz_per_step = build_mttkrp4(cst, S, wl, dev)
        name = "MTTKRP order-4 %s nnz=%d rank=32 on the tensor of C%d" % (
            "x".join(map(str, wl.sparse["X"].dims)), wl.sparse["X"].nnz, cid)
    elif wl.kind in ("ttmc3", "ttmc4"):
        launches, build_s, nnz_per_step = build_chain(cst, S, wl, dev, wl.params.get("compact", False))
        name = "C%d TTMc order-%d %s nnz=%d ranks=%s%s" % (
            cid, wl.sparse["X"].order, "x".join(map(str, wl.sparse["X"].dims)),
            wl.sparse["X"].nnz, wl.params["ranks"], ", rows of nonempty slices only" if wl.params.get("compact") else "")
    elif wl.kind == "sppair4":
        launches, build_s, nnz_per_step = build_sppair(cst, S, wl, dev)
        name = "C7 V=E.E lattice %dx%d nnzE=%d nnzV=%d" % (wl.params["side"], wl.params["side"], nnz_per_step // 2,
                                                          launches[0]["plan"].n_rows)
    elif wl.kind == "spchain3":
        wl.params["restricted"] = args.restricted
        launches, build_s, nnz_per_step = build_spchain(cst, S, wl, dev, args.restricted)
        name = "C6 E=I.C.P%s lattice %dx%d dims(K,i,u,m)=%s nnzI=%d nnzE=%d" % (
            ".L (restricted)" if args.restricted else "", wl.params["side"], wl.params["side"], wl.params["dims"],
            wl.sparse["I"].nnz, launches[0]["plan"].n_rows)
    else:
        launches, build_s, nnz_per_step = build_sptn(cst, S, wl, dev)
        name = "C4 Z=(U.V).W dims(i,j,k,l,m)=%s nnzU=%d nnzW=%d" % (
            wl.params["dims"], wl.sparse["U"].nnz, wl.sparse["W"].nnz)
    if args.small:
        name += " (reduced copy)"
    for L in launches:
        log("plan: %s" % L["plan"].describe().split("|")[0])
        log("  CSF nodes per level %s, algorithmic bytes %.3f GB, flops %.3f G" % (
            L["nodes"], L["bytes"] / 1e9, L["flops"] / 1e9))
    log("CSF build + plan: %.3f s" % build_s)

    def step():
        for L in launches:
            cst.execute(L["plan"], L["factors"], out=L["out"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    for L in launches:
        L["plan"].profile(max(args.steps, 1))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_ms, per_launch_ms = [], []
    for L in launches:
        kt = L["plan"].kernel_times()
        kernel_ms += kt
        per_launch_ms.append(sum(kt) / max(len(kt), 1))
        L["plan"].profile(0)
    ms_per_step = dt / args.steps * 1e3
    avg_kernel_ms = sum(kernel_ms) / max(len(kernel_ms), 1)
    alg_bytes = sum(L["bytes"] for L in launches) / len(launches)          # per launch
    flops_step = sum(L["flops"] for L in launches)
    achieved = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    step_gbs = sum(L["bytes"] for L in launches) / (dt / args.steps) / 1e9

    desc = launches[0]["plan"].describe().split("|")[0]
    family = desc.split()[0].split("=")[1]
    if family == "generic":
        name += " [generic executor]"
    plain = not (args.small or args.restricted or args.all_modes or args.mttkrp4)
    rec = {
        "config_id": cid, "workload": name, "kind": "mttkrp4" if (args.mttkrp4 and wl.kind == "ttmc4") else wl.kind,
        "ms_per_step": ms_per_step, "nnz_per_step": nnz_per_step, "nnz_per_s": nnz_per_step / (dt / args.steps),
        "gflops": flops_step / (dt / args.steps) / 1e9,
        "fp64_frac": flops_step / (dt / args.steps) / 1e12 / FP64_PEAK_TFLOPS,
        "csf_build": dict({"seconds": build_s, "nnz_per_s": nnz_per_step / build_s,
                           "what": "CSF build(s) + plan, once per tensor, outside the timed step"},
                          **({"csf_only_seconds": CSF_ONLY["seconds"], "csf_only_algorithmic_bytes": CSF_ONLY["bytes"],
                              "csf_only_GBps": CSF_ONLY["bytes"] / CSF_ONLY["seconds"] / 1e9,
                              "csf_only_hbm_frac": CSF_ONLY["bytes"] / CSF_ONLY["seconds"] / 1e9 / HBM_PEAK_GBS}
                             if CSF_ONLY else {})),
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(family, cid if plain else None),
                     "kernel": KERNEL_NAMES.get(family, family),
                     "kernel_ms_avg": avg_kernel_ms, "launches_timed": len(kernel_ms),
                     "kernel_ms_per_contraction": per_launch_ms,
                     "algorithmic_bytes_per_launch": alg_bytes,
                     # the same bytes over the whole step (zero-fill and fix-up passes included)
                     "frac_whole_step": step_gbs / HBM_PEAK_GBS},
    }
    if BOUND.get(family) == "mfma":
        flops_launch = flops_step / len(launches)
        tf = flops_launch / (avg_kernel_ms * 1e-3) / 1e12
        rec["roofline"].update({"bound": "mfma", "achieved": tf, "peak": FP64_PEAK_TFLOPS,
                                "unit": "TFLOP/s", "frac": tf / FP64_PEAK_TFLOPS,
                                "algorithmic_flops_per_launch": flops_launch,
                                "frac_whole_step": flops_step / (dt / args.steps) / 1e12 / FP64_PEAK_TFLOPS})
    # matrix instructions the plan's dominant kernel issues per launch ("mfma=<count>" in the plan text):
    # utilisation of the matrix cores by the per-slice stage alone, padding included
    for tok in desc.split():
        if tok.startswith("mfma="):
            n_mfma = int(tok[5:])
            tf = n_mfma * 2048.0 / (avg_kernel_ms * 1e-3) / 1e12
            rec["roofline"]["mfma_stage"] = {"instructions": n_mfma, "flop_per_instruction": 2048,
                                             "achieved": tf, "peak": FP64_PEAK_TFLOPS, "unit": "TFLOP/s",
                                             "frac": tf / FP64_PEAK_TFLOPS}
    if wl.kind in ("ttmc3", "mttkrp3", "ttmc4") and family != "generic" and cid == 1:
        rec["roofline"]["note"] = "0.3 MB problem: launch latency, no roofline claim"
    if not args.no_cpu and args.mttkrp4 and wl.kind == "ttmc4":
        rec["cpu_baseline"] = cpu_baseline_mttkrp4(wl, launches[0]["factors"], cpu_budget)
    if not args.no_cpu and not args.mttkrp4:
        cb = cpu_baseline(wl, cpu_budget)
        if cb is not None:
            rec["cpu_baseline"] = cb
        if cid in (1, 2, 3) and cb is not None:
            with one_thread():
                c1 = cpu_baseline(wl, max(cpu_budget // 8, 1_000_000))
            rec["cpu_baseline_1thread"] = c1
    log("C%d: %.3f ms/step, %.3g nnz/s, roofline %.3f (%s)" % (cid, ms_per_step, rec["nnz_per_s"],
                                                                rec["roofline"]["frac"], rec["roofline"]["bound"]))
    # free the device memory of this configuration before the next one is generated
    for L in launches:
        L["plan"].destroy()
    del launches, wl
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=0,
                    help="0 (default): configurations 5, 2, 3, 4, 1 in one run, the headline on 5, the largest; "
                         "1..5: that configuration alone; 6 = the sparse chain of Sec. 5.1 on lattice maps, "
                         "7 = the four-index product of the same section")
    ap.add_argument("--all-modes", action="store_true",
                    help="configuration 2: a step is the MTTKRP of every mode (0, 1, 2), each on a CSF rooted at its mode")
    ap.add_argument("--mttkrp4", action="store_true",
                    help="configuration 3: instead of the TTMc, the order-4 MTTKRP of rank 32 on the same tensor, "
                         "a chain of three fused statements the generic executor runs as one kernel")
    ap.add_argument("--restricted", action="store_true", help="configuration 6: the form with the K -> i filter")
    ap.add_argument("--small", action="store_true", help="reduced copy of the configuration")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-peaks", action="store_true", help="skip the measured copy / matrix-core ceilings")
    ap.add_argument("--peaks-only", action="store_true",
                    help="measure the copy, fill and fp64 matrix-core ceilings of this GPU, print them and stop")
    ap.add_argument("--generic", action="store_true",
                    help="plan with the generic executor instead of the tuned kernels (configs 1, 2, 3, 5)")
    ap.add_argument("--plan-options", default=None, help="tuning options for every plan, \"name=value,...\"")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one plain 1 GiB device copy (reference for the FETCH_SIZE / "
                         "WRITE_SIZE counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures ONE GPU: the path has no multi-GPU part (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    global PLAN_OPTIONS
    PLAN_OPTIONS = args.plan_options
    if args.generic:
        PLAN_OPTIONS = "force_generic=1" + ("," + PLAN_OPTIONS if PLAN_OPTIONS else "")
    import paper_2401_04836_amd as cst
    from paper_2401_04836_amd import schedules as S
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.peaks_only:
        print(json.dumps({"measured_peak": measured_peaks(cst)}), flush=True)
        return
    if args.calibrate:
        src = torch.ones(1 << 27, dtype=torch.float64, device=dev)        # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                                                     # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        log("calibration copy: 1 GiB read + 1 GiB written by one copy kernel")
        del src, dst

    cids = [5, 2, 3, 4, 1, 6, 7] if args.config == 0 else [args.config]
    # CPU-oracle sample, in multiply-adds' worth of nonzeros per configuration: a few seconds to about ten per
    # configuration in the five-configuration run
    cpu_budget = 400_000_000 if len(cids) == 1 else 1_200_000_000
    recs = [run_config(cst, S, dev, args, cid, cpu_budget) for cid in cids]
    if args.config == 0 and not args.mttkrp4:
        # beside the configurations: the order-4 MTTKRP on configuration 3's tensor (a fused chain in one generic kernel)
        args.mttkrp4 = True
        extra = run_config(cst, S, dev, args, 3, cpu_budget)
        extra["config_id"] = 8
        recs.append(extra)
        args.mttkrp4 = False
    head = recs[0]
    result = {
        "metric": "fused sparse contraction nnz/s", "value": head["nnz_per_s"],
        "unit": "nnz/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": head["workload"], "step": "one fused contraction pass per CSF (build excluded)"},
        "gflops": head["gflops"], "fp64_frac": head["fp64_frac"], "csf_build": head["csf_build"],
        "roofline": head["roofline"],
    }
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
    if "cpu_baseline_1thread" in head:
        result["cpu_baseline_1thread"] = head["cpu_baseline_1thread"]
    if not args.no_peaks:
        result["measured_peak"] = measured_peaks(cst)
    if len(recs) > 1:
        result["configs"] = recs
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
