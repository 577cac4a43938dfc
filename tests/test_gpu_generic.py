"""Generic executor (any contraction tree over one CSF tensor, Sec. 2.2 / 4.2) on the GPU against
the N-ary reference: orders and ranks beyond the tuned kernels, other trees over the same
network, every fusion choice, a fully contracted result, and what it must refuse."""

import numpy as np
import pytest
import torch

from oracle import nary
import paper_2401_04836_amd as cst
from helpers import TOL
import oracle

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _tensor(seed, dims, nnz):
    g = torch.Generator().manual_seed(seed)
    total = int(np.prod(dims))
    cells = torch.randperm(total, generator=g)[:nnz]
    coords = []
    for d in reversed(dims):
        coords.append((cells % d).to(torch.int32))
        cells = cells // d
    coords.reverse()
    vals = torch.randn(nnz, generator=g, dtype=torch.float64)
    return coords, vals


def _dense(seed, *shape):
    g = torch.Generator().manual_seed(seed)
    return torch.rand(*shape, generator=g, dtype=torch.float64) * 2 - 1


def _run(text, x, mode_order, dense, out_shape, fusion=None, flags=0, expect="generic", options=None):
    """x = (coords, vals, dims); dense = [(name, tensor)] in operand order.  Returns a CPU array."""
    coords, vals, dims = x
    csf = cst.build_csf([c.cuda() for c in coords], vals.cuda(), dims, mode_order)
    dev = [(n, t.cuda()) for n, t in dense]
    pl = cst.plan(text, [("X", csf)] + dev, fusion=fusion, flags=flags, options=options)
    desc = pl.describe()
    _say("  " + desc.split("|")[0])
    assert ("family=" + expect) in desc, desc
    if expect == "generic":
        pl.check()                                # segment tables, heavy-node lists, first-leaf tables
    out = cst.execute(pl, [t for _, t in dev])
    torch.cuda.synchronize()
    assert pl.n_rows * pl.row_elems == int(np.prod(out_shape)), (pl.n_rows, pl.row_elems, out_shape)
    return out.cpu().numpy().reshape(out_shape), pl


def _check(got, coords, vals, x_idx, factors, out_idx, extents):
    c = [t.numpy() for t in coords]
    f = [(t.numpy(), l) for t, l in factors]
    want = nary.contract(c, vals.numpy(), x_idx, f, out_idx, extents)
    S = nary.contract_abs(c, vals.numpy(), x_idx, f, out_idx, extents)
    err = oracle.rel_err(got, want, S)
    _say("  rel err %.3e" % err)
    assert err <= TOL


def test_ttmc_order5():
    dims = (23, 9, 11, 7, 13)
    coords, vals = _tensor(301, dims, 5000)
    U = [_dense(302 + m, dims[m], r) for m, r in zip(range(1, 5), (3, 4, 2, 5))]
    text = ("T1[i,j,k,l,d] = X[i,j,k,l,m] * U4[m,d] | i,j,k,l,m,d ; "
            "T2[i,j,k,c,d] = T1[i,j,k,l,d] * U3[l,c] | i,j,k,l,c,d ; "
            "T3[i,j,b,c,d] = T2[i,j,k,c,d] * U2[k,b] | i,j,k,b,c,d ; "
            "Y[i,a,b,c,d] = T3[i,j,b,c,d] * U1[j,a] | i,j,a,b,c,d")
    _say("order-5 TTMc")
    got, _ = _run(text, (coords, vals, dims), [0, 1, 2, 3, 4],
                  [("U4", U[3]), ("U3", U[2]), ("U2", U[1]), ("U1", U[0])], (23, 3, 4, 2, 5))
    _check(got, coords, vals, "ijklm", [(U[0], "ja"), (U[1], "kb"), (U[2], "lc"), (U[3], "md")], "iabcd",
           {"i": 23, "a": 3, "b": 4, "c": 2, "d": 5})


def test_mttkrp_order4_and_fusion_choices():
    dims = (40, 17, 19, 15)
    coords, vals = _tensor(311, dims, 9000)
    B, C, D = _dense(312, 17, 24), _dense(313, 19, 24), _dense(314, 15, 24)
    text = ("T1[i,j,k,r] = X[i,j,k,l] * D[l,r] | i,j,k,l,r ; "
            "T2[i,j,r] = T1[i,j,k,r] * C[k,r] | i,j,k,r ; "
            "M[i,r] = T2[i,j,r] * B[j,r] | i,j,r")
    f = [(B, "jr"), (C, "kr"), (D, "lr")]
    for fusion in (None, [0, 0, 0], [1, 2, 0], [3, 1, 0]):
        _say("order-4 MTTKRP, fusion %s" % (fusion,))
        got, _ = _run(text, (coords, vals, dims), [0, 1, 2, 3], [("D", D), ("C", C), ("B", B)], (40, 24),
                      fusion=fusion)
        _check(got, coords, vals, "ijkl", f, "ir", {"i": 40, "r": 24})


def test_ranks_beyond_the_tuned_kernels_go_generic():
    dims = (50, 30, 20)
    coords, vals = _tensor(321, dims, 4000)
    U2, U3 = _dense(322, 30, 72), _dense(323, 20, 80)
    _say("TTMc order 3, ranks 72 x 80")
    got, _ = _run("T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s ; Y[i,r,s] = T[i,j,s] * U2[j,r] | i,j,r,s",
                  (coords, vals, dims), [0, 1, 2], [("U3", U3), ("U2", U2)], (50, 72, 80))
    _check(got, coords, vals, "ijk", [(U2, "jr"), (U3, "ks")], "irs", {"i": 50, "r": 72, "s": 80})
    B, C = _dense(324, 30, 200), _dense(325, 20, 200)
    _say("MTTKRP order 3, rank 200")
    got, _ = _run("T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; M[i,r] = T[i,j,r] * B[j,r] | i,j,r",
                  (coords, vals, dims), [0, 1, 2], [("C", C), ("B", B)], (50, 200))
    _check(got, coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 50, "r": 200})


def test_other_tree_dense_subtree_first_and_two_levels_summed_at_once():
    # MTTKRP as (B (.) C) first, a dense-only statement, then one contraction over j and k together
    dims = (31, 12, 14)
    coords, vals = _tensor(331, dims, 2500)
    B, C = _dense(332, 12, 10), _dense(333, 14, 10)
    text = ("P[j,k,r] = B[j,r] * C[k,r] | j,k,r ; "
            "M[i,r] = X[i,j,k] * P[j,k,r] | i,j,k,r")
    _say("MTTKRP via the dense Khatri-Rao product first")
    got, _ = _run(text, (coords, vals, dims), [0, 1, 2], [("B", B), ("C", C)], (31, 10))
    _check(got, coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 31, "r": 10})


def test_fully_contracted_result_and_output_index_order():
    dims = (26, 15, 18)
    coords, vals = _tensor(341, dims, 3000)
    A, B, C = _dense(342, 26, 6), _dense(343, 15, 6), _dense(344, 18, 6)
    text = ("T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; "
            "M[i,r] = T[i,j,r] * B[j,r] | i,j,r ; "
            "z[r] = M[i,r] * A[i,r] | i,r")
    _say("inner product of X with a rank-6 Kruskal tensor, per rank component")
    got, pl = _run(text, (coords, vals, dims), [0, 1, 2], [("C", C), ("B", B), ("A", A)], (6,))
    assert pl.n_rows == 1
    _check(got, coords, vals, "ijk", [(A, "ir"), (B, "jr"), (C, "kr")], "r", {"r": 6})
    U2, U3 = _dense(345, 15, 4), _dense(346, 18, 5)
    _say("TTMc with the result's rank indices swapped")
    got, _ = _run("T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s ; Y[i,s,r] = T[i,j,s] * U2[j,r] | i,j,s,r",
                  (coords, vals, dims), [0, 1, 2], [("U3", U3), ("U2", U2)], (26, 5, 4))
    _check(got, coords, vals, "ijk", [(U2, "jr"), (U3, "ks")], "isr", {"i": 26, "s": 5, "r": 4})


def test_generic_matches_tuned_kernels_and_compact_rows():
    dims = (64, 40, 30)
    coords, vals = _tensor(351, dims, 3000)            # some root indices stay empty
    coords[0] = (coords[0] // 2) * 2                   # only even i, duplicates removed below
    key = (coords[0].long() * 40 + coords[1]) * 30 + coords[2]
    _, first = np.unique(key.numpy(), return_index=True)
    coords = [c[first] for c in coords]
    vals = vals[first]
    B, C = _dense(352, 40, 32), _dense(353, 30, 32)
    text = "T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; M[i,r] = T[i,j,r] * B[j,r] | i,j,r"
    tuned, _ = _run(text, (coords, vals, dims), [0, 1, 2], [("C", C), ("B", B)], (64, 32), expect="mttkrp3")
    gen, _ = _run(text, (coords, vals, dims), [0, 1, 2], [("C", C), ("B", B)], (64, 32), options="force_generic=1")
    nrows = int(np.unique(coords[0].numpy()).size)
    comp, pl = _run(text, (coords, vals, dims), [0, 1, 2], [("C", C), ("B", B)], (nrows, 32),
                    flags=cst.OUT_COMPACT, options="force_generic=1")
    _check(gen, coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 64, "r": 32})
    _check(tuned, coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 64, "r": 32})
    assert not gen[1::2].any()                          # odd rows: no nonzeros, exact zeros
    rows = pl.output_rows().cpu().numpy()
    np.testing.assert_array_equal(comp, gen[rows])


def test_fused_leaf_producer_is_inlined_and_equals_the_stored_intermediate():
    # Sec. 2.2: a producer fused with its consumer on the whole sparse prefix needs a scalar only.  The
    # executor then sums the leaves inside the consumer's kernel; fusion depth 0 and generic_fuse=0 store T.
    dims = (70, 45, 38)
    coords, vals = _tensor(391, dims, 9000)
    heavy = torch.randperm(45 * 38, generator=torch.Generator().manual_seed(392))[:1500]     # one long slice
    coords = [torch.cat([c, h]) for c, h in zip(coords, (torch.full((1500,), 5, dtype=torch.int32),
                                                        (heavy // 38).to(torch.int32), (heavy % 38).to(torch.int32)))]
    vals = torch.cat([vals, _dense(393, 1500)])
    key = (coords[0].long() * 45 + coords[1]) * 38 + coords[2]
    _, first = np.unique(key.numpy(), return_index=True)
    coords, vals = [c[first] for c in coords], vals[first]
    x = (coords, vals, dims)
    B, C = _dense(394, 45, 24), _dense(395, 38, 24)
    text = "T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; M[i,r] = T[i,j,r] * B[j,r] | i,j,r"
    f = [("C", C), ("B", B)]
    fused, pl = _run(text, x, [0, 1, 2], f, (70, 24), options="force_generic=1")
    assert "inlined_producers=1" in pl.describe(), pl.describe()
    _check(fused, coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 70, "r": 24})
    for opts, fusion in (("force_generic=1,generic_fuse=0", None), ("force_generic=1", [0, 0])):
        stored, pl = _run(text, x, [0, 1, 2], f, (70, 24), fusion=fusion, options=opts)
        assert "inlined_producers=0" in pl.describe(), pl.describe()
        np.testing.assert_allclose(stored, fused, rtol=0, atol=1e-11)
    _say("long slices cut into segments (span 16), then compact rows")
    seg, pl = _run(text, x, [0, 1, 2], f, (70, 24), options="force_generic=1,generic_span=16")
    assert "inlined_producers=1" in pl.describe()
    _check(seg, coords, vals, "ijk", [(B, "jr"), (C, "kr")], "ir", {"i": 70, "r": 24})
    _say("order 4: the whole chain is inlined; a TTMc (the producer's result has fewer dense indices) is not")
    dims4 = (30, 14, 12, 11)
    c4, v4 = _tensor(396, dims4, 6000)
    B4, C4, D4 = _dense(397, 14, 8), _dense(398, 12, 8), _dense(399, 11, 8)
    t4 = ("T1[i,j,k,r] = X[i,j,k,l] * D[l,r] | i,j,k,l,r ; T2[i,j,r] = T1[i,j,k,r] * C[k,r] | i,j,k,r ; "
          "M[i,r] = T2[i,j,r] * B[j,r] | i,j,r")
    got, pl = _run(t4, (c4, v4, dims4), [0, 1, 2, 3], [("D", D4), ("C", C4), ("B", B4)], (30, 8))
    assert "kernels=1 inlined_producers=2" in pl.describe(), pl.describe()
    _check(got, c4, v4, "ijkl", [(B4, "jr"), (C4, "kr"), (D4, "lr")], "ir", {"i": 30, "r": 8})
    _say("a slice of 40 000 leaves in 20 000 fibers: more segments than one thread adds in the second pass")
    dimsh = (10, 20000, 4)
    ch, vh = _tensor(405, dimsh, 3000)
    cells = torch.randperm(20000 * 4, generator=torch.Generator().manual_seed(406))[:40000]
    keep = ch[0] != 3
    ch = [torch.cat([c[keep], h]) for c, h in zip(ch, (torch.full((40000,), 3, dtype=torch.int32),
                                                       (cells // 4).to(torch.int32), (cells % 4).to(torch.int32)))]
    vh = torch.cat([vh[keep], _dense(407, 40000)])
    Bh, Ch = _dense(408, 20000, 24), _dense(409, 4, 24)
    for opts in ("force_generic=1", "force_generic=1,generic_fuse=0"):
        got, pl = _run(text, (ch, vh, dimsh), [0, 1, 2], [("C", Ch), ("B", Bh)], (10, 24), options=opts)
        _check(got, ch, vh, "ijk", [(Bh, "jr"), (Ch, "kr")], "ir", {"i": 10, "r": 24})
    _say("a leaf mode of 2^24 + 5 indices: row offsets in 64-bit arithmetic")
    dimsw = (20, 30, (1 << 24) + 5)
    cw, vw = _tensor(402, (20, 30, 4096), 6000)
    cw[2] = (cw[2].long() * 4097 % dimsw[2]).to(torch.int32)          # distinct, spread over the whole mode
    cw[2][0] = dimsw[2] - 1
    Bw, Cw = _dense(403, 30, 8), _dense(404, dimsw[2], 8)
    got, pl = _run(text, (cw, vw, dimsw), [0, 1, 2], [("C", Cw), ("B", Bw)], (20, 8), options="force_generic=1")
    assert "inlined_producers=1" in pl.describe(), pl.describe()
    _check(got, cw, vw, "ijk", [(Bw, "jr"), (Cw, "kr")], "ir", {"i": 20, "r": 8})
    U2, U3 = _dense(400, 45, 72), _dense(401, 38, 8)
    got, pl = _run("T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s ; Y[i,r,s] = T[i,j,s] * U2[j,r] | i,j,r,s",
                   x, [0, 1, 2], [("U3", U3), ("U2", U2)], (70, 72, 8))
    assert "inlined_producers=0" in pl.describe(), pl.describe()


@pytest.mark.parametrize("reroot", [0, 1])
def test_every_output_mode_on_one_csf(reroot):
    # Sec. 5.3 runs MTTKRP / TTMc for every mode; here all of them on the SAME CSF (i > j > k).  reroot=0: the
    # generic executor (a result that keeps a level other than the root is stored dense and added into);
    # reroot=1 (default): the plan's private copy of the tensor with the output level at the root and the
    # kernels of the root-mode case
    opts = {"reroot": reroot}
    fam_m, fam_t = ("mttkrp3", "ttmc3") if reroot else ("generic", "generic")
    dims = (33, 21, 27)
    coords, vals = _tensor(371, dims, 3500)
    x = (coords, vals, dims)
    A, B, C = _dense(372, 33, 12), _dense(373, 21, 12), _dense(374, 27, 12)
    _say("MTTKRP mode 1: leaf factor first, then the root factor, result indexed by the middle level")
    got, _ = _run("T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; M[j,r] = T[i,j,r] * A[i,r] | i,j,r",
                  x, [0, 1, 2], [("C", C), ("A", A)], (21, 12), expect=fam_m, options=opts)
    _check(got, coords, vals, "ijk", [(A, "ir"), (C, "kr")], "jr", {"j": 21, "r": 12})
    _say("MTTKRP mode 2: Khatri-Rao rows of the two upper levels at X's fibers only, result indexed by the leaf level")
    got, pl = _run("T[i,j,r] = A[i,r] * B[j,r] | i,j,r ; M[k,r] = X[i,j,k] * T[i,j,r] | i,j,k,r",
                   x, [0, 1, 2], [("A", A), ("B", B)], (27, 12), expect=fam_m, options=opts)
    assert ("private copy of the tensor with level 2 at the root" in pl.describe()) == bool(reroot)
    _check(got, coords, vals, "ijk", [(A, "ir"), (B, "jr")], "kr", {"k": 27, "r": 12})
    again = cst.execute(pl, [A.cuda(), B.cuda()]).cpu().numpy().reshape(27, 12)     # cleared before each run
    np.testing.assert_allclose(again, got, rtol=0, atol=1e-9)
    U1, U2, U3 = _dense(375, 33, 3), _dense(376, 21, 4), _dense(377, 27, 5)
    _say("TTMc mode 1")
    got, _ = _run("T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s ; Y[j,a,s] = T[i,j,s] * U1[i,a] | i,j,a,s",
                  x, [0, 1, 2], [("U3", U3), ("U1", U1)], (21, 3, 5), expect=fam_t, options=opts)
    _check(got, coords, vals, "ijk", [(U1, "ia"), (U3, "ks")], "jas", {"j": 21, "a": 3, "s": 5})
    _say("TTMc mode 2")
    got, _ = _run("P[i,j,a,b] = U1[i,a] * U2[j,b] | i,j,a,b ; Y[k,a,b] = X[i,j,k] * P[i,j,a,b] | i,j,k,a,b",
                  x, [0, 1, 2], [("U1", U1), ("U2", U2)], (27, 3, 4), expect=fam_t, options=opts)
    _check(got, coords, vals, "ijk", [(U1, "ia"), (U2, "jb")], "kab", {"k": 27, "a": 3, "b": 4})
    _say("TTMc mode 2 with the ranks listed the other way round, MTTKRP mode 1 with rank 32 and compact rows")
    got, _ = _run("P[i,j,a,b] = U1[i,a] * U2[j,b] | i,j,a,b ; Y[k,b,a] = X[i,j,k] * P[i,j,a,b] | i,j,k,b,a",
                  x, [0, 1, 2], [("U1", U1), ("U2", U2)], (27, 4, 3), expect=fam_t, options=opts)
    _check(got, coords, vals, "ijk", [(U1, "ia"), (U2, "jb")], "kba", {"k": 27, "a": 3, "b": 4})
    A32, C32 = _dense(378, 33, 32), _dense(379, 27, 32)
    got, pl = _run("T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; M[j,r] = T[i,j,r] * A[i,r] | i,j,r",
                   x, [0, 1, 2], [("C", C32), ("A", A32)], (21, 32), expect=fam_m, options=opts)
    _check(got, coords, vals, "ijk", [(A32, "ir"), (C32, "kr")], "jr", {"j": 21, "r": 32})


def test_trees_that_only_look_like_a_non_root_mttkrp_stay_with_the_generic_executor():
    # the middle index is summed before its factor joins: an outer product with B's rows, not an MTTKRP
    dims = (9, 7, 8)
    coords, vals = _tensor(381, dims, 200)
    B, C = _dense(382, 7, 5), _dense(383, 8, 5)
    got, _ = _run("T[i,r] = X[i,j,k] * C[k,r] | i,j,k,r ; M[j,r] = T[i,r] * B[j,r] | i,j,r",
                  (coords, vals, dims), [0, 1, 2], [("C", C), ("B", B)], (7, 5), expect="generic")
    c = [t.numpy() for t in coords]
    T = np.zeros((9, 5))
    np.add.at(T, c[0], vals.numpy()[:, None] * C.numpy()[c[2]])
    want = T.sum(0)[None, :] * B.numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_inputs_indexed_by_kept_levels_and_results_with_several_sparse_indices():
    dims = (20, 12, 9)
    coords, vals = _tensor(361, dims, 500)
    x = (coords, vals, dims)
    B, C, U3, wj = _dense(362, 12, 4), _dense(364, 9, 4), _dense(363, 9, 4), _dense(365, 12)
    _say("a factor indexed by a level the result keeps, result still a CSF prefix")
    got, _ = _run("T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; S[i,j,r] = T[i,j,r] * B[j,r] | i,j,r ; "
                  "M[i,r] = S[i,j,r] * w[j] | i,j,r", x, [0, 1, 2], [("C", C), ("B", B), ("w", wj)], (20, 4))
    _check(got, coords, vals, "ijk", [(B, "jr"), (C, "kr"), (wj, "j")], "ir", {"i": 20, "r": 4})
    _say("contracting the middle level first leaves (i,k): held dense, the rest of the tree is dense")
    got, _ = _run("T[i,k,r] = X[i,j,k] * B[j,r] | i,j,k,r ; Y[i,r,s] = T[i,k,r] * U3[k,s] | i,k,r,s",
                  x, [0, 1, 2], [("B", B), ("U3", U3)], (20, 4, 4))
    _check(got, coords, vals, "ijk", [(B, "jr"), (U3, "ks")], "irs", {"i": 20, "r": 4, "s": 4})
    _say("a result that keeps two sparse indices comes out dense over both")
    got, _ = _run("T[i,j,s] = X[i,j,k] * U3[k,s] | i,j,k,s", x, [0, 1, 2], [("U3", U3)], (20, 12, 4))
    _check(got, coords, vals, "ijk", [(U3, "ks")], "ijs", {"i": 20, "j": 12, "s": 4})


def test_fused_pair_whose_result_keeps_no_sparse_index():
    # order-2 X: z[r] = sum_{i,k} X[i,k] C[k,r] A[i,r]; the consumer's result node is the (absent) root, so all
    # leaves of X hang below ONE node: leaf segments and the workgroup that adds their partial sums
    dims = (900, 700)
    for nnz in (300, 60_000):
        coords, vals = _tensor(421 + nnz, dims, nnz)
        A, C = _dense(422, 900, 12), _dense(423, 700, 12)
        text = "T[i,r] = X[i,k] * C[k,r] | i,k,r ; z[r] = T[i,r] * A[i,r] | i,r"
        got, pl = _run(text, (coords, vals, dims), [0, 1], [("C", C), ("A", A)], (12,))
        assert "inlined_producers=1" in pl.describe(), pl.describe()
        _check(got, coords, vals, "ik", [(A, "ir"), (C, "kr")], "r", {"r": 12})
        stored, _ = _run(text, (coords, vals, dims), [0, 1], [("C", C), ("A", A)], (12,), options="generic_fuse=0")
        np.testing.assert_allclose(stored, got, rtol=0, atol=1e-9)


def _with_heavy_slice(seed, coords, vals, dims, root, count):
    """Adds `count` nonzeros in root slice `root`, at distinct cells below it, and drops duplicates."""
    g = torch.Generator().manual_seed(seed)
    below = int(np.prod(dims[1:]))
    cells = torch.randperm(below, generator=g)[:count]
    extra = []
    for d in reversed(dims[1:]):
        extra.append((cells % d).to(torch.int32))
        cells = cells // d
    extra.append(torch.full((count,), root, dtype=torch.int32))
    extra.reverse()
    coords = [torch.cat([c, e]) for c, e in zip(coords, extra)]
    vals = torch.cat([vals, torch.rand(count, generator=g, dtype=torch.float64) - 0.5])
    key = torch.zeros(vals.numel(), dtype=torch.int64)
    for c, d in zip(coords, dims):
        key = key * d + c.long()
    _, first = np.unique(key.numpy(), return_index=True)
    return [c[first] for c in coords], vals[first]


def test_fused_chain_of_producers_is_one_kernel():
    # Sec. 2.2 / Fig. 3b: every statement of an MTTKRP chain fused with the next on the whole prefix leaves one
    # loop nest with scalar intermediates.  The executor then runs the chain as ONE kernel, up to three
    # producers deep; it must equal the N-ary sum, the stored form, and itself when cut into leaf segments.
    dims = (40, 17, 19, 15)
    coords, vals = _tensor(431, dims, 9000)
    coords, vals = _with_heavy_slice(432, coords, vals, dims, 7, 3000)
    x = (coords, vals, dims)
    for R in (24, 40):
        B, C, D = _dense(433, 17, R), _dense(434, R, 19), _dense(435, 15, R)         # C stored rank-major
        text = ("T1[i,j,k,r] = X[i,j,k,l] * D[l,r] | i,j,k,l,r ; T2[i,j,r] = T1[i,j,k,r] * C[r,k] | i,j,k,r ; "
                "M[i,r] = T2[i,j,r] * B[j,r] | i,j,r")
        ops = [("D", D), ("C", C), ("B", B)]
        f = [(B, "jr"), (C, "rk"), (D, "lr")]
        _say("order 4, rank %d" % R)
        got, pl = _run(text, x, [0, 1, 2, 3], ops, (40, R))
        assert "kernels=1 inlined_producers=2" in pl.describe(), pl.describe()
        _check(got, coords, vals, "ijkl", f, "ir", {"i": 40, "r": R})
        stored, pl = _run(text, x, [0, 1, 2, 3], ops, (40, R), options="generic_fuse=0")
        assert "kernels=3 inlined_producers=0" in pl.describe(), pl.describe()
        np.testing.assert_allclose(stored, got, rtol=0, atol=1e-10)
        for span in (16, 700):
            seg, pl = _run(text, x, [0, 1, 2, 3], ops, (40, R), options="generic_span=%d" % span)
            assert "kernels=1 inlined_producers=2" in pl.describe(), pl.describe()
            _check(seg, coords, vals, "ijkl", f, "ir", {"i": 40, "r": R})
        # rows of 24 or 40 doubles with the rank index innermost in D and B, rank-major C: one element per lane;
        # all three rank-innermost: two per lane, unless an array does not begin on 16 bytes
        assert "two_elements_per_lane=0" in pl.describe(), pl.describe()
        Ct = C.t().contiguous()
        text2 = text.replace("C[r,k]", "C[k,r]")
        two, pl = _run(text2, x, [0, 1, 2, 3], [("D", D), ("C", Ct), ("B", B)], (40, R), options="generic_span=700")
        assert "two_elements_per_lane=1" in pl.describe(), pl.describe()
        np.testing.assert_allclose(two, got, rtol=0, atol=1e-10)
        # an operand that begins 8 bytes past a 16-byte boundary
        csf = cst.build_csf([c.cuda() for c in coords], vals.cuda(), dims, [0, 1, 2, 3])
        dev = [D.cuda(), Ct.cuda(), torch.zeros(B.numel() + 1, dtype=torch.float64).cuda()[1:].view_as(B).copy_(B.cuda())]
        assert dev[2].data_ptr() % 16 == 8
        pl = cst.plan(text2, [("X", csf), ("D", dev[0]), ("C", dev[1]), ("B", dev[2])])
        one = cst.execute(pl, dev).cpu().numpy().reshape(40, R)
        np.testing.assert_allclose(one, got, rtol=0, atol=1e-10)
        pair, pl = _run(text, x, [0, 1, 2, 3], ops, (40, R), fusion=[3, 1, 0])       # the second pair fused on i only
        assert "kernels=2 inlined_producers=1" in pl.describe(), pl.describe()
        np.testing.assert_allclose(pair, got, rtol=0, atol=1e-10)

    _say("order 5 in one kernel, order 6 in two; two dense indices whose order changes along the chain")
    dims5 = (12, 9, 8, 7, 6)
    c5, v5 = _tensor(436, dims5, 7000)
    c5, v5 = _with_heavy_slice(437, c5, v5, dims5, 2, 2500)
    F = [_dense(438 + m, dims5[m], 5, 3) for m in range(1, 5)]
    t5 = ("T1[i,j,k,l,r,s] = X[i,j,k,l,m] * F4[m,r,s] | i,j,k,l,m,r,s ; T2[i,j,k,s,r] = T1[i,j,k,l,r,s] * F3[l,r,s] | i,j,k,l,s,r ; "
          "T3[i,j,r,s] = T2[i,j,k,s,r] * F2[k,r,s] | i,j,k,r,s ; M[i,s,r] = T3[i,j,r,s] * F1[j,r,s] | i,j,s,r")
    ops5 = [("F4", F[3]), ("F3", F[2]), ("F2", F[1]), ("F1", F[0])]
    f5 = [(F[0], "jrs"), (F[1], "krs"), (F[2], "lrs"), (F[3], "mrs")]
    for opts in (None, "generic_span=32"):
        got, pl = _run(t5, (c5, v5, dims5), [0, 1, 2, 3, 4], ops5, (12, 3, 5), options=opts)
        assert "kernels=1 inlined_producers=3" in pl.describe(), pl.describe()
        _check(got, c5, v5, "ijklm", f5, "isr", {"i": 12, "s": 3, "r": 5})
    dims6 = (6, 5, 6, 5, 4, 7)
    c6, v6 = _tensor(443, dims6, 6000)
    G = [_dense(444 + m, dims6[m], 16) for m in range(1, 6)]
    t6 = ("T1[a,b,c,d,e,r] = X[a,b,c,d,e,f] * G5[f,r] | a,b,c,d,e,f,r ; T2[a,b,c,d,r] = T1[a,b,c,d,e,r] * G4[e,r] | a,b,c,d,e,r ; "
          "T3[a,b,c,r] = T2[a,b,c,d,r] * G3[d,r] | a,b,c,d,r ; T4[a,b,r] = T3[a,b,c,r] * G2[c,r] | a,b,c,r ; "
          "M[a,r] = T4[a,b,r] * G1[b,r] | a,b,r")
    got, pl = _run(t6, (c6, v6, dims6), [0, 1, 2, 3, 4, 5], [("G5", G[4]), ("G4", G[3]), ("G3", G[2]), ("G2", G[1]), ("G1", G[0])], (6, 16))
    assert "kernels=2 inlined_producers=3" in pl.describe(), pl.describe()
    _check(got, c6, v6, "abcdef", [(G[0], "br"), (G[1], "cr"), (G[2], "dr"), (G[3], "er"), (G[4], "fr")], "ar", {"a": 6, "r": 16})

    _say("a chain whose result keeps no sparse index: every leaf below one node")
    dims3 = (300, 40, 50)
    c3, v3 = _tensor(451, dims3, 30_000)
    A, B3, C3 = _dense(452, 300, 12), _dense(453, 40, 12), _dense(454, 50, 12)
    t3 = "T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; T2[i,r] = T[i,j,r] * B[j,r] | i,j,r ; z[r] = T2[i,r] * A[i,r] | i,r"
    got, pl = _run(t3, (c3, v3, dims3), [0, 1, 2], [("C", C3), ("B", B3), ("A", A)], (12,))
    assert "kernels=1 inlined_producers=2" in pl.describe(), pl.describe()
    _check(got, c3, v3, "ijk", [(A, "ir"), (B3, "jr"), (C3, "kr")], "r", {"r": 12})


def test_running_example_with_four_sparse_operands():
    # Sec. 3.1 / Fig. 4: R_ijk = A_ipq B_jpr C_kqr D_jkr as X = A.B ; Y = X.C ; R = Y.D with the layouts and loop
    # orders of the paper's constraint solution, all four tensors sparse.  The executor walks the operand
    # with the most nonzeros and keeps dense copies of the other three.
    P, Q, I, R, J, K = 7, 4, 8, 5, 6, 9
    Ac, Av = _tensor(411, (P, Q, I), 90)
    Bc, Bv = _tensor(412, (R, J, P), 70)
    Cc, Cv = _tensor(413, (R, Q, K), 50)
    Dc, Dv = _tensor(414, (R, J, K), 80)
    text = ("X[r,j,q,i] = A[p,q,i] * B[r,j,p] | r,j,p,q,i ; Y[r,j,k,i] = X[r,j,q,i] * C[r,q,k] | r,j,q,k,i ; "
            "R[j,k,i] = Y[r,j,k,i] * D[r,j,k] | r,j,k,i")
    ops = [(n, cst.build_csf([c.cuda() for c in cc], vv.cuda(), dims, [0, 1, 2]))
           for n, cc, vv, dims in (("A", Ac, Av, (P, Q, I)), ("B", Bc, Bv, (R, J, P)), ("C", Cc, Cv, (R, Q, K)), ("D", Dc, Dv, (R, J, K)))]
    pl = cst.plan(text, ops, fusion=[2, 2, 0])
    desc = pl.describe()
    _say("  " + desc.split("|")[0])
    assert "family=generic" in desc and "dense_copies_of_csf_operands=3" in desc and "X:order2 Y:order2" in desc, desc
    got = cst.execute(pl, []).cpu().numpy().reshape(J, K, I)

    def spread(cc, vv, dims):
        t = np.zeros(dims)
        t[tuple(c.numpy() for c in cc)] = vv.numpy()
        return t
    _check(got, Ac, Av, "pqi", [(torch.from_numpy(spread(Bc, Bv, (R, J, P))), "rjp"), (torch.from_numpy(spread(Cc, Cv, (R, Q, K))), "rqk"),
                                (torch.from_numpy(spread(Dc, Dv, (R, J, K))), "rjk")], "jki", {"j": J, "k": K, "i": I})
    with pytest.raises(cst.ConststnError) as e:
        cst.plan(text, ops, fusion=[2, 2, 0], options={"generic_densify": 0})
    assert e.value.status_name == "EUNSUPPORTED"
    big = cst.build_csf([torch.zeros(1, dtype=torch.int32).cuda()] * 3, torch.ones(1, dtype=torch.float64).cuda(), (R, P, 1 << 30), [0, 1, 2])
    with pytest.raises(cst.ConststnError) as e:       # 5 x 7 x 2^30 doubles: beyond the bound on dense copies
        cst.plan("T[r,j,i] = A2[r,j,p] * B2[r,p,i] | r,j,p,i", [("A2", ops[1][1]), ("B2", big)])
    assert "generic_max_gb" in str(e.value)


def test_generic_refuses_what_it_cannot_store():
    # a Khatri-Rao product over two non-root levels is not a CSF prefix: held dense, 2 GB here
    dims = (20, 4000, 4000)
    coords, vals = _tensor(361, dims, 500)
    csf = cst.build_csf([c.cuda() for c in coords], vals.cuda(), dims, [0, 1, 2])
    B, C = _dense(362, 4000, 16).cuda(), _dense(363, 4000, 16).cuda()
    text = "P[j,k,r] = B[j,r] * C[k,r] | j,k,r ; M[i,r] = X[i,j,k] * P[j,k,r] | i,j,k,r"
    with pytest.raises(cst.ConststnError) as e:
        cst.plan(text, [("X", csf), ("B", B), ("C", C)], options={"generic_max_gb": 1})
    assert "intermediates" in str(e.value)
