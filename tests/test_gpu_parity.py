"""GPU parity: the HIP library against the CPU oracle on the same seeded inputs, element by
element; CSF arrays bit-exact against the reference build; edge cases."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_2401_04836_amd as cst
import workloads as w
from paper_2401_04836_amd import schedules as S
from helpers import TOL, check_csf_bit_exact, compare, run_gpu, run_oracle, to_dev

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)


@pytest.mark.parametrize("dims,nnz", [((23, 17, 31), 3000), ((7, 9, 5, 11), 2000), ((50, 40), 700), ((97,), 40)])
def test_csf_bit_exact_every_mode_order(dims, nnz):
    rng = np.random.default_rng(5)
    flat = rng.choice(int(np.prod(dims)), size=nnz, replace=False)
    coords = [c.astype(np.int32) for c in np.unravel_index(flat, dims)]
    vals = rng.normal(size=nnz)
    dc = [torch.from_numpy(c).cuda() for c in coords]
    dv = torch.from_numpy(vals).cuda()
    for mo in itertools.permutations(range(len(dims))):
        _say("csf dims=%s mode_order=%s" % (dims, mo))
        csf = cst.build_csf(dc, dv, dims, list(mo))
        check_csf_bit_exact(csf, coords, vals, dims, mo)
        assert csf.nnz == nnz and csf.mode_order == tuple(mo)
        csf.destroy()


@pytest.mark.parametrize("dims,nnz", [(((1 << 22) + 3, (1 << 22) + 1, (1 << 25) + 7), 30_011),        # 72 key bits
                                      (((1 << 20) + 1,) * 4, 9_001),                                   # 84
                                      (((1 << 30) + 5, 3, (1 << 30) + 9, (1 << 29) + 1, 7), 5_003)])   # 31+2+31+30+3 = 97
def test_csf_keys_of_two_words(dims, nnz):
    """Coordinate tuples that do not fit one 64-bit sort key (a tensor the size of FROSTT's largest needs 69
    bits): the outer levels go to a second key word.  Clustered coordinates so that every level has nodes
    with several children, plus duplicates of one tuple for the coalescing path."""
    rng = np.random.default_rng(17)
    order = len(dims)
    coords = []
    for m, d in enumerate(dims):
        pool = np.unique(rng.integers(0, d, size=max(2, min(40, d))))           # few distinct values per mode, spread over its range
        pool[-1] = d - 1
        coords.append(pool[rng.integers(0, pool.size, size=nnz)].astype(np.int64))
    key = np.stack(coords, 1)
    _, first = np.unique(key, axis=0, return_index=True)
    coords = [c[np.sort(first)].astype(np.int32) for c in coords]
    n = coords[0].size
    vals = rng.normal(size=n)
    dc = [torch.from_numpy(c).cuda() for c in coords]
    dv = torch.from_numpy(vals).cuda()
    orders = list(itertools.permutations(range(order))) if order <= 3 else [tuple(range(order)), tuple(reversed(range(order))), (1, 3, 0, 2, 4)[:order] if order == 5 else (2, 0, 3, 1)]
    for mo in orders:
        _say("csf dims=%s mode_order=%s (%d nonzeros)" % (dims, mo, n))
        csf = cst.build_csf(dc, dv, dims, list(mo))
        check_csf_bit_exact(csf, coords, vals, dims, mo)
        csf.destroy()
    # the same tuple three times: refused as a set, summed in input order with the flag
    dup_c = [torch.cat([c, c[:1], c[:1]]) for c in dc]
    dup_v = torch.cat([dv, dv[:1] * 2, dv[:1] * 4])
    with pytest.raises(cst.ConststnError) as e:
        cst.build_csf(dup_c, dup_v, dims, list(range(order)))
    assert e.value.status_name == "EDUP"
    csf = cst.build_csf(dup_c, dup_v, dims, list(range(order)), flags=cst.COALESCE_DUPS)
    vals2 = vals.copy()
    vals2[0] = (vals[0] + 2 * vals[0]) + 4 * vals[0]
    check_csf_bit_exact(csf, coords, vals2, dims, tuple(range(order)))
    with pytest.raises(cst.ConststnError) as e:           # 5 x 31 bits: the outer fields alone exceed a word
        cst.build_csf([c[:4] for c in dc[:1]] * 5, dv[:4], ((1 << 30) + 5,) * 5, [0, 1, 2, 3, 4])
    assert e.value.status_name == "EUNSUPPORTED"


def test_mttkrp_on_a_tensor_with_two_word_keys():
    """The contraction kernels read the level arrays only: a CSF built from 72-bit tuples runs like any other."""
    dims = ((1 << 22) + 3, (1 << 22) + 1, (1 << 25) + 7)
    rng = np.random.default_rng(23)
    nnz = 20_000
    coords = [rng.integers(0, 300, size=nnz) * (d // 300) for d in dims]
    key = np.stack(coords, 1)
    _, first = np.unique(key, axis=0, return_index=True)
    coords = [c[first].astype(np.int32) for c in coords]
    vals = rng.normal(size=coords[0].size)
    csf = cst.build_csf([torch.from_numpy(c).cuda() for c in coords], torch.from_numpy(vals).cuda(), dims, [0, 1, 2])
    B = (torch.rand(dims[1], 4, generator=torch.Generator().manual_seed(1), dtype=torch.float64) * 2 - 1)
    C = (torch.rand(dims[2], 4, generator=torch.Generator().manual_seed(2), dtype=torch.float64) * 2 - 1)
    pl = cst.plan(S.MTTKRP3, [("X", csf), ("C", C.cuda()), ("B", B.cuda())], flags=cst.OUT_COMPACT)
    out = cst.execute(pl, [C.cuda(), B.cuda()]).reshape(pl.n_rows, 4).cpu().numpy()
    rows = pl.output_rows().cpu().numpy().astype(np.int64)
    want = oracle.mttkrp3(coords, vals, dims, B.numpy(), C.numpy(), 0)
    S_abs = oracle.mttkrp3_abs(coords, vals, dims, B.numpy(), C.numpy(), 0)
    np.testing.assert_array_equal(rows, np.unique(coords[0]))
    keep = np.zeros(dims[0], dtype=bool)
    keep[rows] = True
    assert not S_abs[~keep].any()
    want, S_abs = want[rows], S_abs[rows]
    assert oracle.rel_err(out, want, S_abs) <= TOL


def test_csf_spans_many_tiles_with_ragged_tail():
    wl = w.make(2, small=True)                       # 150 001 nonzeros: 74 tiles, ragged tail
    X = wl.sparse["X"]
    c, v = X.numpy()
    dc, dv = to_dev(X)
    for mo in ([0, 1, 2], [2, 1, 0], [1, 2, 0]):
        _say("csf c2-small mode_order=%s" % mo)
        csf = cst.build_csf(dc, dv, X.dims, mo)
        check_csf_bit_exact(csf, c, v, X.dims, mo)


@pytest.mark.parametrize("nnz", [1, 63, 64, 65, 255, 256, 257, 2047, 2048, 2049, 4095, 4096, 4097, 6145, 8191, 8192, 8193, 12289])
def test_csf_sizes_at_tile_edges(nnz):
    """Sizes one below, at and one above the lengths the build kernels cut their input into (wavefronts of
    64, chunks of 256, tiles of 2048 and 4096 pairs), and runs of duplicates that begin in one tile and end
    in the next: summed in input order with the flag, refused without."""
    dims = (6, 50, 70)
    rng = np.random.default_rng(300 + nnz)
    flat = rng.choice(int(np.prod(dims)), size=nnz, replace=False)
    coords = [c.astype(np.int32) for c in np.unravel_index(flat, dims)]
    vals = rng.normal(size=nnz)
    dc = [torch.from_numpy(c).cuda() for c in coords]
    dv = torch.from_numpy(vals).cuda()
    for mo in ([0, 1, 2], [2, 0, 1]):
        _say("csf %d nonzeros, mode_order=%s" % (nnz, mo))
        csf = cst.build_csf(dc, dv, dims, mo)
        csf.check()
        check_csf_bit_exact(csf, coords, vals, dims, mo)
    if nnz < 2049:
        return
    # three more copies of the tuples that sort to places 2047 and 4091: the runs then cover places
    # 2047..2050 and, three places further back because of the first run, 4094..4097 -- across the edge of a
    # 2048-pair tile and of a 4096-pair tile
    key = (coords[0].astype(np.int64) * dims[1] + coords[1]) * dims[2] + coords[2]
    rank = np.argsort(key, kind="stable")
    picks = [int(rank[2047])] + ([int(rank[4091])] if nnz > 4094 else [])
    extra = np.array([p for p in picks for _ in range(3)], dtype=np.int64)
    weights = rng.integers(2, 9, size=extra.size).astype(np.float64)
    dup_c = [torch.from_numpy(np.concatenate([c, c[extra]])).cuda() for c in coords]
    dup_v = torch.from_numpy(np.concatenate([vals, vals[extra] * weights])).cuda()
    with pytest.raises(cst.ConststnError) as e:
        cst.build_csf(dup_c, dup_v, dims, [0, 1, 2])
    assert e.value.status_name == "EDUP"
    csf = cst.build_csf(dup_c, dup_v, dims, [0, 1, 2], flags=cst.COALESCE_DUPS)
    want = vals.copy()
    for p, wgt in zip(extra, weights):                    # in input order: the original first, then the copies as appended
        want[p] = want[p] + vals[p] * wgt
    check_csf_bit_exact(csf, coords, want, dims, (0, 1, 2))


def test_csf_errors_and_edge_cases():
    dims = (4, 5, 6)
    c = [torch.tensor([1, 1], dtype=torch.int32).cuda(), torch.tensor([2, 2], dtype=torch.int32).cuda(),
         torch.tensor([3, 3], dtype=torch.int32).cuda()]
    v = torch.tensor([1.5, 2.25], dtype=torch.float64).cuda()
    with pytest.raises(cst.ConststnError) as e:
        cst.build_csf(c, v, dims, [0, 1, 2])
    assert e.value.status_name == "EDUP"
    csf = cst.build_csf(c, v, dims, [0, 1, 2], flags=cst.COALESCE_DUPS)      # summed in input order
    assert csf.nnz == 1 and csf.export(2)[2].cpu().tolist() == [3.75]
    bad = [c[0], c[1], torch.tensor([3, 6], dtype=torch.int32).cuda()]
    with pytest.raises(cst.ConststnError) as e:
        cst.build_csf(bad, v, dims, [0, 1, 2])
    assert e.value.status_name == "ERANGE"
    with pytest.raises(cst.ConststnError) as e:
        cst.build_csf(c, v, dims, [0, 1, 1])
    assert e.value.status_name == "EINVAL"
    empty = [torch.zeros(0, dtype=torch.int32).cuda()] * 3
    csf = cst.build_csf(empty, torch.zeros(0, dtype=torch.float64).cuda(), dims, [2, 0, 1])
    assert csf.nnz == 0 and [csf.nodes(l) for l in range(3)] == [0, 0, 0]
    assert csf.export(0)[1].cpu().tolist() == [0] and csf.export(1)[1].cpu().tolist() == [0]
    # one nonzero
    one = [torch.tensor([3], dtype=torch.int32).cuda(), torch.tensor([4], dtype=torch.int32).cuda(),
           torch.tensor([5], dtype=torch.int32).cuda()]
    csf = cst.build_csf(one, torch.tensor([2.0], dtype=torch.float64).cuda(), dims, [0, 1, 2])
    assert [csf.export(l)[0].cpu().tolist() for l in range(3)] == [[3], [4], [5]]


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_small_configs_match_oracle(cid):
    _say("parity config %d (reduced copy, dense output)" % cid)
    wl = w.make(cid, small=True)
    out, pl, _ = run_gpu(wl, check_csf=True)
    want, S_abs = run_oracle(wl)
    err = compare(out, want, S_abs)
    _say("  %s -> rel err %.3e" % (pl.describe().split("|")[0], err))
    assert err <= TOL


def test_config1_full_size():
    _say("parity config 1 full size")
    wl = w.make(1)
    out, pl, _ = run_gpu(wl, check_csf=True)
    want, S_abs = run_oracle(wl)
    assert compare(out, want, S_abs) <= TOL


@pytest.mark.parametrize("cid", [1, 2, 3, 5])
def test_compact_output(cid):
    _say("compact output config %d" % cid)
    wl = w.make(cid, small=True)
    out, pl, _ = run_gpu(wl, flags=cst.OUT_COMPACT)
    rows = pl.output_rows()
    want, S_abs = run_oracle(wl)
    assert rows.numel() == pl.n_rows and bool((rows[1:] > rows[:-1]).all())
    assert compare(out, want, S_abs, rows=rows) <= TOL


@pytest.mark.parametrize("rank", [32, 20])
def test_mttkrp_compact_rows_with_empty_and_heavy_slices(rank):
    """Rank 32 takes the kernels that split the leaves into hot and cold sub-tensors (rows of the output
    renumbered per sub-tensor); 4001 root indices for 40 003 power-law nonzeros leave most slices empty
    and put a fifth of the leaves into one."""
    _say("mttkrp rank %d, compact rows, empty and heavy slices" % rank)
    wl = w.make(2, small=True, dims=(4001, 211, 503), nnz=40_003, rank=rank)
    out, pl, _ = run_gpu(wl, flags=cst.OUT_COMPACT)
    rows = pl.output_rows()
    assert 0 < rows.numel() < 4001 and bool((rows[1:] > rows[:-1]).all())
    want, S_abs = run_oracle(wl)
    assert compare(out, want, S_abs, rows=rows) <= TOL
    dense, _, _ = run_gpu(wl)
    assert torch.equal(dense[rows.long()], out)


@pytest.mark.parametrize("dual", [0, 35, 53, 88])
def test_mttkrp_hot_and_cold_passes_in_one_launch_or_two(dual):
    """The default runs the hot and the cold sub-tensor as two teams of wavefronts in one launch (the cold
    team into a buffer of its own, added afterwards); other team sizes and the two-launch form must agree."""
    _say("mttkrp rank 32, mttkrp_dual=%d" % dual)
    wl = w.make(2, small=True, dims=(4001, 211, 503), nnz=40_003, rank=32)
    want, S_abs = run_oracle(wl)
    for flags in (0, cst.OUT_COMPACT):
        out, pl, _ = run_gpu(wl, flags=flags, options={"mttkrp_dual": dual})
        assert compare(out, want, S_abs, rows=pl.output_rows() if flags else None) <= TOL
    wl = w.make(2, small=True)
    out, pl, _ = run_gpu(wl, options={"mttkrp_dual": dual})
    want, S_abs = run_oracle(wl)
    assert compare(out, want, S_abs) <= TOL


def test_table_check_covers_what_it_says():
    """The table check runs inside run_gpu for every MTTKRP / TTMc case; here: other families say so, the
    private re-rooted copy is checked like the caller's tensor, and the sparse-result structure handed out by a
    plan passes the CSF check."""
    wl = w.make(3, small=True)
    _, pl, _ = run_gpu(wl)
    with pytest.raises(cst.ConststnError) as e:
        pl.check()
    assert e.value.status_name == "EUNSUPPORTED"
    wl = w.make(2, small=True)
    X = wl.sparse["X"]
    dc, dv = to_dev(X)
    csf = cst.build_csf(dc, dv, X.dims, [0, 1, 2])
    A, C = wl.dense["B"].new_ones(X.dims[0], 32).cuda(), wl.dense["C"].cuda()
    pl = cst.plan("T[i,j,r] = X[i,j,k] * C[k,r] | i,j,k,r ; M[j,r] = T[i,j,r] * A[i,r] | i,j,r", [("X", csf), ("C", C), ("A", A)])
    assert "private copy" in pl.describe()
    pl.check()
    for opts in ({"mttkrp_split": 0}, {"mttkrp_dual": 0}, {"ttmc3_stream": 0}):
        for cid in (2, 5):
            _, pl, csfs = run_gpu(w.make(cid, small=True), options=opts)
            pl.check()
            csfs[0].check()


def test_plan_options_are_checked():
    wl = w.make(1)
    X = wl.sparse["X"]
    dc, dv = to_dev(X)
    csf = cst.build_csf(dc, dv, X.dims, [0, 1, 2])
    U2, U3 = wl.dense["U2"].cuda(), wl.dense["U3"].cuda()
    ops = [("X", csf), ("U3", U3), ("U2", U2)]
    assert "family=generic" in cst.plan(S.TTMC3, ops, options="force_generic=1").describe()
    assert "family=ttmc3" in cst.plan(S.TTMC3, ops, options=" ttmc3_split = 64 , ttmc3_mfma=0 ").describe()
    for bad in ("no_such_option=1", "ttmc3_split", "ttmc3_split=-4", "ttmc3_split=many",
                "ttmc3_split=0", "ttmc3_producers=5", "mttkrp_dual=45", "ttmc3_qn=3", "generic_span=0", "sptn3_tiled=3"):
        with pytest.raises(cst.ConststnError) as e:       # a value outside what the option takes is refused, never clamped
            cst.plan(S.TTMC3, ops, options=bad)
        assert e.value.status_name == "EINVAL", bad
    with pytest.raises(cst.ConststnError) as e:
        cst.plan(S.TTMC3, ops, options="ttmc3_producers=5")
    assert "2, 3, 4, 6, 8" in str(e.value)


def test_mttkrp_mode2_by_rerooted_csf():
    """Mode-2 MTTKRP: CSF k>j>i puts the output mode at the root (layout chosen per output mode)."""
    _say("mttkrp mode 2 via CSF k>j>i")
    wl = w.make(2, small=True)
    X = wl.sparse["X"]
    dc, dv = to_dev(X)
    csf = cst.build_csf(dc, dv, X.dims, [2, 1, 0])
    A, B = wl.dense["A"].cuda(), wl.dense["B"].cuda()
    pl = cst.plan("T[k,j,r] = X[k,j,i] * A[i,r] | k,j,i,r ; M[k,r] = T[k,j,r] * B[j,r] | k,j,r",
                  [("X", csf), ("A", A), ("B", B)])
    out = cst.execute(pl, [A, B]).reshape(pl.n_rows, -1)
    torch.cuda.synchronize()
    c, v = X.numpy()
    want = oracle.mttkrp3(c, v, X.dims, A.cpu().numpy(), B.cpu().numpy(), 2)
    S_abs = oracle.mttkrp3_abs(c, v, X.dims, A.cpu().numpy(), B.cpu().numpy(), 2)
    assert compare(out, want, S_abs) <= TOL


@pytest.mark.parametrize("rank", [1, 3, 8, 17, 32, 50, 64])
def test_mttkrp_ranks_and_heavy_slices(rank):
    _say("mttkrp rank %d" % rank)
    wl = w.make(2, small=True, dims=(301, 211, 503), nnz=40_003, rank=rank)
    out, pl, _ = run_gpu(wl)
    want, S_abs = run_oracle(wl)
    assert compare(out, want, S_abs) <= TOL


@pytest.mark.parametrize("ranks", [(1, 1), (3, 5), (8, 8), (16, 33), (64, 64), (50, 50), (16, 16),
                                   (32, 48), (48, 16), (64, 32)])
def test_ttmc3_ranks(ranks):
    _say("ttmc3 ranks %s" % (ranks,))
    wl = w.make(5, small=True, dims=(501, 409, 211), nnz=30_011, ranks=ranks)
    out, pl, _ = run_gpu(wl)
    want, S_abs = run_oracle(wl)
    assert compare(out, want, S_abs) <= TOL


@pytest.mark.parametrize("ranks", [(1, 1, 1), (3, 5, 2), (16, 16, 16), (7, 16, 9)])
def test_ttmc4_ranks(ranks):
    _say("ttmc4 ranks %s" % (ranks,))
    wl = w.make(3, small=True, dims=(19, 211, 199, 53), nnz=20_011, ranks=ranks)
    out, pl, _ = run_gpu(wl)
    want, S_abs = run_oracle(wl)
    assert compare(out, want, S_abs) <= TOL


def test_determinism_bitwise():
    for cid in (2, 3, 4, 5):
        _say("determinism config %d" % cid)
        wl = w.make(cid, small=True)
        a, _, _ = run_gpu(wl)
        b, _, _ = run_gpu(wl)
        assert torch.equal(a, b)


def test_empty_tensor_and_single_nonzero_execute():
    _say("empty tensor / single nonzero")
    dims = (6, 5, 4)
    U2 = torch.ones(5, 3, dtype=torch.float64).cuda()
    U3 = torch.ones(4, 2, dtype=torch.float64).cuda()
    empty = [torch.zeros(0, dtype=torch.int32).cuda()] * 3
    csf = cst.build_csf(empty, torch.zeros(0, dtype=torch.float64).cuda(), dims, [0, 1, 2])
    pl = cst.plan(S.TTMC3, [("X", csf), ("U3", U3), ("U2", U2)])
    out = cst.execute(pl, [U3, U2])
    assert out.numel() == 6 * 3 * 2 and not bool(out.any())
    plc = cst.plan(S.TTMC3, [("X", csf), ("U3", U3), ("U2", U2)], flags=cst.OUT_COMPACT)
    assert plc.n_rows == 0 and cst.execute(plc, [U3, U2]).numel() == 0
    plm = cst.plan(S.MTTKRP3, [("X", csf), ("C", torch.ones(4, 3, dtype=torch.float64).cuda()),
                               ("B", U2)])
    assert not bool(cst.execute(plm, [torch.ones(4, 3, dtype=torch.float64).cuda(), U2]).any())
    one = [torch.tensor([2], dtype=torch.int32).cuda(), torch.tensor([4], dtype=torch.int32).cuda(),
           torch.tensor([1], dtype=torch.int32).cuda()]
    csf1 = cst.build_csf(one, torch.tensor([-0.5], dtype=torch.float64).cuda(), dims, [0, 1, 2])
    pl1 = cst.plan(S.TTMC3, [("X", csf1), ("U3", U3), ("U2", U2)])
    out = cst.execute(pl1, [U3, U2]).reshape(6, 3, 2).cpu()
    want = torch.zeros(6, 3, 2, dtype=torch.float64)
    want[2] = -0.5
    assert torch.equal(out, want)


def test_unsupported_and_illegal_plans():
    _say("plan errors")
    wl = w.make(1)
    X = wl.sparse["X"]
    dc, dv = to_dev(X)
    csf = cst.build_csf(dc, dv, X.dims, [0, 1, 2])
    U2, U3 = wl.dense["U2"].cuda(), wl.dense["U3"].cuda()
    # legal but unfused: none of the tuned kernels, so the generic executor takes it
    pl = cst.plan(S.TTMC3, [("X", csf), ("U3", U3), ("U2", U2)], fusion=[0, 0])
    assert "family=generic" in pl.describe()
    # two CSF operands outside the tuned sparse x sparse forms: the generic executor walks one and keeps a
    # dense copy of the other (here the same tensor under two names: Z_ij = sum_k X_ijk^2)
    text2 = "Z[i,j] = X[i,j,k] * W[i,j,k] | i,j,k"
    pl = cst.plan(text2, [("X", csf), ("W", csf)])
    assert "family=generic" in pl.describe() and "dense_copies_of_csf_operands=1" in pl.describe()
    got = cst.execute(pl, []).cpu().numpy().reshape(X.dims[0], X.dims[1])
    c, v = X.numpy()
    want = np.zeros((X.dims[0], X.dims[1]))
    np.add.at(want, (c[0], c[1]), v * v)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=0)
    with pytest.raises(cst.ConststnError) as e:
        cst.plan(text2, [("X", csf), ("W", csf)], options={"generic_densify": 0})
    assert e.value.status_name == "EUNSUPPORTED"
    with pytest.raises(cst.ConststnError) as e:      # loop order against the CSF layout
        cst.plan(S.TTMC3.replace("| i,j,k,s", "| j,i,k,s"), [("X", csf), ("U3", U3), ("U2", U2)])
    assert e.value.status_name == "ESCHED"
