"""Three-tensor network Z[i,m] = U[i,j,k] V[j,l] W[k,l,m] (Sec. 1) on the GPU against the oracle:
the tiled matrix-core kernel over block-sparse and scattered inputs, its limits, and the baseline
kernel it falls back to."""

import numpy as np
import pytest
import torch

import workloads as w
from workloads.generators import make_sptn3_scattered
from helpers import TOL, compare, run_gpu, run_oracle
import paper_2401_04836_amd as cst

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _check(wl, label, flags=0, expect=None, options=None):
    """Runs the kernel the options choose (sptn3_tiled=2: the tiled kernel whatever the fill of W's tiles)
    and, where that is the tiled kernel with two wavefronts per SIMD, also the form with one; both
    against the oracle."""
    options = dict(options or {})
    out = _check_one(wl, label, flags, expect, options=options)
    _check_one(wl, label + " (one wavefront per SIMD)", flags,
               expect.replace("two waves", "one wave") if expect else None, "two waves",
               options=dict(options, sptn3_waves=1))
    return out


def _check_one(wl, label, flags=0, expect=None, absent=None, options=None):
    _say("sptn3 %s: dims %s" % (label, wl.params["dims"]))
    out, pl, _ = run_gpu(wl, flags=flags, options=options)
    want, S_abs = run_oracle(wl)
    rows = pl.output_rows() if flags & cst.OUT_COMPACT else None
    err = compare(out, want, S_abs, rows)
    desc = pl.describe()
    _say("  %s -> rel err %.3e" % (desc.split("|")[0], err))
    if expect is not None:
        assert expect in desc, desc
    if absent is not None:
        assert absent not in desc, desc
    assert err <= TOL
    return out


def test_block_sparse_small_tiled_and_baseline_agree_with_oracle():
    wl = w.make(4, small=True)
    a = _check(wl, "block-sparse reduced copy, tiled", expect="tiled two waves")
    b = _check(wl, "block-sparse reduced copy, baseline kernel", expect="baseline", options={"sptn3_tiled": 0})
    assert a.shape == b.shape


def test_single_k_chunk_writes_output_directly():
    wl = w.make(4, small=True)
    _check(wl, "one chunk of the k range", expect="k chunks 1", options={"sptn3_wgs": 1})


def test_scattered_union_longer_than_one_pass():
    # ~27 leaves per (i,k) fiber, 16 slices per group: unions of ~400 > 320 rows -> several passes
    wl = make_sptn3_scattered("sc1", 9101, (50, 700, 30, 100, 70), 40000, 30000)
    _check(wl, "scattered, multi-pass unions", expect="tiled", options={"sptn3_tiled": 2})


def test_scattered_sparse_w_and_ragged_extents():
    # L and M not multiples of 16, fewer than 16 slices in the last group, k values missing in W
    wl = make_sptn3_scattered("sc2", 9102, (37, 90, 23, 45, 19), 9000, 700)
    _check(wl, "scattered, ragged", expect="tiled", options={"sptn3_tiled": 2})
    _check(wl, "scattered, ragged, compact rows", flags=cst.OUT_COMPACT, options={"sptn3_tiled": 2})


def test_many_l_tiles_per_wavefront():
    # L > 4096: a wavefront owns more than 64 tiles of l and works in rounds
    wl = make_sptn3_scattered("sc3", 9103, (20, 40, 6, 4200, 33), 3000, 60000)
    _check(wl, "L = 4200", expect="tiled", options={"sptn3_tiled": 2})


def test_more_w_tiles_than_parked():
    # dense W rows: up to 25 m tiles below one l tile, short unions (one batch per l tile)
    wl = make_sptn3_scattered("sc4", 9104, (18, 30, 5, 40, 400), 1500, 60000)
    _check(wl, "M = 400, many m tiles per l tile", expect="tiled", options={"sptn3_tiled": 2})


def test_m_beyond_tiled_limit_uses_baseline():
    wl = make_sptn3_scattered("sc5", 9105, (18, 30, 5, 40, 401), 1500, 20000)
    _check(wl, "M = 401", expect="baseline")


def test_wide_j_extent_falls_back_to_one_wavefront_per_simd():
    # the bit mask over j of the two-wavefront form no longer fits its LDS beyond J of about 27 000
    wl = make_sptn3_scattered("sc7", 9107, (20, 30000, 6, 40, 33), 3000, 700)
    _check_one(wl, "J = 30000", expect="tiled one wave", absent="two waves", options={"sptn3_tiled": 2})


def test_scattered_w_takes_the_baseline_kernel_unless_told_otherwise():
    # about one nonzero per 16 x 16 tile of W: dense tiles would inflate it 256-fold
    wl = make_sptn3_scattered("sc2", 9102, (37, 90, 23, 45, 19), 9000, 700)
    _check_one(wl, "scattered W, default choice", expect="baseline")


def test_tiled_is_deterministic():
    wl = w.make(4, small=True)
    a, _, _ = run_gpu(wl)
    b, _, _ = run_gpu(wl)
    assert torch.equal(a, b)


def test_empty_slices_and_empty_w_roots():
    # U uses only a few i and k; W misses most k: rows without terms must be exact zeros
    wl = make_sptn3_scattered("sc6", 9106, (64, 50, 40, 30, 20), 300, 200)
    out = _check(wl, "very sparse", options={"sptn3_tiled": 2})
    want, S_abs = run_oracle(wl)
    assert not out.cpu().numpy()[S_abs == 0].any()
