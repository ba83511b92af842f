"""Pins for the DP oracle: brute-force enumeration of every assignment (with the tie-break
tuple), feasibility, never worse than the uniform default, monotone in the budget, and the
first workload's 7^4 enumeration."""
import itertools

import numpy as np
import pytest

from oracle import pipeline, solver
from paper_2210_17357_amd import workloads as W


def brute_force(bins, sizes, n_bins, e_limit=None):
    """Among assignments with sum(bin) <= D (<= e_limit if given) minimise (sum size, sum bin, c_L, ..., c_1)."""
    n_layers, n_cands = bins.shape
    best_key, best = None, None
    for assign in itertools.product(range(n_cands), repeat=n_layers):
        b = [int(bins[l][c]) for l, c in enumerate(assign)]
        if any(v < 0 or v > n_bins for v in b) or sum(b) > (n_bins if e_limit is None else e_limit):
            continue
        key = (sum(int(sizes[l][c]) for l, c in enumerate(assign)), sum(b)) + tuple(reversed(assign))
        if best_key is None or key < best_key:
            best_key, best = key, assign
    return None if best is None else np.array(best, np.int32)


def test_brute_force_random_tables_with_ties():
    rng = np.random.default_rng(0)
    for trial in range(300):
        n_layers = int(rng.integers(1, 6))
        n_cands = int(rng.integers(1, 6))
        n_bins = int(rng.integers(1, 31))
        bins = rng.integers(-1, n_bins + 3, (n_layers, n_cands)).astype(np.int64)
        bins[bins > n_bins] = solver.UNUSABLE if trial % 2 else n_bins + 5
        if trial % 3 == 0:
            bins[:, 0] = 0                                   # zero-error candidates
        sizes = rng.integers(0, 6, (n_layers, n_cands)).astype(np.int64)   # few values -> many ties
        expect = brute_force(bins, sizes, n_bins)
        for fast in (False, True):
            dp, pd = (solver.dp_tables_fast if fast else solver.dp_tables)(bins, sizes, n_bins)
            got = solver.backtrace(dp, pd, bins)
            if expect is None:
                assert got is None
            else:
                assert got is not None and list(got) == list(expect), (trial, fast)


def test_discretise_rules():
    e = np.array([[0.0, 0.5, 1.0, 1.0001, -1e-9, 2.0]])
    b = solver.discretise(e, 1.0, 10)
    assert list(b[0]) == [0, 5, 10, 10, 0, solver.UNUSABLE]
    assert list(solver.discretise(np.array([[0.0, 1e-30]]), 0.0, 10)[0]) == [0, solver.UNUSABLE]
    # floor: the default's own bins never exceed D in total
    rng = np.random.default_rng(1)
    errs = rng.random((50, 3))
    emax = solver.e_max_uniform(errs, 1)
    assert solver.discretise(errs, emax, 1000)[:, 1].sum() <= 1000


def test_first_workload_against_7_pow_4_enumeration():
    w = W.workload("c0_tiny_quant")
    b = W.generate(w)
    res = pipeline.run(b.grads, b.ef, b.offsets, b.numels, b.rows, b.cols, w.candidates, w.default,
                       w.n_bins, bucket=w.bucket)
    bins = solver.discretise(res["errors"], res["e_max"], w.n_bins)
    expect = brute_force(bins, res["sizes"], w.n_bins)
    assert list(res["choice"]) == list(expect)
    uniform = int(res["sizes"][:, w.default].sum())
    assert res["total_size"] <= uniform
    assert bins[np.arange(4), res["choice"]].sum() <= w.n_bins
    # floor discretisation: the real error may exceed the budget by less than L steps
    assert res["total_error"] <= res["e_max"] * (1 + len(b.numels) / w.n_bins)


def test_never_worse_than_default_and_monotone_in_budget():
    rng = np.random.default_rng(2)
    n_layers, n_cands = 12, 5
    errors = np.sort(rng.random((n_layers, n_cands)), axis=1)[:, ::-1].copy()     # error falls with c
    sizes = np.sort(rng.integers(10, 1000, (n_layers, n_cands)), axis=1).astype(np.int64)
    e_max = solver.e_max_uniform(errors, 2)
    prev = None
    for scale in (0.5, 0.75, 1.0, 1.5, 3.0):
        choice, tsize, terr = solver.solve(errors, sizes, e_max * scale, 400)
        if choice is None:
            continue
        if scale >= 1.0:
            assert tsize <= int((sizes[:, 2]).sum())
        if prev is not None:
            assert tsize <= prev
        prev = tsize
    # any discretisation keeps the default feasible
    coarse = solver.solve(errors, sizes, e_max, 20)[1]
    fine = solver.solve(errors, sizes, e_max, 5000)[1]
    assert fine <= int(sizes[:, 2].sum()) and coarse <= int(sizes[:, 2].sum())


def test_infeasible_returns_none():
    errors = np.array([[2.0, 3.0], [2.0, 3.0]])
    sizes = np.array([[1, 1], [1, 1]], np.int64)
    assert solver.solve(errors, sizes, 1.0, 10)[0] is None


def test_listing_initialisation_is_a_special_case():
    # when layer-1 bins are distinct and <= D the virtual start row reproduces the listing's
    # direct initialisation DP[1][bin] = cost, PD[1][bin] = c
    bins = np.array([[3, 1, 0], [2, 1, 0]], np.int64)
    sizes = np.array([[5, 7, 9], [1, 2, 3]], np.int64)
    dp, pd = solver.dp_tables(bins, sizes, 6)
    for c in range(3):
        assert dp[1][bins[0][c]] == sizes[0][c] and pd[1][bins[0][c]] == c
    assert np.sum(dp[1] < solver.INF) == 3


def test_dominated_candidates_never_lie_on_the_traced_path():
    """A property the GPU solver's host step relies on: a candidate that another candidate of the
    same layer beats in bin (strictly) and in size (not larger) can be removed without changing
    the assignment, tie-breaks included.  Checked on the oracle alone, on tables full of ties."""
    rng = np.random.default_rng(5)
    removed = 0
    for trial in range(400):
        n_layers = int(rng.integers(1, 7))
        n_cands = int(rng.integers(2, 7))
        n_bins = int(rng.integers(1, 41))
        bins = rng.integers(-1, n_bins + 2, (n_layers, n_cands)).astype(np.int64)
        bins[bins > n_bins] = solver.UNUSABLE
        sizes = rng.integers(0, 5, (n_layers, n_cands)).astype(np.int64)
        pruned = bins.copy()
        for l in range(n_layers):
            for c in range(n_cands):
                if bins[l, c] == solver.UNUSABLE:
                    continue
                for o in range(n_cands):
                    if bins[l, o] != solver.UNUSABLE and bins[l, o] < bins[l, c] and sizes[l, o] <= sizes[l, c]:
                        pruned[l, c] = solver.UNUSABLE
                        removed += 1
                        break
        dp, pd = solver.dp_tables(bins, sizes, n_bins)
        full = solver.backtrace(dp, pd, bins)
        dp2, pd2 = solver.dp_tables(pruned, sizes, n_bins)
        cut = solver.backtrace(dp2, pd2, pruned)
        assert (full is None) == (cut is None)
        if full is not None:
            assert list(full) == list(cut), trial
    assert removed > 500


def brute_force_weighted(bins, sizes, weights, n_bins):
    """Among assignments with sum(bin) <= D minimise (sum size*T, sum bin, c_L, ..., c_1)."""
    n_layers, n_cands = bins.shape
    best_key, best = None, None
    for assign in itertools.product(range(n_cands), repeat=n_layers):
        b = [int(bins[l][c]) for l, c in enumerate(assign)]
        if any(v < 0 or v > n_bins for v in b) or sum(b) > n_bins:
            continue
        key = (sum(int(sizes[l][c]) * int(weights[l]) for l, c in enumerate(assign)), sum(b)) \
            + tuple(reversed(assign))
        if best_key is None or key < best_key:
            best_key, best = key, assign
    return None if best is None else np.array(best, np.int32)


def test_weighted_objective_against_enumeration():
    """Section "Time optimization": the objective sum size * T(l).  Brute force over all
    assignments on tiny tables, weights including 0 and repeated values."""
    rng = np.random.default_rng(11)
    for trial in range(200):
        n_layers = int(rng.integers(1, 6))
        n_cands = int(rng.integers(1, 5))
        n_bins = int(rng.integers(1, 25))
        errors = rng.integers(0, n_bins + 3, (n_layers, n_cands)).astype(np.float64)
        sizes = rng.integers(0, 6, (n_layers, n_cands)).astype(np.int64)
        weights = rng.integers(0, 4, n_layers).astype(np.int64)
        e_max = float(n_bins)                       # bin = floor(error)
        bins = solver.discretise(errors, e_max, n_bins)
        expect = brute_force_weighted(bins, sizes, weights, n_bins)
        for fast in (False, True):
            got, tsize, tcost, terr = solver.solve_weighted(errors, sizes, weights, e_max, n_bins, fast=fast)
            if expect is None:
                assert got is None
            else:
                assert list(got) == list(expect), trial
                rows = np.arange(n_layers)
                assert tsize == int(sizes[rows, got].sum())
                assert tcost == int((sizes[rows, got] * weights).sum())


def test_weighted_objective_special_cases():
    w = W.workload("c0_tiny_quant")
    batch = W.generate(w)
    cands = list(w.candidates)
    errors = pipeline.profile(batch.grads, batch.ef, batch.offsets, batch.numels, batch.rows, batch.cols, cands)
    sizes = pipeline.sizes_table(batch.numels, batch.rows, batch.cols, cands)
    e_max = solver.e_max_uniform(errors, w.default)
    plain, psize, _ = solver.solve(errors, sizes, e_max, w.n_bins)
    L = len(batch.numels)
    # equal coefficients: the objective is a multiple of the plain one, same assignment
    for c in (1, 7):
        got, tsize, tcost, _ = solver.solve_weighted(errors, sizes, np.full(L, c), e_max, w.n_bins)
        assert list(got) == list(plain) and tsize == psize and tcost == c * psize
    # appendix "Buckets prioritization": T = index of the bucket the layer travels in.  The
    # layers with the larger coefficient end up with sizes no larger than before, in total
    bucket = np.array([1, 1, 2, 2])
    got, tsize, tcost, terr = solver.solve_weighted(errors, sizes, bucket, e_max, w.n_bins)
    rows = np.arange(L)
    assert tcost <= int((sizes[rows, plain] * bucket).sum())       # optimal for ITS objective
    assert tsize >= psize                                          # and no better in plain bytes
    assert sizes[rows, got][bucket == 2].sum() <= sizes[rows, plain][bucket == 2].sum()
    assert terr <= e_max * (1.0 + L / w.n_bins)


def test_strict_budget_against_enumeration_and_its_guarantee():
    """strict: only assignments with sum(bin) <= D - L are accepted (every bin rounds its error
    down by less than one step, so the real errors then sum to less than E_max).  Enumeration with
    that limit and the same tie-break tuple; the guarantee itself on real-valued tables, where the
    plain solve overshoots E_max in a good share of the cases."""
    rng = np.random.default_rng(5)
    for trial in range(200):
        n_layers, n_cands = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        n_bins = int(rng.integers(1, 31))
        bins = rng.integers(-1, n_bins + 3, (n_layers, n_cands)).astype(np.int64)
        bins[bins > n_bins] = solver.UNUSABLE
        if trial % 3 == 0:
            bins[:, 0] = 0
        sizes = rng.integers(0, 6, (n_layers, n_cands)).astype(np.int64)
        limit = solver.strict_limit(n_layers, n_bins)
        assert limit == n_bins - n_layers
        expect = brute_force(bins, sizes, n_bins, e_limit=limit) if limit >= 0 else None
        for fast in (False, True):
            dp, pd = (solver.dp_tables_fast if fast else solver.dp_tables)(bins, sizes, n_bins)
            got = solver.backtrace(dp, pd, bins, limit)
            assert (got is None) == (expect is None), (trial, fast)
            if expect is not None:
                assert list(got) == list(expect), (trial, fast)
    over = 0
    for trial in range(200):
        n_layers, n_cands, n_bins = int(rng.integers(2, 30)), int(rng.integers(2, 8)), int(rng.integers(40, 400))
        errors = np.sort(rng.random((n_layers, n_cands)), axis=1)[:, ::-1] * 10.0 ** rng.uniform(-3, 0, (n_layers, 1))
        sizes = np.sort(rng.integers(1, 1000, (n_layers, n_cands)), axis=1).astype(np.int64)
        e_max = solver.e_max_uniform(errors, n_cands // 2)
        _, _, plain_err = solver.solve(errors, sizes, e_max, n_bins)
        over += plain_err > e_max
        choice, _, terr = solver.solve(errors, sizes, e_max, n_bins, strict=True)
        if choice is not None:
            assert terr <= e_max
    assert over > 20, "the plain solve hardly ever overshoots here: the case shows nothing"
