"""GPU parity, solver: bit-exact choice against the oracle DP on identical tables, brute force on
tiny tables, infeasible budgets, the configs' table sizes."""
import numpy as np
import pytest

from oracle import solver

pytestmark = pytest.mark.gpu


def _handle(L, P, dp_groups=0, strict_budget=False):
    from paper_2210_17357_amd import binding as B
    return B.Handle(1024, L, P, dp_groups=dp_groups, strict_budget=strict_budget)


def _compare(h, errors, sizes, e_max, n_bins):
    from paper_2210_17357_amd import binding as B
    st, choice, tsize, terr = h.solve(errors, sizes, e_max, n_bins)
    ref_choice, ref_size, ref_err = solver.solve(errors, sizes, e_max, n_bins)
    if ref_choice is None:
        assert st == B.EINFEASIBLE
        assert np.array_equal(choice, np.argmin(errors, axis=1))
        return
    assert st == B.OK
    differ = np.flatnonzero(choice != ref_choice)
    assert differ.size == 0, ("route", h.last_solve_groups(), "layers", differ.tolist()[:16], "got",
                              choice[differ][:16].tolist(), "oracle", ref_choice[differ][:16].tolist(),
                              "size", tsize, ref_size)
    assert tsize == ref_size and terr == pytest.approx(ref_err, rel=1e-15)
    if h.late_handovers():
        print("result blocks that arrived after their sequence number so far on this handle:", h.late_handovers())


def test_random_small_tables_with_ties_and_unusable_candidates():
    rng = np.random.default_rng(0)
    h = _handle(8, 8)
    for trial in range(200):
        L, P, D = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 40))
        errors = rng.integers(0, 12, (L, P)).astype(np.float64) * 0.25
        if trial % 4 == 0:
            errors[:, 0] = 0.0
        sizes = rng.integers(0, 5, (L, P)).astype(np.int64)
        e_max = float(rng.integers(0, 20)) * 0.5
        _compare(h, errors, sizes, e_max, D)
    h.close()


def test_handles_created_one_after_another():
    """Each handle's first solves after an earlier handle was destroyed (its pinned result block
    may be handed to the new one with the old contents): the solver's hand-over to the host must
    not take anything left there for its own result."""
    rng = np.random.default_rng(11)
    for trial in range(6):
        L, P, D = 20 + trial, 6, 300
        h = _handle(L, P)
        for _ in range(1 + trial % 3):
            errors = np.sort(rng.random((L, P)), axis=1)[:, ::-1] * 10.0 ** rng.uniform(-4, -1, (L, 1))
            sizes = (rng.integers(1, 30, (L, 1)) * np.arange(1, P + 1) * 10).astype(np.int64)
            _compare(h, errors, sizes, solver.e_max_uniform(errors, 2), D)
        h.close()


@pytest.mark.parametrize("L,P,D", [(62, 7, 1000), (161, 6, 1000), (97, 5, 2000), (292, 13, 4000),
                                   (40, 32, 10000), (97, 49, 10000), (30, 9, 16384), (3, 4, 1023), (3, 4, 1024)])
def test_config_sized_tables(L, P, D):
    rng = np.random.default_rng(L * 1000 + P)
    h = _handle(L, P)
    base = 10.0 ** rng.uniform(-6, -1, (L, 1))
    errors = base * np.sort(rng.random((L, P)), axis=1)[:, ::-1] * np.logspace(0, -3, P)
    sizes = (rng.integers(1, 50, (L, 1)) * np.arange(1, P + 1) * 100).astype(np.int64)
    e_max = solver.e_max_uniform(errors, P // 2)
    _compare(h, errors, sizes, e_max, D)
    _compare(h, errors, sizes, e_max * 0.3, D)
    # large sizes (beyond 32 bits) and many exact ties
    _compare(h, errors, (sizes * 0 + (1 << 33)).astype(np.int64), e_max, D)
    h.close()


def test_invalid_arguments():
    from paper_2210_17357_amd import binding as B
    h = _handle(4, 4)
    errors = np.ones((2, 2))
    sizes = np.ones((2, 2), np.int64)
    for bad_bins in (0, -1, B.lib() and 16385):
        with pytest.raises(B.LgrecoError):
            h.solve(errors, sizes, 1.0, bad_bins)
    with pytest.raises(B.LgrecoError):
        h.solve(np.ones((5, 2)), np.ones((5, 2), np.int64), 1.0, 10)       # more layers than created for
    with pytest.raises(B.LgrecoError):
        h.solve(errors, -sizes, 1.0, 10)
    h.close()


def _compare_weighted(h, errors, sizes, weights, e_max, n_bins):
    from paper_2210_17357_amd import binding as B
    st, choice, tsize, tcost, terr = h.solve_weighted(errors, sizes, weights, e_max, n_bins)
    ref_choice, ref_size, ref_cost, ref_err = solver.solve_weighted(errors, sizes, weights, e_max, n_bins)
    if ref_choice is None:
        assert st == B.EINFEASIBLE
        return
    assert st == B.OK
    assert np.array_equal(choice, ref_choice)
    assert tsize == ref_size and tcost == ref_cost and terr == pytest.approx(ref_err, rel=1e-15)


def test_weighted_objective_small_tables_and_bucket_priorities():
    rng = np.random.default_rng(3)
    h = _handle(64, 8)
    for trial in range(150):
        L, P, D = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 40))
        errors = rng.integers(0, 12, (L, P)).astype(np.float64) * 0.25
        sizes = rng.integers(0, 5, (L, P)).astype(np.int64)
        weights = rng.integers(0, 4, L).astype(np.int64)
        _compare_weighted(h, errors, sizes, weights, float(rng.integers(0, 20)) * 0.5, D)
    # 62 layers in 8 communication buckets, coefficient = bucket index (appendix of the paper)
    L, P, D = 62, 7, 1000
    base = 10.0 ** rng.uniform(-6, -1, (L, 1))
    errors = base * np.sort(rng.random((L, P)), axis=1)[:, ::-1] * np.logspace(0, -3, P)
    sizes = (rng.integers(1, 50, (L, 1)) * np.arange(1, P + 1) * 100).astype(np.int64)
    e_max = solver.e_max_uniform(errors, 2)
    bucket = 1 + (np.arange(L)[::-1] * 8) // L
    _compare_weighted(h, errors, sizes, bucket.astype(np.int64), e_max, D)
    _compare_weighted(h, errors, sizes, np.ones(L, np.int64), e_max, D)
    from paper_2210_17357_amd import binding as B
    with pytest.raises(B.LgrecoError):
        h.solve_weighted(errors, sizes, -np.ones(L, np.int64), e_max, D)
    with pytest.raises(B.LgrecoError):
        h.solve_weighted(errors, sizes, np.full(L, 1 << 44, np.int64), e_max, D)     # product overflow
    h.close()


@pytest.mark.parametrize("groups", [2, 4, 8])
def test_layer_groups_give_the_sequential_result_ties_included(groups):
    """The layers swept in G groups side by side and the groups' tables joined pairwise must give
    Algorithm 1's assignment bit for bit.  Small integer tables are full of exact ties between
    different ways of sharing the bins among the groups: those solves must resolve them the way
    Algorithm 1 would (reported as 1000 + G, or -G if they give up and sweep sequentially), the
    others go straight through the groups (+G)."""
    rng = np.random.default_rng(100 + groups)
    h = _handle(64, 8, dp_groups=groups)
    modes = []
    for trial in range(150):
        L, P, D = int(rng.integers(1, 40)), int(rng.integers(1, 9)), int(rng.integers(1, 60))
        errors = rng.integers(0, 12, (L, P)).astype(np.float64) * 0.25
        if trial % 4 == 0:
            errors[:, 0] = 0.0
        sizes = rng.integers(0, 5, (L, P)).astype(np.int64)
        _compare(h, errors, sizes, float(rng.integers(0, 40)) * 0.5, D)
        modes.append(h.last_solve_groups())
    # tables without structure: real-valued errors, sizes spread over many values -> no ties expected
    for trial in range(30):
        L, P, D = int(rng.integers(20, 64)), int(rng.integers(3, 9)), int(rng.integers(200, 3000))
        base = 10.0 ** rng.uniform(-6, -1, (L, 1))
        errors = base * np.sort(rng.random((L, P)), axis=1)[:, ::-1] * np.logspace(0, -3, P)
        sizes = np.sort(rng.integers(1, 1 << 22, (L, P)), axis=1).astype(np.int64)
        _compare(h, errors, sizes, solver.e_max_uniform(errors, P // 2) * float(rng.uniform(0.3, 1.5)), D)
        modes.append(h.last_solve_groups())
    h.close()
    modes = np.array(modes)
    assert set(np.unique(modes)) <= {groups, 1000 + groups, -groups, 0}
    assert (modes[:150] == 1000 + groups).sum() > 5, "no ambiguous split met: the tie-breaks are not exercised"
    assert (modes[150:] == groups).sum() > 20, "the plain grouped route is hardly taken"
    print("modes:", {int(m): int((modes == m).sum()) for m in np.unique(modes)})


@pytest.mark.parametrize("L,P,D", [(292, 13, 4000), (161, 6, 10000), (97, 49, 10000), (1024, 4, 4090), (300, 9, 16384)])
def test_layer_groups_on_large_tables(L, P, D):
    rng = np.random.default_rng(L + P)
    base = 10.0 ** rng.uniform(-6, -1, (L, 1))
    errors = base * np.sort(rng.random((L, P)), axis=1)[:, ::-1] * np.logspace(0, -3, P)
    sizes = (rng.integers(1, 50, (L, 1)) * np.arange(1, P + 1) * 100).astype(np.int64)
    e_max = solver.e_max_uniform(errors, P // 2)
    seen = set()
    for groups in (0, 1, 2, 8):
        h = _handle(L, P, dp_groups=groups)
        _compare(h, errors, sizes, e_max, D)
        seen.add(h.last_solve_groups())
        _compare(h, errors, sizes, e_max * 0.3, D)
        # identical layers: wherever two layers differ in their candidate, swapping them ties
        same_e = np.tile(errors[:1], (L, 1))
        same_s = np.tile(sizes[:1], (L, 1))
        _compare(h, same_e, same_s, solver.e_max_uniform(same_e, P // 2), D)
        h.close()
    assert seen & {8, 1008, -8}


@pytest.mark.parametrize("groups", [1, 8])
def test_strict_budget_keeps_the_real_errors_within_e_max(groups):
    """strict_budget: only assignments whose bins sum to at most n_bins - L are accepted (the
    oracle's strict solve, pinned by enumeration), so the real errors never exceed E_max; the
    plain solve on the same tables overshoots in a good share of them."""
    from paper_2210_17357_amd import binding as B
    rng = np.random.default_rng(77 + groups)
    plain, strict = _handle(300, 13, dp_groups=groups), _handle(300, 13, dp_groups=groups, strict_budget=True)
    over = infeasible = 0
    for trial in range(60):
        if trial % 3 == 0:
            L, P, D = int(rng.integers(60, 300)), int(rng.integers(3, 13)), int(rng.integers(500, 4000))
        else:
            L, P, D = int(rng.integers(1, 40)), int(rng.integers(1, 9)), int(rng.integers(1, 80))
        errors = np.sort(rng.random((L, P)), axis=1)[:, ::-1] * 10.0 ** rng.uniform(-3, 0, (L, 1))
        sizes = np.sort(rng.integers(1, 1 << 20, (L, P)), axis=1).astype(np.int64)
        e_max = solver.e_max_uniform(errors, P // 2)
        st, choice, tsize, terr = plain.solve(errors, sizes, e_max, D)
        assert st == B.OK
        over += terr > e_max
        ref_choice, ref_size, ref_err = solver.solve(errors, sizes, e_max, D, strict=True)
        st, choice, tsize, terr = strict.solve(errors, sizes, e_max, D)
        if ref_choice is None:
            assert st == B.EINFEASIBLE
            infeasible += 1
            continue
        assert st == B.OK and np.array_equal(choice, ref_choice) and tsize == ref_size
        assert terr <= e_max
        assert int(solver.discretise(errors, e_max, D)[np.arange(L), choice].sum()) <= D - L
    assert over > 10 and infeasible > 0, (over, infeasible)
    plain.close()
    strict.close()
