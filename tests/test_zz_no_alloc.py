"""lgreco_solve_static (the entry point that allocates nothing) against lgreco_emax + lgreco_solve on
the same tables: assignment and total size bit-exact, E_max and total error bit for bit.  Two calls
in a row share the library's static scratch, the second with a smaller problem; limits beyond the
scratch are refused."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _tables(rng, L, P):
    base = 10.0 ** rng.uniform(-6, -1, (L, 1))
    errors = base * np.sort(rng.random((L, P)), axis=1)[:, ::-1] * np.logspace(0, -3, P)
    sizes = (rng.integers(1, 50, (L, 1)) * np.arange(1, P + 1) * 100).astype(np.int64)
    return np.ascontiguousarray(errors), sizes


def _run_static(errors, sizes, default, n_bins):
    import torch
    from paper_2210_17357_amd import binding as B
    L, P = errors.shape
    d_err = torch.from_numpy(errors).cuda()
    d_sz = torch.from_numpy(sizes).cuda()
    d_choice = torch.full((L,), -7, dtype=torch.int32, device="cuda")
    d_res = torch.full((4,), -7, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st = B.solve_static(d_err, d_sz, default, n_bins, d_choice, d_res)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert st == B.OK, st
    res = d_res.cpu().numpy()
    return d_choice.cpu().numpy(), int(res[0]), int(res[1]), res[2:3].view(np.float64)[0], res[3:4].view(np.float64)[0]


def _compare(h, errors, sizes, default, n_bins, scale=1.0):
    from paper_2210_17357_amd import binding as B
    e_max = B.emax(errors, default)
    choice, status, tsize, terr, emax_dev = _run_static(errors, sizes, default, n_bins)
    assert emax_dev == e_max
    st, ref_choice, ref_size, ref_err = h.solve(errors, sizes, e_max, n_bins)
    if st == B.EINFEASIBLE:
        assert status == 1
    else:
        assert st == B.OK and status == 0
        assert tsize == ref_size and terr == ref_err
    assert np.array_equal(choice, ref_choice)


def test_two_calls_in_a_row_second_one_smaller():
    from paper_2210_17357_amd import binding as B
    rng = np.random.default_rng(2)
    h = B.Handle(1024, 512, 16)
    e1, s1 = _tables(rng, 292, 13)
    e2, s2 = _tables(rng, 41, 7)          # odd table size: the last entry is read on its own
    _compare(h, e1, s1, 2, 4000)
    _compare(h, e2, s2, 3, 1000)          # smaller, on the scratch the first call left
    _compare(h, e1, s1, 2, 4000)
    # ties, zero-error candidates (layers the list building fixes), unusable candidates
    for trial in range(40):
        L, P, D = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 40))
        errors = rng.integers(0, 12, (L, P)).astype(np.float64) * 0.25
        if trial % 4 == 0:
            errors[:, 0] = 0.0
        sizes = rng.integers(0, 5, (L, P)).astype(np.int64)
        _compare(h, errors, sizes, int(rng.integers(0, P)), D)
    # a budget nothing fits: a negative default error makes E_max negative, the second layer then
    # has no usable candidate
    e3 = np.array([[-1.0, 2.0], [0.5, 0.25]])
    _compare(h, e3, np.ones((2, 2), np.int64), 0, 10)
    h.close()


def test_paper_default_bins_and_limits():
    import torch
    from paper_2210_17357_amd import binding as B
    rng = np.random.default_rng(5)
    h = B.Handle(1024, 512, 16)
    e1, s1 = _tables(rng, 292, 13)
    _compare(h, e1, s1, 6, 10000)         # the paper's D, 2.9 MB of arg-min table
    h.close()
    d_choice = torch.zeros(1024, dtype=torch.int32, device="cuda")
    d_res = torch.zeros(4, dtype=torch.int64, device="cuda")

    def status(L, P, D):
        return B.solve_static(torch.zeros((L, P), dtype=torch.float64, device="cuda"),
                              torch.zeros((L, P), dtype=torch.int64, device="cuda"), 0, D, d_choice, d_res)
    assert status(1025, 2, 100) == B.ENOSPACE
    assert status(300, 17, 100) == B.ENOSPACE
    assert status(1024, 8, 100) == B.ENOSPACE              # 8192 table entries
    assert status(1024, 4, 4096) == B.ENOSPACE             # arg-min table beyond the scratch
    assert status(1024, 4, 4090) == B.OK
    assert status(4, 4, 16385) == B.ENOSPACE
    assert status(4, 4, 0) == B.EINVAL
    torch.cuda.synchronize()
    # sizes the 32-bit costs of this path cannot hold: reported, nothing chosen
    big = np.full((3, 2), 1 << 31, np.int64)
    choice, st, *_ = _run_static(np.ones((3, 2)), big, 0, 10)
    assert st == 3 and (choice == -1).all()
    choice, st, *_ = _run_static(np.array([[1.0, np.nan], [1.0, 1.0]]), np.ones((2, 2), np.int64), 0, 10)
    assert st == 3 and (choice == -1).all()
