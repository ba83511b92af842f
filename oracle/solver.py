"""Oracle: the layer x discretised-error dynamic program (Algorithm 1 of the paper).

Problem (section "The Constrained Optimization Problem"): choose one candidate c_l per
layer minimising sum size(l, c_l) subject to sum error(l, c_l) <= E_max.  Errors are
discretised with step E_max / D (section "The L-GreCo Framework", Overview) and the
knapsack-style table DP[l][e] = min total size of the first l layers whose binned errors
sum to exactly e is filled layer by layer; PD keeps the arg-min candidate for the
back-trace (Algorithm 1).

Readings where the paper's listing is silent or breaks:
  * bin(l,c) = floor((error * D) / E_max) in fp64, in that operation order; negative errors
    count as 0; a bin above D makes the candidate unusable for that layer.  With floor the
    uniform default always stays feasible.  If E_max <= 0 only zero-error candidates are usable
    (bin 0).
  * The first layer is treated like every other one, starting from a virtual row
    DP[0][0] = 0, DP[0][e > 0] = inf.  This equals the listing's initialisation when the first
    layer's bins are distinct and <= D, and also covers two candidates in one bin (keep the
    smaller) and bins > D (skip).
  * Strict '<' with candidates visited in ascending index: the lowest candidate index wins a
    tie.  The final arg-min takes the lowest e among equal minima.
Sizes are integers (bytes), so there are no floating-point ties.
"""
import math

import numpy as np

INF = np.iinfo(np.int64).max // 4
UNUSABLE = -1


def discretise(errors: np.ndarray, e_max: float, n_bins: int) -> np.ndarray:
    """int64 [L x P] bins; UNUSABLE where the candidate cannot be taken."""
    errors = np.asarray(errors, np.float64)
    bins = np.empty(errors.shape, np.int64)
    for idx, err in np.ndenumerate(errors):
        err = max(float(err), 0.0)
        if e_max > 0.0:
            b = math.floor((err * float(n_bins)) / float(e_max))
            bins[idx] = b if b <= n_bins else UNUSABLE
        else:
            bins[idx] = 0 if err <= 0.0 else UNUSABLE
    return bins


def dp_tables(bins: np.ndarray, sizes: np.ndarray, n_bins: int):
    """DP and PD from the recurrence the table is defined by (section "The L-GreCo Framework";
    Algorithm 1 fills the same table): with the virtual start row DP[0] = (0, inf, inf, ...),

        DP[l][e] = min over usable candidates c of layer l with bin(l, c) <= e
                   of DP[l-1][e - bin(l, c)] + size(l, c),
        PD[l][e] = the lowest such c that attains the minimum (-1 where no c applies).

    Every cell is evaluated on its own, straight from this definition."""
    n_layers, n_cands = bins.shape
    dp = np.full((n_layers + 1, n_bins + 1), INF, np.int64)
    pd = np.full((n_layers + 1, n_bins + 1), -1, np.int64)
    dp[0][0] = 0
    for l in range(1, n_layers + 1):
        usable = [(c, int(bins[l - 1][c]), int(sizes[l - 1][c])) for c in range(n_cands)
                  if bins[l - 1][c] != UNUSABLE and bins[l - 1][c] <= n_bins]
        for e in range(n_bins + 1):
            reach = [(int(dp[l - 1][e - b]) + cost, c) for c, b, cost in usable
                     if b <= e and dp[l - 1][e - b] < INF]
            if reach:
                dp[l][e], pd[l][e] = min(reach)        # smallest total, then lowest candidate index
    return dp, pd


def dp_tables_fast(bins: np.ndarray, sizes: np.ndarray, n_bins: int):
    """Same recurrence, one row at a time as a (min, +) step: candidate c contributes the previous
    row shifted right by bin(l, c) plus size(l, c); the new row is the element-wise minimum of
    the contributions and PD the first (lowest c) contribution attaining it.  Used where the
    cell-by-cell form would take minutes."""
    n_layers, n_cands = bins.shape
    dp = np.full((n_layers + 1, n_bins + 1), INF, np.int64)
    pd = np.full((n_layers + 1, n_bins + 1), -1, np.int64)
    dp[0][0] = 0
    for l in range(1, n_layers + 1):
        contrib = np.full((n_cands, n_bins + 1), INF, np.int64)
        for c in range(n_cands):
            b = int(bins[l - 1][c])
            if b == UNUSABLE or b > n_bins:
                continue
            prev = dp[l - 1][:n_bins + 1 - b]
            contrib[c][b:] = np.where(prev >= INF, INF, prev + np.int64(sizes[l - 1][c]))
        dp[l] = contrib.min(axis=0)
        first = contrib.argmin(axis=0)                 # numpy argmin: the first minimum along c
        pd[l] = np.where(dp[l] < INF, first, -1)
    return dp, pd


def backtrace(dp: np.ndarray, pd: np.ndarray, bins: np.ndarray, e_limit=None):
    """Algorithm 1, reconstruction: lowest e among the minima of the last row, then walk back.
    With e_limit only the cells 0..e_limit of the last row are looked at (see solve, strict).
    Returns None if no assignment fits."""
    n_layers = bins.shape[0]
    last = dp[n_layers] if e_limit is None else dp[n_layers][:max(e_limit + 1, 0)]
    if last.size == 0:
        return None
    best = int(last.min())
    if best >= INF:
        return None
    e = int(np.argmin(last))                       # numpy argmin: first (lowest e) minimum
    choice = np.zeros(n_layers, np.int32)
    for l in range(n_layers, 0, -1):
        c = int(pd[l][e])
        choice[l - 1] = c
        e -= int(bins[l - 1][c])
    assert e == 0
    return choice


def strict_limit(n_layers: int, n_bins: int) -> int:
    """Largest bin sum that guarantees sum error <= E_max: every bin rounds its error down by less
    than one step E_max / D, so sum error < (sum bin + L) * E_max / D, which is at most E_max when
    sum bin <= D - L (section "The Constrained Optimization Problem" asks for sum error <= E_max;
    the discretised constraint sum bin <= D alone allows an overshoot of up to L steps)."""
    return n_bins - n_layers


def solve(errors: np.ndarray, sizes: np.ndarray, e_max: float, n_bins: int, fast: bool = True, strict: bool = False):
    """Returns (choice int32[L] or None, total_size, total_error).  strict: accept only
    assignments whose bins sum to at most strict_limit, so that the real errors stay within E_max."""
    errors = np.asarray(errors, np.float64)
    sizes = np.asarray(sizes, np.int64)
    bins = discretise(errors, e_max, n_bins)
    dp, pd = (dp_tables_fast if fast else dp_tables)(bins, sizes, n_bins)
    choice = backtrace(dp, pd, bins, strict_limit(errors.shape[0], n_bins) if strict else None)
    if choice is None:
        return None, None, None
    rows = np.arange(errors.shape[0])
    return choice, int(sizes[rows, choice].sum()), float(np.sum(errors[rows, choice]))


def solve_weighted(errors: np.ndarray, sizes: np.ndarray, weights: np.ndarray, e_max: float, n_bins: int,
                   fast: bool = True):
    """Time-based objective (section "Time optimization"; appendix "Buckets prioritization"):
    minimise sum_l size(l, c_l) * T(l) under the same error constraint.  T(l) are non-negative
    integers here (the paper's regression coefficients, scaled by the caller; a bucket index in
    the appendix), so the table stays exact.  Algorithm 1 runs unchanged on the weighted costs.
    Returns (choice or None, total_size (unweighted bytes), total_cost, total_error)."""
    errors = np.asarray(errors, np.float64)
    sizes = np.asarray(sizes, np.int64)
    weights = np.asarray(weights, np.int64)
    assert weights.shape == (errors.shape[0],) and (weights >= 0).all()
    cost = sizes * weights[:, None]
    bins = discretise(errors, e_max, n_bins)
    dp, pd = (dp_tables_fast if fast else dp_tables)(bins, cost, n_bins)
    choice = backtrace(dp, pd, bins)
    if choice is None:
        return None, None, None, None
    rows = np.arange(errors.shape[0])
    return (choice, int(sizes[rows, choice].sum()), int(cost[rows, choice].sum()),
            float(np.sum(errors[rows, choice])))


def e_max_uniform(errors: np.ndarray, default: int) -> float:
    """Error budget: total error of the uniform default setting, summed in layer order
    (Algorithm 1, second step; section "The Error Bound")."""
    total = 0.0
    for l in range(errors.shape[0]):
        total += float(errors[l][default])
    return total
