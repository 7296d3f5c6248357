"""Pins for the oracle's reshape search (paper Sec. 3.2: Eq. 8 with both alphas 0, Algorithm 1).

The cost of a reshape is pinned against a construction that shares nothing with the oracle's CSR code
(numpy reshape / nonzero for D, scipy for the entropy), against a closed form for K = 1, and on a
tensor with a planted column structure.  The search is pinned by re-walking the algorithm's rules over
those independent costs, and by the properties the domain restrictions imply.
"""
import math

import numpy as np
import pytest
from scipy.stats import entropy


def _D_numpy(xhat, rows, cols):
    m = xhat.reshape(rows, cols)
    ri, ci = np.nonzero(m)                     # row-major order
    v = m[ri, ci].astype(np.int64)
    r = np.count_nonzero(m, axis=1).astype(np.int64)
    return np.concatenate([v, ci.astype(np.int64), r])


def _cost_numpy(xhat, rows):
    cols = xhat.size // rows
    D = _D_numpy(xhat, rows, cols)
    cnt = np.bincount(D)
    return D.size * entropy(cnt[cnt > 0], base=2), D.size


def _divisors_desc(T):
    return [n for n in range(T, 0, -1) if T % n == 0]


def _n_min(T, Q):
    return max(math.isqrt(T) + 1, -(-T // (1 << Q)))


def _sparse(n, seed, density=0.4, levels=256):
    rng = np.random.default_rng(seed)
    x = rng.integers(1, levels, n) * (rng.random(n) < density)
    return x.astype(np.uint8)


@pytest.mark.parametrize("T,Q,seed", [(360, 8, 0), (1024, 8, 1), (2310, 6, 2), (4096, 4, 3), (5040, 8, 4), (997, 8, 5)])
def test_cost_matches_an_independent_construction(oracle, T, Q, seed):
    x = _sparse(T, seed, levels=1 << Q)
    for N in _divisors_desc(T):
        if N < _n_min(T, Q):
            break
        got, len_d = oracle.reshape_cost(x, N, Q)
        want, want_len = _cost_numpy(x, N)
        assert len_d == want_len == 2 * np.count_nonzero(x) + N
        assert got == pytest.approx(want, rel=1e-12, abs=1e-9)


def test_k1_closed_form(oracle):
    # N = T, K = 1: c is all zeros, r is the zero mask, so the histogram is known without any CSR code
    T, Q = 6000, 8
    x = _sparse(T, 11)
    nnz = int(np.count_nonzero(x))
    cnt = np.bincount(x[x != 0], minlength=256).astype(np.int64)   # v
    cnt[0] += nnz + (T - nnz)                                       # c entries, and rows without a nonzero
    cnt[1] += nnz                                                   # rows with their one nonzero
    length = 2 * nnz + T
    want = length * math.log2(length) - sum(int(c) * math.log2(int(c)) for c in cnt if c)
    got, len_d = oracle.reshape_cost(x, T, Q)
    assert len_d == length
    assert got == pytest.approx(want, rel=1e-12)


def test_planted_column_structure_is_cheapest_at_its_period(oracle):
    # nonzeros only in column 0 of the 8-column view, one per row, all of the same value: for K = 8 every
    # column index is 0 and every row count is 1; for smaller K the column index or the row count varies
    T, Q, K = 8 * 4096, 8, 8
    x = np.zeros(T, np.uint8)
    x[::K] = 7
    costs = {k: oracle.reshape_cost(x, T // k, Q)[0] for k in (1, 2, 4, 8, 16)}
    assert costs[8] < min(costs[1], costs[2], costs[4])
    n_best, best, cands = oracle.search_reshape(x, Q)
    assert T // n_best in (8, 16, 32, 64, 128, 256)   # the walk goes on while the cost keeps falling
    assert best == pytest.approx(min(c for _, c in cands))


@pytest.mark.parametrize("T,Q,seed,density", [(360, 8, 0, 0.4), (4096, 8, 1, 0.3), (4096, 3, 2, 0.6), (5040, 8, 3, 0.5),
                                              (30030, 8, 4, 0.2), (65536, 8, 5, 0.45), (6144, 2, 6, 0.5)])
def test_search_walks_the_domain_as_the_algorithm_states(oracle, T, Q, seed, density):
    x = _sparse(T, seed, density, levels=1 << Q)
    n_best, best, cands = oracle.search_reshape(x, Q)
    # the same walk over independently computed costs
    nmin = _n_min(T, Q)
    want_best, want_n, prev, walked = math.inf, T, math.inf, []
    for N in _divisors_desc(T):
        if N < nmin:
            break
        cost, _ = _cost_numpy(x, N)
        walked.append(N)
        if cost < want_best:
            want_best, want_n = cost, N
        if cost > prev:
            break
        prev = cost
    assert [n for n, _ in cands] == walked
    assert n_best == want_n
    assert best == pytest.approx(want_best, rel=1e-12)
    # what the domain restrictions imply
    if cands:
        assert T % n_best == 0 and n_best >= nmin and n_best * n_best > T and T // n_best <= (1 << Q)
        costs = [c for _, c in cands]
        assert all(costs[i + 1] <= costs[i] for i in range(len(costs) - 2))   # falling until the last step
        assert best == min(costs)


def test_degenerate_inputs(oracle):
    # prime T: only N = T is in the domain
    x = _sparse(997, 1)
    n_best, best, cands = oracle.search_reshape(x, 8)
    assert n_best == 997 and [n for n, _ in cands] == [997]
    # T = 1: N_min = 2 > T, nothing to evaluate
    n_best, best, cands = oracle.search_reshape(np.array([5], np.uint8), 8)
    assert n_best == 1 and math.isinf(best) and cands == []
    # all zeros: D is r = 0 everywhere, zero entropy for every N; the first N is kept and the walk never stops early
    x = np.zeros(4096, np.uint8)
    n_best, best, cands = oracle.search_reshape(x, 8)
    assert n_best == 4096 and best == 0.0 and [n for n, _ in cands] == [4096, 2048, 1024, 512, 256, 128]
