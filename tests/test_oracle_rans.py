"""Pins for the oracle's coder (Eq. 2-4), normaliser and size bound (Eq. 1).  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import bigint_rans as big

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "eq2_two_symbol_example.txt")


def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        n, s0, sym, f, F, s1 = line.split()
        rows.append((int(n), int(s0), sym, int(f), int(F), int(s1)))
    return rows


def test_hand_example_of_eq2_and_eq4(oracle):
    rows = _golden_rows()
    assert len(rows) == 2
    for n, s0, _, f, F, s1 in rows:
        s, w = oracle.encode_step(s0, f, F, n)
        assert (s, w) == (s1, None)
        back, slot = oracle.decode_step(s1, f, F, n)
        assert back == s0 and F <= slot < F + f
    # the same example through the unbounded coder (A = 0, B = 1; encoding is last-to-first)
    assert big.encode([1, 0], [3, 1], 2, s0=4) == 23
    assert big.decode(23, 2, [3, 1], 2) == ([1, 0], 4)


def _tables(n_sym, M):
    """All tables of n_sym positive frequencies with sum 2^M."""
    total = 1 << M
    for cuts in itertools.combinations(range(1, total), n_sym - 1):
        edges = (0,) + cuts + (total,)
        yield [edges[i + 1] - edges[i] for i in range(n_sym)]


def _info_bits(seq, f, M):
    return sum(math.log2((1 << M) / f[x]) for x in seq)


def _check_stream(oracle, seq, f, M):
    """Round trip, big-integer agreement and the code-length bracket for one coder."""
    state, words = oracle.encode_stream(seq, f, M)
    assert (1 << 16) <= state < (1 << 32)
    got = oracle.decode_stream(state, words, len(seq), f, M)
    assert list(got) == list(seq)
    sb = big.encode(seq, f, M)
    dec, s_end = big.decode(sb, len(seq), f, M)
    assert dec == list(seq) and s_end == 1 << 16
    if len(words) == 0:
        assert state == sb          # no renormalisation: the 32-bit coder IS Eq. 2
    # Both coders carry 16 bits (the initial state) plus sum log2(2^M/f), up to the effect of
    # floor(s/f) on a state >= 2^16: each step moves log2(state) by at most log2(1 + 2^(M-16))
    # away from the ideal log2(2^M/f), in either direction.
    ideal = 16 + _info_bits(seq, f, M)
    slack = len(seq) * math.log2(1 + 2.0 ** (M - 16)) + 1e-6
    assert abs(16 * len(words) + math.log2(state) - ideal) <= slack
    assert abs(big.code_length_bits(sb) - ideal) <= slack
    return len(words), state


@pytest.mark.parametrize("M", [2, 3, 4])
def test_brute_force_tiny_alphabets(oracle, M):
    n_checked = 0
    for n_sym in (2, 3):
        tables = list(_tables(n_sym, M))
        if M == 4 and n_sym == 3:
            tables = tables[::7]
        for f in tables:
            max_len = 6 if n_sym == 2 else 4
            for length in range(0, max_len + 1):
                for seq in itertools.product(range(n_sym), repeat=length):
                    _check_stream(oracle, seq, f, M)
                    n_checked += 1
    assert n_checked > 700


@pytest.mark.parametrize("M", [8, 12, 14, 15])
def test_long_streams_roundtrip_and_bigint(oracle, M):
    rng = np.random.default_rng(M)
    for A in (2, 17, 256):
        if A > (1 << M):
            continue
        p = rng.dirichlet(np.ones(A) * 0.3)
        seq = rng.choice(A, size=3000, p=p)
        cnt = np.bincount(seq, minlength=A).astype(np.uint64)
        f, F = oracle.normalize(cnt, M)
        nw, state = _check_stream(oracle, [int(v) for v in seq], [int(v) for v in f], M)
        info = _info_bits(seq, f, M)
        # Eq. 1: expected size = sum of -log2 p; the coder is within the state's 16 bits of it
        slack = 3000 * math.log2(1 + 2.0 ** (M - 16)) + 1e-6
        assert info - 16 - slack <= 16 * nw <= info + slack


def test_renormalisation_emits_at_most_one_word_and_keeps_state_in_range(oracle):
    rng = np.random.default_rng(5)
    M = 12
    f = np.array([1, 4095], np.uint16)            # a very rare symbol: worst case for the state
    F = [0, 1]
    s = 1 << 16
    for _ in range(20000):
        x = int(rng.random() < 0.3)
        s, w = oracle.encode_step(s, int(f[x]), F[x], M)
        assert (1 << 16) <= s < (1 << 32)
    # f = 2^M (single symbol) leaves the state unchanged and never emits
    s2, w2 = oracle.encode_step(123456, 1 << M, 0, M)
    assert (s2, w2) == (123456, None)


@pytest.mark.parametrize("M", [4, 8, 12, 15])
def test_normalize_invariants(oracle, M):
    rng = np.random.default_rng(M)
    for trial in range(200):
        A = int(rng.integers(1, min(300, 1 << M) + 1))
        cnt = rng.integers(0, 5, A).astype(np.uint64) * rng.integers(0, 1000, A).astype(np.uint64)
        if cnt.sum() == 0:
            cnt[rng.integers(0, A)] = 1
        f, F = oracle.normalize(cnt, M)
        assert int(f.astype(np.int64).sum()) == 1 << M
        assert np.array_equal(f > 0, cnt > 0)
        assert F[0] == 0 and F[-1] == 1 << M and np.array_equal(np.diff(F.astype(np.int64)), f)


def test_normalize_special_cases(oracle):
    f, F = oracle.normalize(np.array([0, 0, 7, 0], np.uint64), 12)
    assert list(f) == [0, 0, 4096, 0]
    # equal counts: the surplus goes to the lowest index
    f, _ = oracle.normalize(np.array([1, 1, 1], np.uint64), 4)      # 16/3 -> 5,5,5 (+1)
    assert list(f) == [6, 5, 5]
    # exact powers of two stay exact
    f, _ = oracle.normalize(np.array([8, 4, 2, 2], np.uint64), 4)
    assert list(f) == [8, 4, 2, 2]
    # deficit: many singletons force f = 1 and the largest pays
    cnt = np.array([1000] + [1] * 15, np.uint64)
    f, _ = oracle.normalize(cnt, 4)
    assert list(f) == [1] + [1] * 15
    cnt = np.array([1000, 900] + [1] * 10, np.uint64)
    f, _ = oracle.normalize(cnt, 4)       # rounds to 8, 7, 1 x10 = 25 -> take 7 from a0, 2 from a1
    assert list(f) == [1, 5] + [1] * 10
    # too many present symbols
    with pytest.raises(oracle.OracleError) as e:
        oracle.normalize(np.ones(17, np.uint64), 4)
    assert e.value.code == oracle.ERR_ALPHABET
    # empty
    f, F = oracle.normalize(np.zeros(5, np.uint64), 4)
    assert f.sum() == 0


def test_normalize_permuting_equal_counts_is_deterministic(oracle):
    cnt = np.array([5, 9, 9, 5, 9], np.uint64)
    f, _ = oracle.normalize(cnt, 5)
    # 32*9/37 = 7.78 -> 8 ; 32*5/37 = 4.32 -> 4 ; sum = 32, nothing to fix
    assert list(f) == [4, 8, 8, 4, 8]
    cnt = np.array([3, 3, 3, 3, 3, 3, 3], np.uint64)       # 32/7 = 4.57 -> 5 each = 35 -> deficit 3
    f, _ = oracle.normalize(cnt, 5)
    assert list(f) == [2, 5, 5, 5, 5, 5, 5]


def test_model_overhead_bound(oracle):
    """Cross-entropy of the normalised table exceeds the empirical entropy H of Eq. 1 only slightly."""
    rng = np.random.default_rng(11)
    for M in (12, 14):
        seq = np.clip(np.round(rng.standard_normal(200000) * 20 + 128), 0, 255).astype(np.int64)
        cnt = np.bincount(seq, minlength=256).astype(np.uint64)
        f, _ = oracle.normalize(cnt, M)
        p = cnt[cnt > 0] / cnt.sum()
        H = -(p * np.log2(p)).sum()
        CE = (p * np.log2((1 << M) / f[cnt > 0])).sum()
        present = int((cnt > 0).sum())
        assert H - 1e-9 <= CE <= H + math.log2((1 << M) / ((1 << M) - present)) + 0.01
