"""Pins for the oracle's sparse representation (Sec. 3.1), container and whole path.  CPU only."""
import itertools
import math
import struct

import numpy as np
import pytest
import scipy.sparse as sp

from paper_2511_11664_amd import synth


def test_csr_matches_scipy_and_naive_on_all_tiny_matrices(oracle):
    for rows, cols in ((3, 3), (2, 4), (4, 2), (1, 5), (5, 1)):
        for vals in itertools.product(range(3), repeat=rows * cols):
            m = np.array(vals, np.uint8).reshape(rows, cols)
            v, c, r = oracle.csr(m, rows, cols)
            ri, ci = np.nonzero(m)                                # row-major order of the nonzeros
            assert np.array_equal(v, m[ri, ci]) and np.array_equal(c, ci)
            assert np.array_equal(r, np.bincount(ri, minlength=rows))   # NON-cumulative row counts
            if (rows, cols) == (2, 4):
                ref = sp.csr_matrix(m)
                ref.sort_indices()
                assert np.array_equal(v, ref.data) and np.array_equal(c, ref.indices)
                assert np.array_equal(r, np.diff(ref.indptr))    # standard CSR keeps the cumulative sum instead
            assert np.array_equal(oracle.csr_expand(v, c, r, rows, cols, 8).reshape(rows, cols), m)


def test_csr_structural_invariants(oracle):
    rng = np.random.default_rng(0)
    for rows, cols in ((64, 7), (10, 300), (1, 1000), (1000, 1)):
        x = (rng.integers(0, 256, rows * cols) * (rng.random(rows * cols) < 0.3)).astype(np.uint8)
        v, c, r = oracle.csr(x, rows, cols)
        nnz = int(np.count_nonzero(x))
        assert v.size == c.size == nnz and r.size == rows and int(r.sum()) == nnz
        assert v.min(initial=1) >= 1 and c.max(initial=0) < cols and r.max(initial=0) <= cols
        p = oracle.make_params(8, 12, rows, cols, oracle.MODE_CSR, 4, 0, 0)
        D = oracle.symbols_D(x, p)
        assert D.size == 2 * nnz + rows                             # l_D = 2 nnz + N
        assert np.array_equal(D[:nnz], v) and np.array_equal(D[nnz:2 * nnz], c) and np.array_equal(D[2 * nnz:], r)
        # strictly increasing columns inside a row
        start = np.concatenate([[0], np.cumsum(r)]).astype(np.int64)
        for i in range(rows):
            assert np.all(np.diff(c[start[i]:start[i + 1]].astype(np.int64)) > 0)


def test_csr_expand_rejects_malformed(oracle):
    v = np.array([1, 2], np.uint16)
    c = np.array([0, 1], np.uint16)
    r = np.array([2, 0], np.uint16)
    assert oracle.csr_expand(v, c, r, 2, 2, 8).tolist() == [1, 2, 0, 0]
    for bad in (dict(v=np.array([0, 2], np.uint16)), dict(v=np.array([1, 256], np.uint16)),
                dict(c=np.array([0, 2], np.uint16)), dict(c=np.array([1, 1], np.uint16)),
                dict(r=np.array([1, 0], np.uint16)), dict(r=np.array([3, 0], np.uint16))):
        args = dict(v=v, c=c, r=r)
        args.update(bad)
        with pytest.raises(oracle.OracleError) as e:
            oracle.csr_expand(args["v"], args["c"], args["r"], 2, 2, 8)
        assert e.value.code == oracle.ERR_CORRUPT


def test_alphabet(oracle):
    assert oracle.alphabet(oracle.MODE_DENSE, 8, 100000) == 256
    assert oracle.alphabet(oracle.MODE_CSR, 8, 7) == 256
    assert oracle.alphabet(oracle.MODE_CSR, 8, 256) == 257        # r can equal K
    assert oracle.alphabet(oracle.MODE_CSR, 4, 3136) == 3137


def test_histogram_is_the_count_of_every_symbol_of_D(oracle):
    """Sec. 3.1 "Concatenation and rANS Encoding": one frequency vector over the whole of D.  Against numpy's
    bincount on ragged lengths; the last (and the first) symbol of D is unique in some cases, so that a loop
    which stops one symbol early, starts one late or counts one twice is caught."""
    rng = np.random.default_rng(3)
    for length in (0, 1, 2, 3, 7, 64, 65, 1000, 4097, 70001):
        for A in (2, 5, 256, 257, 3137):
            D = rng.integers(0, A - 1, length).astype(np.uint16)      # symbol A - 1 stays free
            if length >= 2:
                D[-1] = A - 1                                          # occurs once, at the very end
            got = oracle.histogram(D, A)
            want = np.bincount(D, minlength=A).astype(np.uint64)
            assert got.dtype == np.uint64 and got.size == A
            assert np.array_equal(got, want)
            assert int(got.sum()) == length
            if length >= 2:
                assert got[A - 1] == 1
                D2 = D.copy()
                D2[0] = A - 1                                          # and once at the very start
                assert oracle.histogram(D2, A)[A - 1] == 2
    # the histograms of v, c and r, padded to a common length and added, are the histogram of D = v (+) c (+) r
    x = (rng.integers(0, 256, 60 * 37) * (rng.random(60 * 37) < 0.4)).astype(np.uint8)
    p = oracle.make_params(8, 12, 60, 37, oracle.MODE_CSR, 4, 0, 0)
    D = oracle.symbols_D(x, p)
    m = x.reshape(60, 37)
    ri, ci = np.nonzero(m)
    parts = (np.bincount(m[ri, ci], minlength=256), np.bincount(ci, minlength=256),
             np.bincount(np.count_nonzero(m, axis=1), minlength=256))
    assert np.array_equal(oracle.histogram(D, 256), (parts[0] + parts[1] + parts[2]).astype(np.uint64))


def _fields(buf):
    """Re-read every header field straight from the bytes."""
    magic, ver, mode, dt, q, m, rsv = struct.unpack_from("<4sHBBBBH", buf, 0)
    T, N, K, lenD = struct.unpack_from("<QQQQ", buf, 12)
    A, S, cs, nc = struct.unpack_from("<IIII", buf, 44)
    xmin, xmax = struct.unpack_from("<ff", buf, 60)
    return dict(magic=magic, ver=ver, mode=mode, dt=dt, q=q, m=m, rsv=rsv, T=T, N=N, K=K, lenD=lenD, A=A, S=S,
                cs=cs, nc=nc, xmin=xmin, xmax=xmax, tail=bytes(buf[68:128]))


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("S,cs,n", [(1, 0, 1000), (3, 30, 1000), (32, 0, 5000), (32, 64, 5000), (64, 128, 127),
                                    (8, 8, 9), (5, 0, 3)])
def test_container_layout_and_roundtrip(oracle, mode, S, cs, n):
    rng = np.random.default_rng(n + S)
    cols = 10 if n % 10 == 0 else 1
    x = (np.maximum(rng.standard_normal(n), 0) * 2).astype(np.float32)
    p = oracle.make_params(6, 10, n // cols, cols, mode, S, cs, 0)
    buf, sym = oracle.compress(x, p)
    sym_ref, qi = oracle.quantize(x, 6)
    assert np.array_equal(sym, sym_ref)
    D = oracle.symbols_D(sym, p)
    h = _fields(buf)
    nc = 0 if D.size == 0 else (1 if cs == 0 else -(-D.size // cs))
    A = oracle.alphabet(mode, 6, cols)
    assert h == dict(magic=b"RIF1", ver=1, mode=mode, dt=0, q=6, m=10, rsv=0, T=n, N=n // cols, K=cols,
                     lenD=D.size, A=A, S=S, cs=cs, nc=nc, xmin=qi.x_min, xmax=qi.x_max, tail=bytes(60))
    sec = oracle.container_sections(buf)
    # the one frequency vector over all of D, counted here without the oracle's histogram routine
    f, _ = oracle.normalize(np.bincount(D, minlength=A).astype(np.uint64), 10)
    assert np.array_equal(sec["f"], f)
    # directory and chunk sizes
    table_bytes = (2 * A + 7) // 8 * 8
    pos = 0
    clen = cs if cs else D.size
    for k, (states, nwords, words) in enumerate(sec["chunks"]):
        assert sec["off"][k] == pos
        size = 8 * S + 2 * int(nwords.sum())
        pos += (size + 3) // 4 * 4
        chunk = D[k * clen:(k + 1) * clen]
        for j in range(S):                                       # stream j = local symbols j, j+S, ...
            st, w = oracle.encode_stream(chunk[j::S], f, 10)
            assert st == states[j] and np.array_equal(w, words[j])
    assert sec["off"][-1] == pos and len(buf) == 128 + table_bytes + 8 * (nc + 1) + pos
    # decode
    D2, _ = oracle.decode_container(buf)
    assert np.array_equal(D2, D)
    sym2, qi2, y = oracle.decompress(buf)
    assert np.array_equal(sym2, sym) and qi2.as_tuple() == qi.as_tuple()
    assert np.array_equal(y, oracle.dequantize(sym, qi))


def test_size_against_entropy_bound(oracle):
    """Eq. 1: payload words ~ l_D * cross-entropy of the stored table, within the per-stream state slack."""
    rng = np.random.default_rng(2)
    x = np.maximum(rng.standard_normal(60000), 0).astype(np.float32)
    for mode, cols in ((0, 1), (1, 8)):
        for S, cs in ((32, 0), (64, 4096)):
            M = 12
            p = oracle.make_params(8, M, x.size // cols, cols, mode, S, cs, 0)
            buf, sym = oracle.compress(x, p)
            D = oracle.symbols_D(sym, p)
            sec = oracle.container_sections(buf)
            f = sec["f"].astype(np.float64)
            info = float(np.sum(np.log2((1 << M) / f[D])))
            words = sum(int(nw.sum()) for _, nw, _ in sec["chunks"])
            n_streams = S * len(sec["chunks"])
            slack = D.size * math.log2(1 + 2.0 ** (M - 16))
            assert info - 16 * n_streams - slack <= 16 * words <= info + slack


def test_empty_and_degenerate_inputs(oracle):
    p = oracle.make_params(8, 12, 0, 4, 0, 32, 0, 0)
    buf, sym = oracle.compress(np.zeros(0, np.float32), p)
    assert len(buf) == 128 + 512 + 8 and sym.size == 0
    s2, qi, y = oracle.decompress(buf)
    assert s2.size == 0
    p = oracle.make_params(8, 12, 0, 4, 1, 32, 0, 0)
    buf, _ = oracle.compress(np.zeros(0, np.float32), p)
    assert oracle.decompress(buf)[0].size == 0
    # constant tensor: one symbol, f = 2^M, no words at all
    for mode in (0, 1):
        p = oracle.make_params(8, 12, 25, 4, mode, 8, 16, 0)
        buf, sym = oracle.compress(np.full(100, -2.5, np.float32), p)
        sec = oracle.container_sections(buf)
        assert all(int(nw.sum()) == 0 for _, nw, _ in sec["chunks"])
        s2, qi, y = oracle.decompress(buf)
        assert np.all(s2 == 0) and np.all(y == np.float32(-2.5))


def test_argument_errors(oracle):
    x = np.ones(100, np.float32)
    def code(**kw):
        base = dict(q_bits=8, freq_bits=12, rows=10, cols=10, mode=0, n_streams=4, chunk_syms=8, in_dtype=0)
        base.update(kw)
        try:
            oracle.compress(x, oracle.make_params(**base))
        except oracle.OracleError as e:
            return e.code
        return 0
    assert code() == 0
    assert code(q_bits=0) == oracle.ERR_ARG and code(q_bits=9) == oracle.ERR_ARG
    assert code(freq_bits=0) == oracle.ERR_ARG and code(freq_bits=16) == oracle.ERR_ARG
    assert code(n_streams=0) == oracle.ERR_ARG and code(mode=2) == oracle.ERR_ARG
    assert code(rows=9) == oracle.ERR_SHAPE and code(cols=0) == oracle.ERR_SHAPE
    assert code(chunk_syms=6) == oracle.ERR_SHAPE
    # more present symbols than 2^M
    y = np.arange(100, dtype=np.float32)
    with pytest.raises(oracle.OracleError) as e:
        oracle.compress(y, oracle.make_params(8, 4, 10, 10, 0, 4, 0, 0))
    assert e.value.code == oracle.ERR_ALPHABET
    # CSR with K + 1 > 65536
    z = np.ones(65536, np.float32)
    with pytest.raises(oracle.OracleError) as e:
        oracle.compress(z, oracle.make_params(8, 12, 1, 65536, 1, 4, 0, 0))
    assert e.value.code == oracle.ERR_ALPHABET


def test_corruption_is_detected_not_crashing(oracle):
    rng = np.random.default_rng(9)
    x = np.maximum(rng.standard_normal(3000), 0).astype(np.float32)
    for mode, cols in ((0, 1), (1, 6)):
        p = oracle.make_params(8, 11, x.size // cols, cols, mode, 16, 256, 0)
        buf, sym = oracle.compress(x, p)
        ok = 0
        for trial in range(1500):
            b = bytearray(buf)
            kind = trial % 3
            if kind == 0:
                b[rng.integers(0, len(b))] ^= 1 << int(rng.integers(0, 8))
            elif kind == 1:
                b = b[:rng.integers(0, len(b))]
            else:
                pos = int(rng.integers(0, len(b)))
                b[pos:pos + 4] = rng.integers(0, 256, len(b[pos:pos + 4]), dtype=np.uint8).tobytes()
            try:
                s2, _, _ = oracle.decompress(bytes(b))
                ok += 1                      # a mutation the validation cannot see (e.g. x_min bits)
                if kind == 1:
                    assert False, "a truncated container must never decode"
            except oracle.OracleError as e:
                assert e.code == oracle.ERR_CORRUPT
        assert ok < 150


@pytest.mark.parametrize("name,shrink,over", [
    ("c1", 1, dict(mode=0)), ("c1", 1, {}), ("c1", 1, dict(cols=7, chunk_syms=32 * 128)),
    ("c2", 64, dict(mode=0)), ("c2", 64, {}), ("c3", 128, dict(q_bits=6, cols=64)),
    ("c4", 16, {}), ("c5a", 64, {}), ("c5b", 64, dict(chunk_syms=1 << 20)),
])
def test_whole_path_on_synthetic_workloads(oracle, name, shrink, over):
    w = synth.workload(name, shrink, **over)
    x = synth.make(w).numpy()
    p = oracle.make_params(w.q_bits, w.freq_bits, w.rows, w.cols, w.mode, w.n_streams, w.chunk_syms, w.in_dtype)
    buf, sym = oracle.compress(x, p)
    s2, qi, y = oracle.decompress(buf, w.in_dtype)
    assert np.array_equal(s2, sym)
    assert sym.max() == (1 << w.q_bits) - 1 or w.name.startswith("c4") or w.name.startswith("c5")
    err = np.abs(y.astype(np.float64) - x.astype(np.float64)).max()
    assert err <= qi.scale * 1.01 + (abs(float(x.astype(np.float64).max())) * 2 ** -10 if w.in_dtype else 0)
    assert len(buf) < x.nbytes


def test_container_digests_of_formula_inputs_are_unchanged():
    """The oracle's containers for inputs given by closed formulas against the digests stored by
    tests/golden/make_oracle_digests.py: an unintended change of the arithmetic or the layout changes a digest."""
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_oracle_digests", os.path.join(here, "golden", "make_oracle_digests.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = {}
    for line in open(os.path.join(here, "golden", "oracle_container_digests.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, n, h = line.split()
        stored[name] = (int(n), h)
    got = {name: (n, h) for name, n, h in mod.digests()}
    assert got == stored
