"""The all-cores timing driver of the oracle (oracle/rans_oracle_mt.cpp) produces the oracle's own bytes and
values for any thread count: it only cuts the work into pieces and calls the oracle's routines.  CPU only."""
import numpy as np
import pytest

from paper_2511_11664_amd import synth


@pytest.mark.parametrize("name,shrink,over", [
    ("c1", 1, dict(mode=0)), ("c1", 1, dict(cols=7, chunk_syms=32 * 128)), ("c1", 1, {}),
    ("c2", 64, {}), ("c3", 128, dict(q_bits=6, cols=64)), ("c4", 16, {}), ("c5a", 64, {}),
])
@pytest.mark.parametrize("threads", [1, 3, 8])
def test_threaded_driver_equals_the_oracle(oracle, name, shrink, over, threads):
    w = synth.workload(name, shrink, **over)
    x = synth.make(w).numpy()
    p = oracle.make_params(w.q_bits, w.freq_bits, w.rows, w.cols, w.mode, w.n_streams, w.chunk_syms, w.in_dtype)
    want, sym = oracle.compress(x, p)
    got = oracle.compress_mt(x, p, threads)
    assert got == want
    s1, _, y1 = oracle.decompress(want, w.in_dtype)
    s2, y2 = oracle.decompress_mt(want, w.in_dtype, threads)
    assert np.array_equal(s1, s2) and np.array_equal(y1.view(np.uint8), y2.view(np.uint8))


def test_threaded_driver_edge_cases(oracle):
    for n, rows, cols, mode in ((0, 0, 4, 0), (0, 0, 4, 1), (1, 1, 1, 1), (5, 5, 1, 0), (12, 3, 4, 1)):
        x = np.linspace(-1.0, 2.0, n).astype(np.float32) if n else np.zeros(0, np.float32)
        p = oracle.make_params(8, 12, rows, cols, mode, 4, 8, 0)
        want, _ = oracle.compress(x, p)
        assert oracle.compress_mt(x, p, 8) == want
        s1, _, y1 = oracle.decompress(want)
        s2, y2 = oracle.decompress_mt(want, 0, 8)
        assert np.array_equal(s1, s2) and np.array_equal(y1, y2)
    # errors pass through
    bad = np.array([1.0, np.nan, 2.0, 3.0], np.float32)
    with pytest.raises(oracle.OracleError) as e:
        oracle.compress_mt(bad, oracle.make_params(8, 12, 4, 1, 0, 4, 0, 0), 3)
    assert e.value.code == oracle.ERR_NONFINITE
    good, _ = oracle.compress(np.arange(100, dtype=np.float32), oracle.make_params(8, 12, 100, 1, 0, 4, 16, 0))
    cut = bytearray(good)
    cut[-3] ^= 0x40
    with pytest.raises(oracle.OracleError) as e:
        oracle.decompress_mt(bytes(cut), 0, 4)
    assert e.value.code == oracle.ERR_CORRUPT
