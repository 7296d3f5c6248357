"""The C-ABI library loads and exports every symbol include/rans_if.h declares; host-only calls.  CPU only."""
import ctypes as C
import os
import re

import pytest

from paper_2511_11664_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.SO_PATH):
        B.build_library()
    return B.lib()


def test_every_declared_symbol_is_exported(lib):
    text = open(os.path.join(ROOT, "include", "rans_if.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(rans_[a-z_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name)


def test_struct_layouts_match_header():
    assert C.sizeof(B.Params) == 40 and C.sizeof(B.QInfo) == 16 and C.sizeof(B.Header) == 72
    assert C.sizeof(B.ReshapeResult) == 32 + 16 * B.RESHAPE_MAX_CAND


def test_workspace_bytes_and_argument_errors(lib):
    p = B.make_params(8, 14, 16384, 4096, B.MODE_DENSE, 1024, 1 << 18, B.F16)
    rc, ws, mx = B.rans_workspace_bytes(p, 16384 * 4096)
    assert rc == 0 and ws > 2 * 16384 * 4096 and mx > 2 * 16384 * 4096
    def rc_of(**kw):
        base = dict(q_bits=8, freq_bits=12, rows=10, cols=10, mode=0, n_streams=4, chunk_syms=8, in_dtype=0)
        base.update(kw)
        return B.rans_workspace_bytes(B.make_params(**base), 100)[0]
    assert rc_of() == 0
    assert rc_of(q_bits=0) == B.ERR_ARG and rc_of(q_bits=9) == B.ERR_ARG
    assert rc_of(freq_bits=0) == B.ERR_ARG and rc_of(freq_bits=16) == B.ERR_ARG
    assert rc_of(n_streams=0) == B.ERR_ARG and rc_of(mode=2) == B.ERR_ARG and rc_of(in_dtype=2) == B.ERR_ARG
    assert rc_of(rows=9) == B.ERR_SHAPE and rc_of(cols=0) == B.ERR_SHAPE and rc_of(chunk_syms=6) == B.ERR_SHAPE
    assert B.rans_workspace_bytes(B.make_params(8, 12, 1, 65536, 1, 4, 0, 0), 65536)[0] == B.ERR_ALPHABET
    assert B.rans_workspace_bytes(B.make_params(8, 12, 1, (1 << 30) + 1, 0, 4, 0, 0), (1 << 30) + 1)[0] == B.ERR_ARG


def test_peek_header_agrees_with_oracle_container(lib, oracle):
    import numpy as np
    x = np.maximum(np.random.default_rng(0).standard_normal(600), 0).astype(np.float32)
    for mode, cols in ((0, 1), (1, 6)):
        p = oracle.make_params(6, 11, 600 // cols, cols, mode, 16, 64, 0)
        buf, _ = oracle.compress(x, p)
        rc, h = B.rans_peek_header(buf[:128])
        oh = oracle.parse_header(buf)
        assert rc == 0
        assert (h.p.q_bits, h.p.freq_bits, h.p.rows, h.p.cols, h.p.mode, h.p.n_streams, h.p.chunk_syms,
                h.p.in_dtype) == (6, 11, 600 // cols, cols, mode, 16, 64, 0)
        assert (h.n_elems, h.len_d, h.alphabet, h.n_chunks) == (oh.n_elems, oh.len_D, oh.A, oh.n_chunks)
        assert (h.x_min, h.x_max) == (oh.x_min, oh.x_max)
        bad = bytearray(buf[:128])
        bad[0] ^= 1
        assert B.rans_peek_header(bytes(bad))[0] == B.ERR_CORRUPT
        assert B.rans_peek_header(buf[:100])[0] == B.ERR_CORRUPT
        bad = bytearray(buf[:128])
        bad[48] ^= 1            # S no longer divides chunk_syms / does not match n_chunks
        assert B.rans_peek_header(bytes(bad))[0] == B.ERR_CORRUPT


def test_strerror(lib):
    assert B.rans_strerror(0) == "ok" and "corrupt" in B.rans_strerror(B.ERR_CORRUPT)
