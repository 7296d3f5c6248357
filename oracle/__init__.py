"""CPU oracle for the rANS intermediate-feature codec -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``rans_oracle.c`` (plain C, written from the paper's
Sec. 2.1 and Sec. 3.1).  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does, and
this package imports nothing from the GPU library.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_DIR, "librans_oracle.so")
_SRC = os.path.join(_DIR, "rans_oracle.c")

OK, ERR_ARG, ERR_SHAPE, ERR_ALPHABET, ERR_CAPACITY, ERR_NONFINITE, ERR_CORRUPT = 0, -1, -2, -3, -4, -6, -7
MODE_DENSE, MODE_CSR = 0, 1
F32, F16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, no fast-math)."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < max(
        os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_DIR, "rans_oracle.h")))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
               "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_SO_MT = os.path.join(_DIR, "librans_oracle_mt.so")
_SRC_MT = os.path.join(_DIR, "rans_oracle_mt.cpp")


def build_mt(force: bool = False) -> str:
    """Compile the all-cores timing driver (rans_oracle_mt.cpp: std::thread around the oracle's own routines)
    together with the oracle into one shared library."""
    srcs = (_SRC, _SRC_MT, os.path.join(_DIR, "rans_oracle.h"))
    stale = (not os.path.exists(_SO_MT)) or os.path.getmtime(_SO_MT) < max(os.path.getmtime(f) for f in srcs)
    if force or stale:
        obj = os.path.join(_DIR, "rans_oracle_mt_c.o")
        subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-fPIC",
                        "-c", "-o", obj, _SRC], check=True)
        subprocess.run(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared",
                        "-fPIC", "-pthread", "-I", _DIR, "-o", _SO_MT, _SRC_MT, obj, "-lm"], check=True)
        os.remove(obj)
    return _SO_MT


class Params(C.Structure):
    _fields_ = [("q_bits", C.c_uint32), ("freq_bits", C.c_uint32), ("rows", C.c_uint64),
                ("cols", C.c_uint64), ("mode", C.c_uint32), ("n_streams", C.c_uint32),
                ("chunk_syms", C.c_uint32), ("in_dtype", C.c_uint32)]


class QInfo(C.Structure):
    _fields_ = [("x_min", C.c_float), ("x_max", C.c_float), ("scale", C.c_float),
                ("zero_point", C.c_float)]

    def as_tuple(self):
        return (np.float32(self.x_min), np.float32(self.x_max), np.float32(self.scale),
                np.float32(self.zero_point))


class Header(C.Structure):
    _fields_ = [("p", Params), ("n_elems", C.c_uint64), ("len_D", C.c_uint64), ("A", C.c_uint32),
                ("n_chunks", C.c_uint32), ("x_min", C.c_float), ("x_max", C.c_float),
                ("table_off", C.c_size_t), ("dir_off", C.c_size_t), ("payload_off", C.c_size_t)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_half_to_float.restype = C.c_float
        _lib.orc_half_to_float.argtypes = [C.c_uint16]
        _lib.orc_float_to_half.restype = C.c_uint16
        _lib.orc_float_to_half.argtypes = [C.c_float]
        _lib.orc_quantize_one.restype = C.c_uint8
        _lib.orc_quantize_one.argtypes = [C.c_float, C.POINTER(QInfo), C.c_uint32]
        _lib.orc_dequantize_one.restype = C.c_float
        _lib.orc_dequantize_one.argtypes = [C.c_uint8, C.POINTER(QInfo)]
        _lib.orc_alphabet.restype = C.c_uint32
        _lib.orc_alphabet.argtypes = [C.c_uint32, C.c_uint32, C.c_uint64]
        _lib.orc_container_bound.restype = C.c_size_t
        _lib.orc_container_bound.argtypes = [C.c_uint64, C.POINTER(Params), C.c_uint64]
        _lib.orc_rans_decode_step.restype = C.c_uint32
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _dtype_code(x: np.ndarray) -> int:
    if x.dtype == np.float32:
        return F32
    if x.dtype == np.float16:
        return F16
    raise TypeError("oracle takes float32 or float16 arrays")


def make_params(q_bits, freq_bits, rows, cols, mode, n_streams, chunk_syms, in_dtype) -> Params:
    return Params(q_bits, freq_bits, rows, cols, mode, n_streams, chunk_syms, in_dtype)


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle error {code}")
        self.code = code


def _check(rc):
    if rc != OK:
        raise OracleError(rc)


# ---------------------------------------------------------------- pieces

def half_to_float(h: int) -> np.float32:
    return np.float32(lib().orc_half_to_float(h))


def float_to_half(x) -> int:
    return int(lib().orc_float_to_half(C.c_float(float(x))))


def minmax(x: np.ndarray):
    x = np.ascontiguousarray(x).reshape(-1)
    mn, mx = C.c_float(), C.c_float()
    _check(lib().orc_minmax(_ptr(x), C.c_uint64(x.size), _dtype_code(x), C.byref(mn), C.byref(mx)))
    return np.float32(mn.value), np.float32(mx.value)


def qinfo_from_minmax(x_min, x_max, q_bits) -> QInfo:
    qi = QInfo()
    _check(lib().orc_qinfo_from_minmax(C.c_float(float(x_min)), C.c_float(float(x_max)), q_bits, C.byref(qi)))
    return qi


def quantize(x: np.ndarray, q_bits: int):
    """Eq. 6 over a tensor -> (uint8 symbols, QInfo)."""
    x = np.ascontiguousarray(x).reshape(-1)
    sym = np.empty(x.size, np.uint8)
    qi = QInfo()
    _check(lib().orc_quantize(_ptr(x), C.c_uint64(x.size), _dtype_code(x), q_bits, _ptr(sym), C.byref(qi)))
    return sym, qi


def quantize_one(x, qi: QInfo, q_bits: int) -> int:
    return int(lib().orc_quantize_one(C.c_float(float(x)), C.byref(qi), q_bits))


def dequantize(sym: np.ndarray, qi: QInfo, out_dtype=F32) -> np.ndarray:
    sym = np.ascontiguousarray(sym, np.uint8).reshape(-1)
    out = np.empty(sym.size, np.float32 if out_dtype == F32 else np.float16)
    _check(lib().orc_dequantize(_ptr(sym), C.c_uint64(sym.size), C.byref(qi), out_dtype, _ptr(out)))
    return out


def csr(xhat: np.ndarray, rows: int, cols: int):
    """Modified CSR of Sec. 3.1 -> (v, c, r) as uint16 arrays."""
    xhat = np.ascontiguousarray(xhat, np.uint8).reshape(-1)
    assert xhat.size == rows * cols
    v = np.empty(max(xhat.size, 1), np.uint16)
    c = np.empty(max(xhat.size, 1), np.uint16)
    r = np.empty(max(rows, 1), np.uint16)
    nnz = C.c_uint64()
    _check(lib().orc_csr(_ptr(xhat), C.c_uint64(rows), C.c_uint64(cols), _ptr(v), _ptr(c), _ptr(r), C.byref(nnz)))
    return v[:nnz.value].copy(), c[:nnz.value].copy(), r[:rows].copy()


def csr_expand(v, c, r, rows, cols, q_bits) -> np.ndarray:
    v = np.ascontiguousarray(v, np.uint16)
    c = np.ascontiguousarray(c, np.uint16)
    r = np.ascontiguousarray(r, np.uint16)
    out = np.empty(max(rows * cols, 1), np.uint8)
    _check(lib().orc_csr_expand(_ptr(v), _ptr(c), _ptr(r), C.c_uint64(v.size), C.c_uint64(rows),
                                C.c_uint64(cols), q_bits, _ptr(out)))
    return out[:rows * cols]


def alphabet(mode, q_bits, cols) -> int:
    return int(lib().orc_alphabet(mode, q_bits, C.c_uint64(cols)))


def symbols_D(xhat: np.ndarray, p: Params) -> np.ndarray:
    """Eq. 7: D = v (+) c (+) r in CSR mode, D = xhat in DENSE mode (uint16)."""
    if p.mode == MODE_DENSE:
        return np.ascontiguousarray(xhat, np.uint8).reshape(-1).astype(np.uint16)
    v, c, r = csr(xhat, p.rows, p.cols)
    return np.concatenate([v, c, r]).astype(np.uint16)


def histogram(D: np.ndarray, A: int) -> np.ndarray:
    D = np.ascontiguousarray(D, np.uint16)
    cnt = np.zeros(A, np.uint64)
    lib().orc_histogram(_ptr(D), C.c_uint64(D.size), A, _ptr(cnt))
    return cnt


def normalize(cnt: np.ndarray, M: int):
    """counts -> (f uint16[A], F uint32[A+1]) with sum f = 2^M."""
    cnt = np.ascontiguousarray(cnt, np.uint64)
    f = np.zeros(cnt.size, np.uint16)
    F = np.zeros(cnt.size + 1, np.uint32)
    _check(lib().orc_normalize(_ptr(cnt), cnt.size, M, _ptr(f), _ptr(F)))
    return f, F


def encode_step(state: int, fx: int, Fx: int, M: int):
    """One Eq. 2 step with renormalisation -> (new_state, emitted_word or None)."""
    s = C.c_uint32(state)
    w = C.c_uint16(0)
    em = lib().orc_rans_encode_step(C.byref(s), fx, Fx, M, C.byref(w))
    return s.value, (w.value if em else None)


def decode_step(state: int, fx: int, Fx: int, M: int):
    """One Eq. 4 step (symbol already selected) -> (new_state, slot)."""
    s = C.c_uint32(state)
    slot = lib().orc_rans_decode_step(C.byref(s), fx, Fx, M)
    return s.value, slot


def encode_stream(symbols, f, M):
    """One coder over ``symbols`` with table f -> (final_state, words in read order)."""
    D = np.ascontiguousarray(symbols, np.uint16)
    f = np.ascontiguousarray(f, np.uint16)
    F = np.concatenate([[0], np.cumsum(f.astype(np.uint64))]).astype(np.uint32)
    words = np.zeros(max(D.size, 1), np.uint16)
    nw, st = C.c_uint64(), C.c_uint32()
    _check(lib().orc_encode_stream(_ptr(D), C.c_uint64(0), C.c_uint64(1), C.c_uint64(D.size), _ptr(f), _ptr(F),
                                   M, _ptr(words), C.byref(nw), C.byref(st)))
    return st.value, words[:nw.value].copy()


def decode_stream(state, words, n, f, M):
    """Inverse of encode_stream -> symbols (raises OracleError(ERR_CORRUPT) on failure)."""
    words = np.ascontiguousarray(words, np.uint16)
    f = np.ascontiguousarray(f, np.uint16)
    F = np.concatenate([[0], np.cumsum(f.astype(np.uint64))]).astype(np.uint32)
    D = np.zeros(max(n, 1), np.uint16)
    _check(lib().orc_decode_stream(C.c_uint32(state), _ptr(words), C.c_uint64(words.size), _ptr(f), _ptr(F),
                                   f.size, M, _ptr(D), C.c_uint64(0), C.c_uint64(1), C.c_uint64(n)))
    return D[:n]


def encode_container(D: np.ndarray, p: Params, n_elems: int, x_min=0.0, x_max=0.0) -> bytes:
    D = np.ascontiguousarray(D, np.uint16)
    cap = lib().orc_container_bound(C.c_uint64(D.size), C.byref(p), C.c_uint64(n_elems))
    out = np.empty(cap, np.uint8)
    nb = C.c_size_t()
    _check(lib().orc_encode_container(_ptr(D), C.c_uint64(D.size), C.byref(p), C.c_uint64(n_elems),
                                      C.c_float(float(x_min)), C.c_float(float(x_max)), _ptr(out),
                                      C.c_size_t(cap), C.byref(nb)))
    return out[:nb.value].tobytes()


def parse_header(buf) -> Header:
    a = np.frombuffer(bytes(buf), np.uint8)
    h = Header()
    _check(lib().orc_parse_header(_ptr(a), C.c_size_t(a.size), C.byref(h)))
    return h


def decode_container(buf):
    """container -> (D uint16, Header), fully validated."""
    a = np.frombuffer(bytes(buf), np.uint8)
    h = parse_header(buf)
    D = np.empty(max(h.len_D, 1), np.uint16)
    _check(lib().orc_decode_container(_ptr(a), C.c_size_t(a.size), _ptr(D), C.c_uint64(D.size), C.byref(h)))
    return D[:h.len_D], h


def container_sections(buf):
    """Split a container into its parts for inspection: dict with header, f,
    directory, and per chunk (states, nwords, list of per-stream word arrays)."""
    a = np.frombuffer(bytes(buf), np.uint8)
    h = parse_header(buf)
    f = a[h.table_off:h.table_off + 2 * h.A].view("<u2").copy()
    off = a[h.dir_off:h.dir_off + 8 * (h.n_chunks + 1)].view("<u8").copy()
    chunks = []
    S = h.p.n_streams
    for k in range(h.n_chunks):
        ck = a[h.payload_off + int(off[k]):h.payload_off + int(off[k + 1])]
        states = ck[:4 * S].view("<u4").copy()
        nwords = ck[4 * S:8 * S].view("<u4").copy()
        pos = 8 * S
        words = []
        for j in range(S):
            n = int(nwords[j])
            words.append(ck[pos:pos + 2 * n].view("<u2").copy())
            pos += 2 * n
        chunks.append((states, nwords, words))
    return {"header": h, "f": f, "off": off, "chunks": chunks}


# ---------------------------------------------------------------- whole path

def compress(x: np.ndarray, p: Params):
    """tensor -> (container bytes, uint8 symbols)."""
    x = np.ascontiguousarray(x).reshape(-1)
    assert _dtype_code(x) == p.in_dtype
    worst_len = x.size if p.mode == MODE_DENSE else 2 * x.size + p.rows
    cap = lib().orc_container_bound(C.c_uint64(worst_len), C.byref(p), C.c_uint64(x.size))
    out = np.empty(cap, np.uint8)
    sym = np.empty(max(x.size, 1), np.uint8)
    nb = C.c_size_t()
    _check(lib().orc_compress(_ptr(x), C.c_uint64(x.size), C.byref(p), _ptr(out), C.c_size_t(cap),
                              C.byref(nb), _ptr(sym)))
    return out[:nb.value].tobytes(), sym[:x.size]


def decompress(buf, out_dtype=F32):
    """container -> (uint8 symbols, QInfo, dequantised array)."""
    a = np.frombuffer(bytes(buf), np.uint8)
    h = parse_header(buf)
    sym = np.empty(max(h.n_elems, 1), np.uint8)
    out = np.empty(max(h.n_elems, 1), np.float32 if out_dtype == F32 else np.float16)
    qi = QInfo()
    _check(lib().orc_decompress(_ptr(a), C.c_size_t(a.size), _ptr(sym), C.c_uint64(sym.size), C.byref(qi),
                                out_dtype, _ptr(out)))
    return sym[:h.n_elems], qi, out[:h.n_elems]


_lib_mt = None


def lib_mt():
    global _lib_mt
    if _lib_mt is None:
        _lib_mt = C.CDLL(build_mt())
        _lib_mt.orc_container_bound.restype = C.c_size_t
        _lib_mt.orc_container_bound.argtypes = [C.c_uint64, C.POINTER(Params), C.c_uint64]
    return _lib_mt


def compress_mt(x: np.ndarray, p: Params, n_threads: int) -> bytes:
    """The oracle's container, computed by n_threads threads (timing driver; same bytes as compress)."""
    x = np.ascontiguousarray(x).reshape(-1)
    assert _dtype_code(x) == p.in_dtype
    worst_len = x.size if p.mode == MODE_DENSE else 2 * x.size + p.rows
    cap = lib_mt().orc_container_bound(C.c_uint64(worst_len), C.byref(p), C.c_uint64(x.size))
    out = np.empty(cap, np.uint8)
    nb = C.c_size_t()
    _check(lib_mt().orc_mt_compress(_ptr(x), C.c_uint64(x.size), C.byref(p), _ptr(out), C.c_size_t(cap), C.byref(nb),
                                    C.c_uint(n_threads)))
    return out[:nb.value].tobytes()


def decompress_mt(buf, out_dtype, n_threads: int):
    """container -> (uint8 symbols, dequantised array) by n_threads threads (same values as decompress)."""
    a = np.frombuffer(bytes(buf), np.uint8) if not isinstance(buf, np.ndarray) else buf
    hh = Header()
    _check(lib().orc_parse_header(_ptr(a), C.c_size_t(a.size), C.byref(hh)))
    sym = np.empty(max(hh.n_elems, 1), np.uint8)
    out = np.empty(max(hh.n_elems, 1), np.float32 if out_dtype == F32 else np.float16)
    _check(lib_mt().orc_mt_decompress(_ptr(a), C.c_size_t(a.size), _ptr(sym), C.c_uint64(sym.size), out_dtype, _ptr(out),
                                      C.c_uint(n_threads)))
    return sym[:hh.n_elems], out[:hh.n_elems]


def reshape_cost(xhat: np.ndarray, n_rows: int, q_bits: int):
    """Size proxy l_D * H(p(N)) in bits for the reshape [N, T/N] (Sec. 3.2, Eq. 8 with both alphas 0)."""
    xhat = np.ascontiguousarray(xhat, dtype=np.uint8).ravel()
    cost = C.c_double()
    len_d = C.c_uint64()
    _check(lib().orc_reshape_cost(_ptr(xhat), C.c_uint64(xhat.size), C.c_uint64(n_rows), C.c_uint32(q_bits),
                                  C.byref(cost), C.byref(len_d)))
    return cost.value, len_d.value


def search_reshape(xhat: np.ndarray, q_bits: int, cap: int = 4096):
    """Algorithm 1: returns (N_tilde, best_cost, [(N, cost) for every N evaluated, in order])."""
    xhat = np.ascontiguousarray(xhat, dtype=np.uint8).ravel()
    n_best = C.c_uint64()
    best = C.c_double()
    cand_n = np.zeros(cap, dtype=np.uint64)
    cand_c = np.zeros(cap, dtype=np.float64)
    n_cand = C.c_uint32()
    _check(lib().orc_search_reshape(_ptr(xhat), C.c_uint64(xhat.size), C.c_uint32(q_bits), C.byref(n_best),
                                    C.byref(best), _ptr(cand_n), _ptr(cand_c), C.c_uint32(cap), C.byref(n_cand)))
    k = min(n_cand.value, cap)
    return n_best.value, best.value, list(zip(cand_n[:k].tolist(), cand_c[:k].tolist()))
