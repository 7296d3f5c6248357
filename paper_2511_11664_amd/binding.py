"""ctypes binding of ``librans_if.so`` (include/rans_if.h): argument marshalling only.

Every function here has the name and argument order of its C counterpart and
passes ``tensor.data_ptr()`` / the current HIP stream through; all computation
happens in the library's kernels.  There is no fallback: if the shared library
is missing or fails to load, ``lib()`` raises.

``Codec`` is a convenience holder for the buffers one (params, n_elems) pair
needs (workspace, container, size word); it allocates with torch and calls the
same entry points.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import torch

_DIR = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_DIR)
SO_PATH = os.path.join(_DIR, "librans_if.so")
SRC_PATH = os.path.join(_DIR, "csrc", "rans_if.hip")
INC_DIR = os.path.join(_ROOT, "include")

OK, ERR_ARG, ERR_SHAPE, ERR_ALPHABET, ERR_CAPACITY, ERR_WORKSPACE, ERR_NONFINITE, ERR_CORRUPT, ERR_HIP = (
    0, -1, -2, -3, -4, -5, -6, -7, -8)
MODE_DENSE, MODE_CSR = 0, 1
F32, F16 = 0, 1

HIPCC_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-ffp-contract=off",
               "-fhip-fp32-correctly-rounded-divide-sqrt",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose: bool = False) -> str:
    """Compile csrc/rans_if.hip for gfx950 into librans_if.so (in-tree)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", INC_DIR, "-shared", "-fPIC", "-o", SO_PATH, SRC_PATH]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout, res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building librans_if.so")
    return SO_PATH


class Params(C.Structure):
    _fields_ = [("q_bits", C.c_uint32), ("freq_bits", C.c_uint32), ("rows", C.c_uint64),
                ("cols", C.c_uint64), ("mode", C.c_uint32), ("n_streams", C.c_uint32),
                ("chunk_syms", C.c_uint32), ("in_dtype", C.c_uint32)]


class QInfo(C.Structure):
    _fields_ = [("x_min", C.c_float), ("x_max", C.c_float), ("scale", C.c_float),
                ("zero_point", C.c_float)]


RESHAPE_MAX_CAND = 128


class ReshapeResult(C.Structure):
    _fields_ = [("rows", C.c_uint64), ("cols", C.c_uint64), ("cost_bits", C.c_double),
                ("n_evaluated", C.c_uint32), ("n_candidates", C.c_uint32),
                ("cand_rows", C.c_uint64 * RESHAPE_MAX_CAND), ("cand_cost", C.c_double * RESHAPE_MAX_CAND)]


class Header(C.Structure):
    _fields_ = [("p", Params), ("n_elems", C.c_uint64), ("len_d", C.c_uint64),
                ("alphabet", C.c_uint32), ("n_chunks", C.c_uint32),
                ("x_min", C.c_float), ("x_max", C.c_float)]


NOALLOC_WS_BYTES = 32 << 20

EXPORTS = ("rans_workspace_bytes", "rans_quantize", "rans_encode", "rans_decode", "rans_dequantize",
           "rans_compress", "rans_compress_noalloc", "rans_decompress", "rans_peek_header", "rans_last_status",
           "rans_search_workspace_bytes", "rans_search_reshape", "rans_selftest_divide",
           "rans_profile_enable", "rans_profile_reset", "rans_profile_read",
           "rans_strerror", "rans_profile_kernel_name")

_lib = None


def lib() -> C.CDLL:
    """Load the shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(SO_PATH):
            raise RuntimeError(f"{SO_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(SO_PATH)
        vp, u64, sz, u32 = C.c_void_p, C.c_uint64, C.c_size_t, C.c_uint32
        PP, HP = C.POINTER(Params), C.POINTER(Header)
        L.rans_workspace_bytes.argtypes = [PP, u64, C.POINTER(sz), C.POINTER(sz)]
        L.rans_quantize.argtypes = [vp, u64, PP, vp, vp, vp, sz, vp]
        L.rans_encode.argtypes = [vp, u64, PP, vp, vp, sz, vp, vp, sz, vp]
        L.rans_decode.argtypes = [vp, sz, HP, vp, u64, vp, vp, sz, vp]
        L.rans_dequantize.argtypes = [vp, u64, vp, u32, vp, vp]
        L.rans_compress.argtypes = [vp, u64, PP, vp, sz, vp, vp, sz, vp]
        L.rans_compress_noalloc.argtypes = [vp, u64, PP, vp, sz, vp, C.POINTER(vp), vp]
        L.rans_decompress.argtypes = [vp, sz, HP, u32, vp, u64, vp, sz, vp]
        L.rans_peek_header.argtypes = [vp, sz, HP]
        L.rans_last_status.argtypes = [vp, vp]
        L.rans_search_workspace_bytes.argtypes = [u64, u32, C.POINTER(sz)]
        L.rans_search_reshape.argtypes = [vp, u64, u32, vp, vp, sz, vp]
        L.rans_selftest_divide.argtypes = [vp, u64, vp]
        L.rans_strerror.argtypes = [C.c_int]
        L.rans_strerror.restype = C.c_char_p
        L.rans_profile_enable.argtypes = [u64, u32]
        L.rans_profile_reset.argtypes = []
        L.rans_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(u64)]
        L.rans_profile_kernel_name.argtypes = [C.c_int]
        L.rans_profile_kernel_name.restype = C.c_char_p
        for name in EXPORTS[:-2]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


class RansError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"rans_if error {code}: {lib().rans_strerror(code).decode()}")
        self.code = code


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _p(t):
    """Device pointer of a tensor (None -> NULL); a plain integer is taken as an address."""
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr() if t is not None else 0)


def make_params(q_bits, freq_bits, rows, cols, mode, n_streams, chunk_syms, in_dtype) -> Params:
    return Params(q_bits, freq_bits, rows, cols, mode, n_streams, chunk_syms, in_dtype)


def params_of(w) -> Params:
    """Params of a synth.Workload."""
    return Params(w.q_bits, w.freq_bits, w.rows, w.cols, w.mode, w.n_streams, w.chunk_syms, w.in_dtype)


# ------------------------------------------------------------------ raw entry points

def rans_workspace_bytes(p: Params, n_elems: int):
    ws, mx = C.c_size_t(), C.c_size_t()
    rc = lib().rans_workspace_bytes(C.byref(p), n_elems, C.byref(ws), C.byref(mx))
    return rc, ws.value, mx.value


def rans_quantize(d_x, n_elems, p, d_sym, d_qinfo, d_ws) -> int:
    return lib().rans_quantize(_p(d_x), n_elems, C.byref(p), _p(d_sym), _p(d_qinfo), _p(d_ws),
                               d_ws.numel() * d_ws.element_size(), _stream())


def rans_encode(d_sym, n_elems, p, d_qinfo, d_stream, d_stream_bytes, d_ws) -> int:
    return lib().rans_encode(_p(d_sym), n_elems, C.byref(p), _p(d_qinfo), _p(d_stream), d_stream.numel(),
                             _p(d_stream_bytes), _p(d_ws), d_ws.numel() * d_ws.element_size(), _stream())


def rans_decode(d_stream, stream_bytes, hdr, d_sym, d_qinfo, d_ws) -> int:
    return lib().rans_decode(_p(d_stream), stream_bytes, C.byref(hdr) if hdr is not None else None, _p(d_sym),
                             d_sym.numel() if d_sym is not None else 0, _p(d_qinfo), _p(d_ws),
                             d_ws.numel() * d_ws.element_size(), _stream())


def rans_dequantize(d_sym, n_elems, d_qinfo, out_dtype, d_x_out) -> int:
    return lib().rans_dequantize(_p(d_sym), n_elems, _p(d_qinfo), out_dtype, _p(d_x_out), _stream())


def rans_compress(d_x, n_elems, p, d_stream, d_stream_bytes, d_ws) -> int:
    return lib().rans_compress(_p(d_x), n_elems, C.byref(p), _p(d_stream), d_stream.numel(), _p(d_stream_bytes),
                               _p(d_ws), d_ws.numel() * d_ws.element_size(), _stream())


def rans_compress_noalloc(d_x, n_elems, p, d_stream, d_stream_bytes):
    """-> (rc, device address of the library's own workspace, for rans_last_status)."""
    ws = C.c_void_p()
    rc = lib().rans_compress_noalloc(_p(d_x), n_elems, C.byref(p), _p(d_stream), d_stream.numel(), _p(d_stream_bytes),
                                     C.byref(ws), _stream())
    return rc, ws.value


def rans_decompress(d_stream, stream_bytes, hdr, out_dtype, d_x_out, d_ws) -> int:
    return lib().rans_decompress(_p(d_stream), stream_bytes, C.byref(hdr) if hdr is not None else None, out_dtype,
                                 _p(d_x_out), d_x_out.numel() if d_x_out is not None else 0, _p(d_ws),
                                 d_ws.numel() * d_ws.element_size(), _stream())


def rans_peek_header(h_bytes: bytes):
    hdr = Header()
    buf = (C.c_uint8 * len(h_bytes)).from_buffer_copy(h_bytes)
    rc = lib().rans_peek_header(C.cast(buf, C.c_void_p), len(h_bytes), C.byref(hdr))
    return rc, hdr


def rans_last_status(d_ws) -> int:
    return lib().rans_last_status(_p(d_ws), _stream())


def rans_selftest_divide(d_mismatches, n_random: int) -> int:
    """d_mismatches: a device tensor of one 32-bit word."""
    return lib().rans_selftest_divide(_p(d_mismatches), n_random, _stream())


def rans_search_workspace_bytes(n_elems: int, q_bits: int):
    ws = C.c_size_t()
    rc = lib().rans_search_workspace_bytes(n_elems, q_bits, C.byref(ws))
    return rc, ws.value


def rans_search_reshape(d_sym, n_elems, q_bits, d_result, d_ws) -> int:
    """d_result: a device byte tensor of at least sizeof(ReshapeResult) bytes."""
    return lib().rans_search_reshape(_p(d_sym), n_elems, q_bits, _p(d_result), _p(d_ws),
                                     d_ws.numel() * d_ws.element_size(), _stream())


def search_reshape(d_sym, q_bits: int) -> ReshapeResult:
    """Algorithm 1 on a device tensor of quantised symbols; allocates its workspace, synchronises, returns the result."""
    import torch
    n = d_sym.numel()
    rc, ws_bytes = rans_search_workspace_bytes(n, q_bits)
    if rc:
        raise RansError(rc)
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=d_sym.device)
    off = (-ws.data_ptr()) % 256
    ws = ws[off:off + ws_bytes]
    res = torch.zeros(C.sizeof(ReshapeResult), dtype=torch.uint8, device=d_sym.device)
    rc = rans_search_reshape(d_sym, n, q_bits, res, ws)
    if rc:
        raise RansError(rc)
    host = res.cpu().numpy().tobytes()
    return ReshapeResult.from_buffer_copy(host)


def rans_strerror(code: int) -> str:
    return lib().rans_strerror(code).decode()


def profile_kernel_names():
    names, i = [], 0
    while True:
        nm = lib().rans_profile_kernel_name(i)
        if nm is None:
            return names
        names.append(nm.decode())
        i += 1


def rans_profile_enable(kernels="all", every: int = 1) -> int:
    """kernels: "all", an iterable of kernel names, or a falsy value to switch recording off.
    every: bracket only every n-th launch of each enabled kernel."""
    if not kernels:
        return lib().rans_profile_enable(0, 1)
    names = profile_kernel_names()
    mask = (1 << len(names)) - 1 if kernels == "all" else sum(1 << names.index(k) for k in kernels)
    return lib().rans_profile_enable(mask, every)


def rans_profile_reset() -> int:
    return lib().rans_profile_reset()


def rans_profile_read() -> dict:
    """{kernel name: {"total_ms": float, "count": int}} for kernels with at least one record (synchronises)."""
    out = {}
    for i, nm in enumerate(profile_kernel_names()):
        ms, cnt = C.c_double(), C.c_uint64()
        rc = lib().rans_profile_read(i, C.byref(ms), C.byref(cnt))
        if rc:
            raise RansError(rc)
        if cnt.value:
            out[nm] = {"total_ms": ms.value, "count": cnt.value}
    return out


# ------------------------------------------------------------------ buffer holder

class Codec:
    """Buffers for one (params, n_elems): workspace, container, size word, qinfo."""

    def __init__(self, p: Params, n_elems: int, device="cuda:0"):
        self.p, self.n = p, n_elems
        rc, ws, mx = rans_workspace_bytes(p, n_elems)
        if rc:
            raise RansError(rc)
        self.device = torch.device(device)
        self.ws = torch.empty(ws + 256, dtype=torch.uint8, device=self.device)
        self.stream = torch.empty(mx + 16, dtype=torch.uint8, device=self.device)
        self.nbytes = torch.zeros(1, dtype=torch.int64, device=self.device)
        self.qinfo = torch.zeros(4, dtype=torch.float32, device=self.device)

    def _check(self, rc, sync=True):
        if rc:
            raise RansError(rc)
        if sync:
            st = rans_last_status(self.ws)
            if st:
                raise RansError(st)

    def compress(self, x: torch.Tensor, check=True) -> int:
        """tensor -> container in self.stream; returns its size in bytes (synchronises if check)."""
        self._check(rans_compress(x, self.n, self.p, self.stream, self.nbytes, self.ws), check)
        return int(self.nbytes.item()) if check else -1

    def quantize(self, x, sym, check=True):
        self._check(rans_quantize(x, self.n, self.p, sym, self.qinfo, self.ws), check)

    def encode(self, sym, check=True) -> int:
        self._check(rans_encode(sym, self.n, self.p, self.qinfo, self.stream, self.nbytes, self.ws), check)
        return int(self.nbytes.item()) if check else -1

    def header(self, nbytes: int) -> Header:
        rc, h = rans_peek_header(bytes(self.stream[:128].cpu().numpy()))
        if rc:
            raise RansError(rc)
        return h

    def decode(self, nbytes, hdr, sym, check=True):
        self._check(rans_decode(self.stream, nbytes, hdr, sym, self.qinfo, self.ws), check)

    def decompress(self, nbytes, hdr, out, check=True):
        dt = F16 if out.dtype == torch.float16 else F32
        self._check(rans_decompress(self.stream, nbytes, hdr, dt, out, self.ws), check)

    def container(self, nbytes: int) -> bytes:
        return bytes(self.stream[:nbytes].cpu().numpy())


def compress_with_search(x: torch.Tensor, q_bits: int, freq_bits: int, n_streams: int, chunk_syms: int):
    """The paper's whole edge side (Fig. 1(c) with the reshape of Algorithm 1): quantise, search the reshape
    N~ on the quantised symbols, then code D = v (+) c (+) r for [N~, T / N~].  The search result has to come
    back to the host, because rows and cols are host-side parameters of the encoder.
    Returns (container bytes as a device tensor view, Params used, ReshapeResult)."""
    n = x.numel()
    in_dtype = F16 if x.dtype == torch.float16 else F32
    # any valid reshape serves for the quantise step (Eq. 6 does not depend on it)
    pq = make_params(q_bits, freq_bits, n, 1, MODE_DENSE, n_streams, chunk_syms, in_dtype)
    cq = Codec(pq, n, x.device)
    sym = torch.empty(n, dtype=torch.uint8, device=x.device)
    cq.quantize(x.reshape(-1), sym)
    res = search_reshape(sym, q_bits)
    p = make_params(q_bits, freq_bits, res.rows, res.cols, MODE_CSR, n_streams, chunk_syms, in_dtype)
    ce = Codec(p, n, x.device)
    ce.qinfo.copy_(cq.qinfo)
    nbytes = ce.encode(sym)
    return ce.stream[:nbytes], p, res
