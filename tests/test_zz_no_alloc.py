"""rans_compress_noalloc (the entry point for callers that cannot allocate: its workspace is a device array of
the library itself) against rans_compress and the oracle, through the C ABI.  Two calls in a row share the
array, the second with a smaller input; sizes beyond the array are refused."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_11664_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def _oparams(p):
    return oracle.make_params(p.q_bits, p.freq_bits, p.rows, p.cols, p.mode, p.n_streams, p.chunk_syms, p.in_dtype)


def _one(w):
    x_cpu = synth.make(w)
    p = B.params_of(w)
    n = w.numel
    print(f"[case] noalloc {w.name} n={n} mode={w.mode} K={w.cols} S={w.n_streams} cs={w.chunk_syms}", flush=True)
    x = x_cpu.cuda()
    codec = B.Codec(p, n)                       # buffers of the existing entry point (its own workspace)
    nb_ref = codec.compress(x)
    ref = codec.stream[:nb_ref].clone()
    out = torch.full_like(codec.stream, 0x5A)
    nbytes = torch.zeros(1, dtype=torch.int64, device="cuda")
    rc, ws_addr = B.rans_compress_noalloc(x, n, p, out, nbytes)
    assert rc == 0 and ws_addr and ws_addr % 256 == 0
    assert B.rans_last_status(ws_addr) == 0
    assert int(nbytes.item()) == nb_ref
    assert torch.equal(out[:nb_ref], ref), "bytes differ from rans_compress"
    want, _ = oracle.compress(x_cpu.numpy(), _oparams(p))
    assert bytes(out[:nb_ref].cpu().numpy()) == want, "bytes differ from the oracle"
    return ws_addr


def test_noalloc_matches_the_workspace_entry_point_on_consecutive_calls():
    a1 = _one(synth.workload("c1", 1, cols=7, chunk_syms=2048))          # CSR, 200 704 elements
    a2 = _one(synth.workload("t1", 1))                                   # smaller, DENSE
    a3 = _one(synth.workload("t1", 2, mode=1, cols=4))                   # smaller again, CSR
    a4 = _one(synth.workload("c1", 1, mode=0, chunk_syms=2048))          # larger again
    assert a1 == a2 == a3 == a4                                          # the one array of this GPU


def test_noalloc_errors():
    w = synth.workload("t1", 1)
    p = B.params_of(w)
    x = synth.make(w).cuda()
    out = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    nbytes = torch.zeros(1, dtype=torch.int64, device="cuda")
    # beyond the array: refused on the host, nothing launched
    big = 1 << 24
    pb = B.make_params(8, 12, big, 1, B.MODE_DENSE, 1024, 1 << 18, B.F32)
    rc, need, _ = B.rans_workspace_bytes(pb, big)
    assert rc == 0 and need > B.NOALLOC_WS_BYTES
    rc, _ = B.rans_compress_noalloc(x, big, pb, out, nbytes)
    assert rc == B.ERR_WORKSPACE
    # a data error is reported through the array's status word and as a size of 0; the next call is clean
    xb = x.clone()
    xb[17] = float("inf")
    rc, ws_addr = B.rans_compress_noalloc(xb, w.numel, p, out, nbytes)
    assert rc == 0 and B.rans_last_status(ws_addr) == B.ERR_NONFINITE and int(nbytes.item()) == 0
    rc, ws_addr = B.rans_compress_noalloc(x, w.numel, p, out, nbytes)
    assert rc == 0 and B.rans_last_status(ws_addr) == 0 and int(nbytes.item()) > 0
    # argument errors as in rans_compress
    rc, _ = B.rans_compress_noalloc(x, w.numel, p, out[1:], nbytes)
    assert rc == B.ERR_ARG
