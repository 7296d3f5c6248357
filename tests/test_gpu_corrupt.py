"""Corrupt containers on the GPU decoder: every mutation must end in RANS_ERR_CORRUPT or in a clean
decode, never in an out-of-bounds access.  The kernels bounds-check every size and offset they read."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_11664_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("mode,cols,M,S,cs", [
    (0, 1, 11, 16, 512),
    (1, 6, 11, 16, 512),
    (0, 1, 14, 1024, 4096),   # two chunks of 1024 streams at M = 14: groups of 512 lanes, per-slot table
    (1, 6, 12, 600, 2400),    # groups of 256 lanes, the last one ragged
])
def test_mutated_containers_are_rejected_or_decode_cleanly(mode, cols, M, S, cs):
    rng = np.random.default_rng(9)
    n = 6000
    x = np.maximum(rng.standard_normal(n), 0).astype(np.float32)
    op = oracle.make_params(8, M, n // cols, cols, mode, S, cs, 0)
    buf, sym_ref = oracle.compress(x, op)
    p = B.make_params(8, M, n // cols, cols, mode, S, cs, B.F32)
    codec = B.Codec(p, n)
    out = torch.empty(n, dtype=torch.uint8, device="cuda")
    n_bad = n_ok = 0
    for trial in range(120):
        b = bytearray(buf)
        kind = trial % 3
        if kind == 0:
            b[rng.integers(0, len(b))] ^= 1 << int(rng.integers(0, 8))
        elif kind == 1:
            b = b[:max(129, int(rng.integers(0, len(b))))]
        else:
            pos = int(rng.integers(128, len(b)))
            b[pos:pos + 4] = rng.integers(0, 256, len(b[pos:pos + 4]), dtype=np.uint8).tobytes()
        print(f"[corrupt] mode={mode} trial={trial} kind={kind} len={len(b)}", flush=True)
        try:
            oracle_ok = True
            oracle.decompress(bytes(b))
        except oracle.OracleError:
            oracle_ok = False
        codec.stream[:len(b)].copy_(torch.frombuffer(bytes(b), dtype=torch.uint8))
        rc, hdr_m = B.rans_peek_header(bytes(b[:128]))       # what a receiver would do with these bytes
        if rc == 0:
            rc = B.rans_decode(codec.stream, len(b), hdr_m, out, None, codec.ws)
        st = B.rans_last_status(codec.ws) if rc == 0 else rc
        assert st in (0, B.ERR_CORRUPT, B.ERR_WORKSPACE, B.ERR_CAPACITY)
        assert (st == 0) == oracle_ok, f"oracle_ok={oracle_ok} gpu status={st}"
        n_bad += st != 0
        n_ok += st == 0
    assert n_bad > 60
