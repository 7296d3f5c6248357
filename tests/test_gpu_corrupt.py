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


def _mutations(v, c, r, K, Q, A, rng):
    """(name, v, c, r) variants of a valid modified CSR: each keeps the lengths (so l_D and the container geometry
    stay valid) and breaks, or merely changes, the structure that the expand step must check (Sec. 3.1)."""
    nnz, N = v.size, r.size
    ends = np.cumsum(r.astype(np.int64))
    starts = ends - r
    long_rows = np.nonzero(r >= 2)[0]
    out = []

    def variant(name, fn):
        vv, cc, rr = v.copy(), c.copy(), r.copy()
        if fn(vv, cc, rr) is not False:
            out.append((name, vv, cc, rr))

    for pick in range(3):
        if long_rows.size:
            i = int(long_rows[rng.integers(0, long_rows.size)])
            j = int(starts[i] + rng.integers(0, r[i] - 1))

            def swap(vv, cc, rr, j=j):
                cc[j], cc[j + 1] = cc[j + 1], cc[j]
            variant(f"columns swapped inside row {i}", swap)

            def equal(vv, cc, rr, j=j):
                cc[j + 1] = cc[j]
            variant(f"equal columns inside row {i}", equal)
        j = int(rng.integers(0, nnz))

        def zero_value(vv, cc, rr, j=j):
            vv[j] = 0
        variant(f"stored zero at {j}", zero_value)
        if (1 << Q) < A:
            def big_value(vv, cc, rr, j=j):
                vv[j] = 1 << Q
            variant(f"value 2^Q at {j}", big_value)
        if K < A:
            def big_col(vv, cc, rr, j=j):
                cc[j] = K
            variant(f"column K at {j}", big_col)
        i = int(rng.integers(0, N - 1))

        def one_more(vv, cc, rr, i=i):
            rr[i] += 1
        variant(f"row {i} one longer, sum of r off by one", one_more)

        def shift_down(vv, cc, rr, i=i):  # the last nonzero of row i becomes the first of row i + 1
            if rr[i] == 0:
                return False
            rr[i] -= 1
            rr[i + 1] += 1
        variant(f"nonzero moved from row {i} to row {i + 1}", shift_down)

        def shift_up(vv, cc, rr, i=i):    # the first nonzero of row i + 1 becomes the last of row i
            if rr[i + 1] == 0:
                return False
            rr[i] += 1
            rr[i + 1] -= 1
        variant(f"nonzero moved from row {i + 1} to row {i}", shift_up)
        if K + 1 < A:
            def too_long(vv, cc, rr, i=i):  # r[i] > K, the sum kept by the rows around it
                need = K + 1 - int(rr[i])
                for i2 in list(range(i + 1, N)) + list(range(0, i)):
                    take = min(need, int(rr[i2]))
                    rr[i2] -= take
                    need -= take
                    if need == 0:
                        break
                if need:
                    return False
                rr[i] = K + 1
            variant(f"row {i} with K + 1 nonzeros", too_long)
    # changes that leave a valid structure: a different matrix must come out, the same on both sides
    into_empty = np.nonzero((r[:-1] >= 1) & (r[1:] == 0))[0]
    for i in into_empty[:2]:
        def down(vv, cc, rr, i=int(i)):
            rr[i] -= 1
            rr[i + 1] += 1
        variant(f"last nonzero of row {int(i)} moved into the empty row behind it", down)
    from_next = np.nonzero((r[:-1] == 0) & (r[1:] >= 1))[0]
    for i in from_next[:2]:
        def up(vv, cc, rr, i=int(i)):
            rr[i] += 1
            rr[i + 1] -= 1
        variant(f"first nonzero of row {int(i) + 1} moved into the empty row before it", up)
    last_of_row = ends[r >= 1] - 1
    for j in last_of_row[:: max(1, last_of_row.size // 3)][:3]:
        def nudge(vv, cc, rr, j=int(j)):
            if cc[j] + 1 >= K:
                return False
            cc[j] += 1
        variant(f"last column of a row raised by one at {int(j)}", nudge)
    return out


@pytest.mark.parametrize("N,K,Q,S,cs", [
    (5000, 4, 8, 32, 4096),      # more rows than lanes in a tile of the expand kernel
    (3000, 7, 6, 64, 0),
    (40, 300, 8, 32, 2048),      # long rows, K + 1 above 2^Q
    (700, 16, 4, 16, 1024),
    (3, 9000, 8, 64, 0),         # one row per tile, several steps of nonzeros per lane
])
def test_crafted_csr_structures_are_judged_like_the_oracle(N, K, Q, S, cs):
    """Valid rANS containers around a D whose CSR structure was altered by hand: the decision (reject, or decode)
    and, where it decodes, every symbol must be the oracle's."""
    rng = np.random.default_rng(N * 31 + K)
    n = N * K
    x = np.maximum(rng.standard_normal(n) - 0.3, 0).astype(np.float32)
    xhat, qi = oracle.quantize(x, Q)
    op = oracle.make_params(Q, 13, N, K, oracle.MODE_CSR, S, cs, 0)
    v, c, r = oracle.csr(xhat, N, K)
    A = oracle.alphabet(oracle.MODE_CSR, Q, K)
    p = B.make_params(Q, 13, N, K, B.MODE_CSR, S, cs, B.F32)
    codec = B.Codec(p, n)
    out = torch.empty(n, dtype=torch.uint8, device="cuda")
    n_rejected = n_decoded = 0
    cases = [("unchanged", v, c, r)] + _mutations(v, c, r, K, Q, A, rng)
    for name, vv, cc, rr in cases:
        print(f"[crafted] N={N} K={K} {name}", flush=True)
        D = np.concatenate([vv, cc, rr]).astype(np.uint16)
        buf = oracle.encode_container(D, op, n, float(x.min()), float(x.max()))
        try:
            sym_ref, _, _ = oracle.decompress(buf)
        except oracle.OracleError:
            sym_ref = None
        codec.stream[:len(buf)].copy_(torch.frombuffer(bytearray(buf), dtype=torch.uint8))
        rc, hdr = B.rans_peek_header(buf[:128])
        assert rc == 0
        rc = B.rans_decode(codec.stream, len(buf), hdr, out, None, codec.ws)
        st = B.rans_last_status(codec.ws) if rc == 0 else rc
        assert st in (0, B.ERR_CORRUPT), name
        assert (st == 0) == (sym_ref is not None), f"{name}: oracle accepts={sym_ref is not None}, gpu status={st}"
        if st == 0:
            assert np.array_equal(out.cpu().numpy(), sym_ref), name
            n_decoded += 1
        else:
            n_rejected += 1
    assert n_decoded >= 2 and n_rejected >= 6
