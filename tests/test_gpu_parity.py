"""GPU library vs CPU oracle, element by element, through the C ABI.  Needs an MI355X (-m gpu).

Bar: quantised symbols, quantiser parameters, container bytes and decoded symbols bit-exact;
dequantised floats within 1 ulp (they are expected to be bit-identical: same binary32 operations,
no FMA contraction on either side).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_11664_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def _oparams(p):
    return oracle.make_params(p.q_bits, p.freq_bits, p.rows, p.cols, p.mode, p.n_streams, p.chunk_syms, p.in_dtype)


def _ulp_diff(a, b):
    if a.dtype == np.float32:
        ia, ib = a.view(np.int32).astype(np.int64), b.view(np.int32).astype(np.int64)
    else:
        ia, ib = a.view(np.int16).astype(np.int64), b.view(np.int16).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7fffffff if a.dtype == np.float32 else ia & 0x7fff), ia)
    ib = np.where(ib < 0, -(ib & 0x7fffffff if a.dtype == np.float32 else ib & 0x7fff), ib)
    return np.abs(ia - ib).max(initial=0)


def _check_all(x_cpu: torch.Tensor, p: B.Params, tag=""):
    """Fused and unfused paths against the oracle for one tensor."""
    print(f"[case] {tag} n={x_cpu.numel()} dtype={x_cpu.dtype} Q={p.q_bits} M={p.freq_bits} N={p.rows} K={p.cols} "
          f"mode={p.mode} S={p.n_streams} cs={p.chunk_syms}", flush=True)
    n = x_cpu.numel()
    xn = x_cpu.numpy()
    ref, sym_ref = oracle.compress(xn, _oparams(p))
    _, qi_ref = oracle.quantize(xn, p.q_bits)
    codec = B.Codec(p, n)
    xd = x_cpu.cuda()
    # fused
    nbytes = codec.compress(xd)
    got = codec.container(nbytes)
    assert nbytes == len(ref), f"container size {nbytes} != oracle {len(ref)}"
    assert got == ref, "container bytes differ"
    # unfused: quantize -> encode
    sym = torch.empty(max(n, 1), dtype=torch.uint8, device="cuda")
    codec.quantize(xd, sym)
    assert np.array_equal(sym[:n].cpu().numpy(), sym_ref), "quantised symbols differ"
    q = codec.qinfo.cpu().numpy()
    assert np.array_equal(q.view(np.uint32), np.array(qi_ref.as_tuple(), np.float32).view(np.uint32)), "qinfo differs"
    nb2 = codec.encode(sym)
    assert codec.container(nb2) == ref, "rans_encode bytes differ from rans_compress"
    # decode (with header hint, and letting the library read the header)
    hdr = codec.header(nbytes)
    for h in (hdr, None):
        out_sym = torch.full((max(n, 1),), 0xAB, dtype=torch.uint8, device="cuda")
        codec.qinfo.zero_()
        codec.decode(nbytes, h, out_sym)
        assert np.array_equal(out_sym[:n].cpu().numpy(), sym_ref), "decoded symbols differ"
        assert np.array_equal(codec.qinfo.cpu().numpy().view(np.uint32), q.view(np.uint32))
    # decompress + dequantize
    for dt, code in ((torch.float32, oracle.F32), (torch.float16, oracle.F16)):
        y_ref = oracle.dequantize(sym_ref, qi_ref, code)
        out = torch.empty(max(n, 1), dtype=dt, device="cuda")
        codec.decompress(nbytes, hdr, out)
        y = out[:n].cpu().numpy()
        assert _ulp_diff(y, y_ref) <= 1
        assert np.array_equal(y.view(np.uint8), y_ref.view(np.uint8)), "dequantised floats not bit-identical"
        out2 = torch.empty(max(n, 1), dtype=dt, device="cuda")
        rc = B.rans_dequantize(sym, n, codec.qinfo, code, out2)
        assert rc == 0
        assert np.array_equal(out2[:n].cpu().numpy().view(np.uint8), y_ref.view(np.uint8))
    return nbytes


def _relu_normal(n, seed, dtype=torch.float32, shift=0.0, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.relu(torch.randn(n, generator=g) + shift) * scale).to(dtype)


def _normal(n, seed, dtype=torch.float32, mean=0.3, std=2.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(n, generator=g) * std + mean).to(dtype)


DENSE_CASES = [
    # n, dtype, Q, M, S, cs
    (1, torch.float32, 8, 12, 1, 0),
    (7, torch.float32, 8, 12, 32, 0),
    (1000, torch.float32, 8, 12, 32, 0),
    (4099, torch.float32, 8, 12, 32, 64),
    (65536 + 13, torch.float32, 8, 12, 64, 1024),
    (100003, torch.float16, 8, 14, 1024, 4096),
    (300000, torch.float16, 8, 14, 1024, 1 << 16),
    (50001, torch.float32, 6, 14, 256, 2560),
    (50001, torch.float32, 4, 10, 300, 600),
    (50001, torch.float16, 2, 8, 5, 50),
    (50001, torch.float32, 1, 1, 64, 0),
    (20000, torch.float32, 3, 15, 64, 6400),
    (50001, torch.float32, 8, 8, 64, 640),
    # more encoder work-groups than the chip holds at once (their placement waits on lower-numbered ones)
    (1000003, torch.float32, 8, 12, 64, 128),
    (2000003, torch.float16, 8, 14, 1024, 1024),
    # more work-groups than the encoder places itself: separate size scan and gather kernels
    (1200007, torch.float32, 8, 12, 32, 64),
    # few chunks of many streams: the decoder splits a chunk over groups of 512 (M = 14) or 256 lanes, the last
    # group ragged
    (200003, torch.float16, 8, 14, 600, 600 * 64),
    (200003, torch.float32, 8, 12, 1000, 1000 * 40),
    (150001, torch.float32, 7, 13, 777, 0),
]


@pytest.mark.parametrize("n,dtype,Q,M,S,cs", DENSE_CASES)
def test_dense_parity(n, dtype, Q, M, S, cs):
    for seed, x in ((0, _relu_normal(n, n, dtype)), (1, _normal(n, n + 1, dtype))):
        p = B.make_params(Q, M, n, 1, B.MODE_DENSE, S, cs, B.F16 if dtype == torch.float16 else B.F32)
        _check_all(x, p, f"dense seed={seed}")


CSR_CASES = [
    # rows, cols, dtype, Q, M, S, cs
    (1, 1, torch.float32, 8, 12, 1, 0),
    (3, 5, torch.float32, 8, 12, 4, 0),
    (64, 7, torch.float32, 8, 12, 32, 0),
    (1000, 7, torch.float32, 8, 12, 32, 320),
    (997, 13, torch.float16, 8, 12, 64, 1024),
    (300, 256, torch.float32, 8, 12, 1024, 8192),
    (4096 + 5, 16, torch.float32, 4, 10, 256, 2048),
    (64, 3136, torch.float32, 8, 12, 32, 0),
    (17, 9000, torch.float32, 6, 15, 128, 12800),
    (40000, 1, torch.float32, 8, 12, 64, 640),
    (2, 65535, torch.float32, 8, 15, 64, 0),
    (200000, 5, torch.float32, 8, 12, 64, 256),
    # the coder's LDS staging of D with an 8-byte-entry table (alphabet between 1024 and 8192), and one chunk of
    # thousands of rows (many 16-row tiles, ragged first tile, all three parts of D inside one chunk)
    (50, 3000, torch.float32, 8, 13, 64, 640),
    (3000, 64, torch.float16, 8, 12, 64, 0),
    (3000, 64, torch.float32, 6, 12, 128, 128 * 200),
    # few chunks of many streams (ragged last group of the decoder), alphabet of 257 symbols at M = 14 and 12
    (2000, 256, torch.float16, 8, 14, 600, 600 * 100),
    (2000, 256, torch.float32, 8, 12, 1000, 0),
    # rows inside a lane's 16 symbols (K divides 16: the compaction kernel also makes the row counts), ragged ends
    (4099, 2, torch.float32, 8, 12, 64, 1024),
    (1237, 8, torch.float16, 8, 12, 32, 0),
    (20001, 4, torch.float32, 3, 11, 128, 4096),
    (333, 16, torch.float32, 8, 12, 64, 2048),
    # rows that start with a tile of 4096 symbols (K divides 4096, K >= 64): row counts from the tile's own prefix
    (37, 4096, torch.float32, 8, 13, 64, 4096),
    (5, 2048, torch.float16, 8, 12, 32, 0),
    (129, 128, torch.float32, 8, 12, 64, 1024),
]


@pytest.mark.parametrize("rows,cols,dtype,Q,M,S,cs", CSR_CASES)
def test_csr_parity(rows, cols, dtype, Q, M, S, cs):
    n = rows * cols
    if cols > 20000:      # keep the number of distinct column symbols below 2^M
        x = torch.zeros(n)
        g = torch.Generator().manual_seed(5)
        idx = torch.randperm(n, generator=g)[:3000]
        x[idx] = torch.rand(3000, generator=g) + 0.1
        xs = [x.to(dtype)]
    else:
        xs = [_relu_normal(n, n, dtype, shift=-0.5), _relu_normal(n, n + 1, dtype, shift=1.0)]
    for i, x in enumerate(xs):
        p = B.make_params(Q, M, rows, cols, B.MODE_CSR, S, cs, B.F16 if dtype == torch.float16 else B.F32)
        _check_all(x, p, f"csr case={i}")


def test_quantiser_matches_ieee_division_everywhere_it_takes_the_hoisted_reciprocal_path():
    """Symbols must equal the oracle's (which divides with the CPU's IEEE binary32 division) for every binary16
    value at several scales, and for wide random binary32 samples inside and outside the fast-path range."""
    halves = torch.arange(65536, dtype=torch.int32).to(torch.int16).view(torch.float16)
    halves = halves[torch.isfinite(halves)]
    cases = []
    for bound in (65504.0, 1000.0, 97.3, 7.25, 1.0, 0.11, 3e-3, 6.2e-5):
        x = halves[halves.abs().float() <= bound]
        cases.append((x.contiguous(), 8))
        cases.append((x[x >= 0].contiguous(), 5))
    g = torch.Generator().manual_seed(77)
    for scale in (1e-12, 1e-6, 1e-3, 1.0, 37.0, 1e4, 1e8, 3e12):
        x = torch.randn(1 << 20, generator=g) * scale
        cases.append((x, 8))
        bits = torch.randint(0, 1 << 31, (1 << 20,), generator=g, dtype=torch.int64).to(torch.int32)
        y = bits.view(torch.float32)
        y = torch.where(torch.isfinite(y) & (y.abs() < 1e30), y, torch.zeros_like(y)).clamp(-scale, scale)
        cases.append((y.contiguous(), 7))
    for x, Q in cases:
        n = x.numel()
        p = B.make_params(Q, 12, n, 1, B.MODE_DENSE, 32, 0, B.F16 if x.dtype == torch.float16 else B.F32)
        codec = B.Codec(p, n)
        sym = torch.empty(n, dtype=torch.uint8, device="cuda")
        codec.quantize(x.cuda(), sym)
        ref, qi = oracle.quantize(x.numpy(), Q)
        print(f"[case] quantiser n={n} dtype={x.dtype} Q={Q} scale={qi.scale}", flush=True)
        assert np.array_equal(sym.cpu().numpy(), ref)


def test_unaligned_buffers():
    """Views that start at odd element offsets take the scalar load paths."""
    n = 30011
    base = _relu_normal(n + 3, 3)
    x = base[1:1 + n]
    p = B.make_params(8, 12, n, 1, B.MODE_DENSE, 32, 640, B.F32)
    ref, sym_ref = oracle.compress(x.numpy().copy(), _oparams(p))
    codec = B.Codec(p, n)
    xd = base.cuda()[1:1 + n]
    assert xd.data_ptr() % 16 != 0
    assert codec.container(codec.compress(xd)) == ref
    symbuf = torch.empty(n + 8, dtype=torch.uint8, device="cuda")
    sym = symbuf[3:3 + n]
    codec.quantize(xd, sym)
    assert np.array_equal(sym.cpu().numpy(), sym_ref)
    assert codec.container(codec.encode(sym)) == ref
    pc = B.make_params(8, 12, n // 7 if n % 7 == 0 else n, 7 if n % 7 == 0 else 1, B.MODE_CSR, 32, 640, B.F32)
    refc, _ = oracle.compress(x.numpy().copy(), _oparams(pc))
    cc = B.Codec(pc, n)
    cc.qinfo.copy_(codec.qinfo)
    assert cc.container(cc.encode(sym)) == refc
    assert cc.container(cc.compress(xd)) == refc  # CSR from the unaligned tensor: element-wise quantise path
    # fp16 tensor at an odd element offset, CSR with several tiles of symbols per work-group step
    n2 = 70001
    b16 = _relu_normal(n2 + 3, 4, torch.float16)
    x16 = b16[1:1 + n2]
    p16 = B.make_params(8, 12, n2, 1, B.MODE_CSR, 64, 1280, B.F16)
    ref16, _ = oracle.compress(x16.numpy().copy(), _oparams(p16))
    c16 = B.Codec(p16, n2)
    assert c16.container(c16.compress(b16.cuda()[1:1 + n2])) == ref16


def test_edge_cases():
    # empty tensor, both modes
    for mode in (B.MODE_DENSE, B.MODE_CSR):
        p = B.make_params(8, 12, 0, 4, mode, 32, 0, B.F32)
        _check_all(torch.zeros(0), p, "empty")
    # constant tensors (s = 0), negative zero, single element
    for mode in (B.MODE_DENSE, B.MODE_CSR):
        _check_all(torch.full((1000,), -2.5), B.make_params(8, 12, 250, 4, mode, 8, 16, B.F32), "constant")
        _check_all(torch.zeros(1000), B.make_params(8, 12, 250, 4, mode, 8, 16, B.F32), "zeros")
        x = torch.tensor([-0.0, 0.0, 1.0, 0.5] * 10)
        _check_all(x, B.make_params(8, 12, 10, 4, mode, 3, 6, B.F32), "negzero")
    # more streams than symbols; chunk of exactly S symbols
    _check_all(_relu_normal(10, 1), B.make_params(8, 12, 10, 1, 0, 64, 64, B.F32), "S>n")
    _check_all(_relu_normal(1000, 2), B.make_params(8, 12, 1000, 1, 0, 8, 8, B.F32), "cs=S")
    # tiny and huge magnitudes, denormals
    _check_all(_normal(5000, 3) * 1e-41, B.make_params(8, 12, 5000, 1, 0, 32, 0, B.F32), "denormal")
    _check_all(_normal(5000, 4) * 1e37, B.make_params(8, 12, 5000, 1, 0, 32, 0, B.F32), "huge")
    _check_all(_normal(5000, 5, mean=1e6, std=1.0), B.make_params(8, 12, 5000, 1, 0, 32, 0, B.F32), "offset")
    x16 = torch.tensor([6.0e-8, 65504.0, -65504.0, 1.0, 0.0] * 100, dtype=torch.float16)
    _check_all(x16, B.make_params(8, 12, 500, 1, 0, 32, 0, B.F16), "fp16 extremes")
    # normalisation with a deficit: 4096 distinct column symbols crowd a 2^12 table
    rows, cols = 64, 4090
    x = torch.zeros(rows * cols)
    g = torch.Generator().manual_seed(9)
    x[torch.randperm(rows * cols, generator=g)[:60000]] = 1.0
    _check_all(x, B.make_params(2, 12, rows, cols, B.MODE_CSR, 32, 0, B.F32), "deficit")


def _inexact_entries(container: bytes, A: int, M: int) -> int:
    """Symbols whose division-free multiplier (Eq. 2 as multiply-high and shift) is not exact for every state the
    coder can meet: computed from the stored frequency table, with the condition the table kernels state."""
    f = np.frombuffer(container[128:128 + 2 * A], dtype="<u2").astype(np.int64)
    bad = 0
    for fa in f:
        fa = int(fa)
        if fa < 2 or fa & (fa - 1) == 0:
            continue
        k = fa.bit_length() - 1
        two = 1 << (32 + k)
        e = (two // fa + 1) * fa - two
        bad += ((fa << (32 - M)) - 1) * e >= two
    return bad


def test_both_table_forms_and_the_alphabet_switches():
    """The encoder builds its table itself for alphabets up to 512 symbols (one wave up to 256, wave plus work-group
    above), k_normalize above that; a frequency table with a multiplier that is not exact makes the coder use its other
    table form.  Every combination has to give the oracle's bytes."""
    n = 60000
    forms = set()
    for seed, dens in ((1, 0.004), (2, 0.01), (3, 0.02), (4, 0.03), (5, 0.05), (6, 0.08)):
        g = torch.Generator().manual_seed(100 + seed)
        x = torch.relu(torch.randn(n, generator=g)) * (torch.rand(n, generator=g) < dens)
        p = B.make_params(8, 12, n, 1, B.MODE_DENSE, 64, 4096, B.F32)
        ref, _ = oracle.compress(x.numpy(), _oparams(p))
        forms.add((256, _inexact_entries(ref, 256, 12) > 0))
        _check_all(x, p, f"dominant symbol d={dens} A=256")
    # the same for a 301-symbol alphabet: 2000 rows of 300 columns, nearly all of them empty (r = 0 dominates D)
    N, K = 2000, 300
    for seed, dens in ((1, 0.0001), (3, 0.0001), (4, 0.0002), (5, 0.00005), (6, 0.0002)):
        g = torch.Generator().manual_seed(200 + seed)
        x = torch.relu(torch.randn(N * K, generator=g)) * (torch.rand(N * K, generator=g) < dens)
        p = B.make_params(8, 12, N, K, B.MODE_CSR, 64, 4096, B.F32)
        ref, _ = oracle.compress(x.numpy(), _oparams(p))
        forms.add((301, _inexact_entries(ref, 301, 12) > 0))
        _check_all(x, p, f"dominant symbol d={dens} A=301")
    assert {(256, True), (256, False), (301, True), (301, False)} <= forms, forms
    # alphabet sizes on both sides of the switches (CSR: A = K + 1 for K >= 2^Q)
    for K in (255, 256, 511, 512, 1023, 1024, 1500):
        rows = 40
        x = _relu_normal(rows * K, 7 + K)
        _check_all(x, B.make_params(8, 12, rows, K, B.MODE_CSR, 32, 2048, B.F32), f"alphabet {K + 1}")


def test_table_divisions_equal_integer_division():
    """The frequency-table kernels divide through a reciprocal estimate and an exact remainder check; on the device
    that runs them: every divisor of the encoder's multipliers (Eq. 2), and 2^24 quotients of the kind Sec. 3.2's
    normalisation takes, against integer division."""
    bad = torch.full((1,), 123, dtype=torch.int32, device="cuda")
    print("[case] division self-test", flush=True)
    assert B.rans_selftest_divide(bad, 1 << 24) == 0
    torch.cuda.synchronize()
    assert int(bad.item()) == 0


def test_data_errors():
    n = 4096
    p = B.make_params(8, 12, n, 1, B.MODE_DENSE, 32, 0, B.F32)
    codec = B.Codec(p, n)
    for bad in (float("nan"), float("inf"), float("-inf")):
        x = _relu_normal(n, 1)
        x[77] = bad
        with pytest.raises(B.RansError) as e:
            codec.compress(x.cuda())
        assert e.value.code == B.ERR_NONFINITE
        assert int(codec.nbytes.item()) == 0
    x = torch.tensor([-3e38, 3e38] * 2048)
    with pytest.raises(B.RansError) as e:
        codec.compress(x.cuda())
    assert e.value.code == B.ERR_NONFINITE
    # a good call afterwards works again
    x = _relu_normal(n, 2)
    ref, _ = oracle.compress(x.numpy(), _oparams(p))
    assert codec.container(codec.compress(x.cuda())) == ref
    # too many distinct symbols for 2^M
    p4 = B.make_params(8, 4, n, 1, B.MODE_DENSE, 32, 0, B.F32)
    c4 = B.Codec(p4, n)
    with pytest.raises(B.RansError) as e:
        c4.compress(x.cuda())
    assert e.value.code == B.ERR_ALPHABET
    # the literal "rows = 256" reshape of the ResNet-style workload has K + 1 > 65536
    rc, _, _ = B.rans_workspace_bytes(B.make_params(8, 12, 256, 100352, B.MODE_CSR, 1024, 0, B.F32), 256 * 100352)
    assert rc == B.ERR_ALPHABET
    # capacity
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    rc = B.rans_compress(x.cuda(), n, p, small, codec.nbytes, codec.ws)
    assert rc == 0 and B.rans_last_status(codec.ws) == B.ERR_CAPACITY and int(codec.nbytes.item()) == 0
    # caller-provided symbols outside {0..2^Q-1}
    p2 = B.make_params(2, 12, n, 1, B.MODE_DENSE, 32, 0, B.F32)
    c2 = B.Codec(p2, n)
    sym = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
    rc = B.rans_encode(sym, n, p2, c2.qinfo, c2.stream, c2.nbytes, c2.ws)
    assert rc == 0 and B.rans_last_status(c2.ws) == B.ERR_ARG
    # the status is sticky: a failed call is still reported after later good calls on the same workspace, once
    xb = _relu_normal(n, 3)
    xb[5] = float("nan")
    good = codec.compress(x.cuda())
    hdr = codec.header(good)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    keep = codec.stream.clone()
    assert B.rans_compress(xb.cuda(), n, p, codec.stream, codec.nbytes, codec.ws) == 0      # fails on the device
    assert B.rans_decompress(keep, good, hdr, B.F32, out, codec.ws) == 0                     # succeeds
    assert B.rans_compress(x.cuda(), n, p, codec.stream, codec.nbytes, codec.ws) == 0        # succeeds
    assert B.rans_last_status(codec.ws) == B.ERR_NONFINITE
    assert B.rans_last_status(codec.ws) == 0                                                 # reading cleared it
    assert codec.container(int(codec.nbytes.item())) == ref
    # the first of two different errors is the one reported
    assert B.rans_compress(x.cuda(), n, p, small, codec.nbytes, codec.ws) == 0               # capacity
    assert B.rans_compress(xb.cuda(), n, p, codec.stream, codec.nbytes, codec.ws) == 0       # non-finite
    assert B.rans_last_status(codec.ws) == B.ERR_CAPACITY and B.rans_last_status(codec.ws) == 0
    # a workspace needs no initialisation: whatever bytes it holds, a good call reports no error
    for fill in (0x00, 0xAB, 0xFF):
        codec.ws.fill_(fill)
        assert B.rans_compress(x.cuda(), n, p, codec.stream, codec.nbytes, codec.ws) == 0
        assert B.rans_last_status(codec.ws) == 0
        assert codec.container(int(codec.nbytes.item())) == ref
    # host-side argument errors
    assert B.rans_compress(x.cuda(), n, p, codec.stream, codec.nbytes, codec.ws[:1024]) == B.ERR_WORKSPACE
    assert B.rans_compress(x.cuda(), n, p, codec.stream[1:], codec.nbytes, codec.ws) == B.ERR_ARG
    import ctypes as C
    rc = B.lib().rans_compress(C.c_void_p(x.cuda().data_ptr()), n, C.byref(p), None, 1 << 20,
                               C.c_void_p(codec.nbytes.data_ptr()), C.c_void_p(codec.ws.data_ptr()),
                               codec.ws.numel(), None)
    assert rc == B.ERR_ARG


@pytest.mark.parametrize("name,shrink,over", [
    ("c1", 1, dict(mode=0)),
    ("c1", 1, {}),
    ("c1", 1, dict(cols=7, chunk_syms=32 * 128)),
    ("c1", 1, dict(mode=0, chunk_syms=32 * 64)),
    ("c2", 32, dict(mode=0, chunk_syms=1 << 18)),
    ("c2", 32, dict(chunk_syms=1 << 18)),
    ("c2", 32, {}),
    ("c3", 64, dict(chunk_syms=1 << 18)),
    ("c3", 64, dict(q_bits=6, cols=64, chunk_syms=1 << 18)),
    ("c3", 64, dict(q_bits=6, mode=0, chunk_syms=1 << 18)),
    ("c4", 8, {}),
    ("c5a", 32, {}),
    ("c5b", 32, dict(chunk_syms=1 << 20)),
])
def test_synthetic_workloads(name, shrink, over):
    w = synth.workload(name, shrink, **over)
    x = synth.make(w)
    nbytes = _check_all(x, B.params_of(w), f"{name}/{shrink} {over}")
    assert nbytes < x.numel() * x.element_size()


# the configurations bench.py reports, at their full size and in its launch configuration
FULL_SIZE = [(label, name, over) for label, name, over in synth.BENCH_CONFIGS]


@pytest.mark.parametrize("label,name,over", FULL_SIZE, ids=[c[0] for c in FULL_SIZE])
def test_full_size_configs_whole_container(label, name, over):
    """Whole container and whole decompressed tensor against the oracle at the full size of every configuration
    bench.py reports (c5a is the one its headline line is timed on)."""
    w = synth.workload(name, 1, **over)
    x = synth.make(w)
    p = B.params_of(w)
    print(f"[case] {label}: {name} full size {over} n={w.numel}", flush=True)
    ref, sym_ref = oracle.compress(x.numpy(), _oparams(p))
    codec = B.Codec(p, w.numel)
    xd = x.cuda()
    nbytes = codec.compress(xd)
    assert nbytes == len(ref)
    got = codec.stream[:nbytes].cpu().numpy()
    assert np.array_equal(got, np.frombuffer(ref, np.uint8))
    del got
    hdr = codec.header(nbytes)
    out = torch.empty(w.numel, dtype=x.dtype, device="cuda")
    codec.decompress(nbytes, hdr, out)
    qi = oracle.qinfo_from_minmax(hdr.x_min, hdr.x_max, w.q_bits)
    y_ref = oracle.dequantize(sym_ref, qi, w.in_dtype)
    assert np.array_equal(out.cpu().numpy().view(np.uint8), y_ref.view(np.uint8))
    sym = torch.empty(w.numel, dtype=torch.uint8, device="cuda")
    codec.decode(nbytes, hdr, sym)
    assert np.array_equal(sym.cpu().numpy(), sym_ref)


@pytest.mark.parametrize("N,K,Q,M,density", [
    (5_600_001, 3, 8, 12, 0.30),     # K below 16, not a divisor of 16: rows that straddle lanes; 4096-row tiles
    (1_400_003, 12, 8, 12, 0.45),
    (168_011, 100, 6, 13, 0.30),     # K >= 16 that does not divide the tile: row ends through memory
    (50_503, 333, 8, 13, 0.15),      # alphabet of K + 1 symbols
    (3_407, 5000, 8, 14, 0.05),      # a few rows per tile
])
def test_large_csr_odd_shapes(N, K, Q, M, density):
    """Tensors above 16.7 M elements (where the expand kernel sizes its tiles by the load of the fullest compute
    unit, and every kernel runs in the launch shape of the large configurations) with row and column counts that
    divide nothing: container, decoded symbols and dequantised values against the oracle."""
    n = N * K
    g = torch.Generator().manual_seed(N % 1000 + K)
    x = torch.rand(n, generator=g)
    x = torch.where(x < density, x + 0.01, torch.zeros(()))
    p = B.make_params(Q, M, N, K, B.MODE_CSR, 1024, 80 * 1024, B.F32)
    print(f"[case] large CSR N={N} K={K} Q={Q} M={M} n={n}", flush=True)
    ref, sym_ref = oracle.compress(x.numpy(), _oparams(p))
    codec = B.Codec(p, n)
    nbytes = codec.compress(x.cuda())
    assert nbytes == len(ref)
    assert np.array_equal(codec.stream[:nbytes].cpu().numpy(), np.frombuffer(ref, np.uint8))
    hdr = codec.header(nbytes)
    sym = torch.empty(n, dtype=torch.uint8, device="cuda")
    codec.decode(nbytes, hdr, sym)
    assert np.array_equal(sym.cpu().numpy(), sym_ref)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    codec.decompress(nbytes, hdr, out)
    qi = oracle.qinfo_from_minmax(hdr.x_min, hdr.x_max, Q)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), oracle.dequantize(sym_ref, qi, oracle.F32).view(np.uint32))


@pytest.mark.parametrize("name,over", [("c5a", {}), ("c2", dict(mode=0, chunk_syms=100352)), ("c4", dict(chunk_syms=18432))])
def test_full_size_dense_configs_repeated(name, over):
    """The dense encoder's three ways of sharing a compute unit among its work-groups (wave priorities in turn:
    c5a; a timed sleep before the look-back: c2 with 98 rows per stream; neither: c4 in small chunks) give the
    same container on every one of many calls in a row (the first one is compared with the oracle's by
    test_full_size_configs_whole_container)."""
    w = synth.workload(name, 1, **over)
    xd = synth.make(w).cuda()
    p = B.params_of(w)
    print(f"[case] {name} {over} full size, repeated", flush=True)
    codec = B.Codec(p, w.numel)
    first = None
    for it in range(30):
        assert B.rans_compress(xd, w.numel, p, codec.stream, codec.nbytes, codec.ws) == 0
        assert B.rans_last_status(codec.ws) == 0, f"call {it}"
        nbytes = int(codec.nbytes.item())
        got = codec.stream[:nbytes].clone()
        if first is None:
            first = got
        assert got.numel() == first.numel() and torch.equal(got, first), f"call {it}"


def test_full_size_csr_config_repeated():
    """c3 in CSR form at full size (fp32 64x512x28x28, N x 256, Q=8, M=14, S=1024, 2^16-symbol chunks): the whole
    container against the oracle's, and the same bytes on every one of many calls in a row.  Thousands of
    work-groups add to the histogram of D, the encoder's work-groups each build the table from it and place their
    words by looking at the totals of the ones before them; anything that depends on how the work-groups happen to
    be timed shows up here as an error status or as different bytes on some of the calls."""
    w = synth.workload("c3", 1, mode=1, cols=256, chunk_syms=65536)  # more chunks than the benchmark's row
    x = synth.make(w)
    p = B.params_of(w)
    print("[case] c3 CSR full size, repeated", flush=True)
    ref, _ = oracle.compress(x.numpy(), _oparams(p))
    ref = torch.from_numpy(np.frombuffer(ref, np.uint8).copy()).cuda()
    codec = B.Codec(p, w.numel)
    xd = x.cuda()
    for it in range(40):
        assert B.rans_compress(xd, w.numel, p, codec.stream, codec.nbytes, codec.ws) == 0
        assert B.rans_last_status(codec.ws) == 0, f"call {it}"
        nbytes = int(codec.nbytes.item())
        assert nbytes == ref.numel(), f"call {it}"
        assert torch.equal(codec.stream[:nbytes], ref), f"call {it}"
    hdr = codec.header(nbytes)
    sym = torch.empty(w.numel, dtype=torch.uint8, device="cuda")
    qinfo = torch.empty(4, dtype=torch.float32, device="cuda")
    assert B.rans_decode(codec.stream, nbytes, hdr, sym, qinfo, codec.ws) == 0
    assert B.rans_last_status(codec.ws) == 0
    sym_ref, _ = oracle.quantize(x.numpy(), 8)
    assert np.array_equal(sym.cpu().numpy(), sym_ref)


def _random_cases(seed, count):
    """Seeded parameter mixes: sizes, dtypes, bit widths, table sizes, stream and chunk counts, both modes."""
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(count):
        q = int(rng.integers(1, 9))
        dtype = torch.float16 if rng.random() < 0.4 else torch.float32
        s = int(rng.choice([1, 3, 32, 64, 100, 256, 300, 512, 640, 1024, 1500, 2048]))
        if rng.random() < 0.5:   # dense
            n = int(rng.integers(1, 250000))
            m = int(rng.integers(q, 16))
            rows, cols, mode = n, 1, B.MODE_DENSE
            length = n
        else:
            cols = int(rng.choice([1, 2, 4, 7, 16, 60, 64, 255, 256, 257, 1000, 5000]))
            rows = int(rng.integers(1, max(2, 250000 // cols)))
            n = rows * cols
            need = max(q, int(np.ceil(np.log2(cols + 1))))
            m = int(rng.integers(need, 16))
            mode = B.MODE_CSR
            length = 2 * n + rows
        per_chunk = int(rng.choice([0, 1, 2, 8, 64, 300]))
        cs = per_chunk * s
        if cs and (length + cs - 1) // cs > 20000:   # keeps the grid within what a small test should launch
            cs = 0
        cases.append((i, n, rows, cols, mode, dtype, q, m, s, cs, float(rng.choice([0.0, -0.5, 0.8])),
                      float(rng.choice([1.0, 1e-3, 300.0]))))
    return cases


@pytest.mark.parametrize("case", _random_cases(2511, 48), ids=lambda c: f"r{c[0]}")
def test_random_parameter_mixes(case):
    i, n, rows, cols, mode, dtype, q, m, s, cs, shift, scale = case
    x = _relu_normal(n, 1000 + i, dtype, shift=shift, scale=scale)
    p = B.make_params(q, m, rows, cols, mode, s, cs, B.F16 if dtype == torch.float16 else B.F32)
    _check_all(x, p, f"random {i}")


def test_formula_inputs_match_the_stored_oracle_digests():
    """The containers of the formula-given inputs of tests/golden/make_oracle_digests.py, made by the HIP path,
    against the digests that script stored from the oracle."""
    import hashlib
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_oracle_digests", os.path.join(here, "golden", "make_oracle_digests.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = {}
    for line in open(os.path.join(here, "golden", "oracle_container_digests.txt")):
        if not line.startswith("#") and line.strip():
            name, nb, h = line.split()
            stored[name] = (int(nb), h)
    for name, x, q, m, rows, cols, mode, s, cs in mod.cases():
        print(f"[case] formula input {name}", flush=True)
        p = B.make_params(q, m, rows, cols, mode, s, cs, B.F16 if x.dtype == np.float16 else B.F32)
        codec = B.Codec(p, x.size)
        xd = torch.from_numpy(x.copy()).cuda() if x.size else torch.zeros(0, device="cuda")
        got = codec.container(codec.compress(xd))
        assert (len(got), hashlib.sha256(got).hexdigest()) == stored[name], name
