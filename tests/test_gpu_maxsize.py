"""The largest tensors the library accepts (2^30 elements), where the oracle cannot code the whole input in
seconds: every output the oracle can compute one by one is compared on samples, and the rest is checked through
properties that hold at any size.

  * extrema in the header against torch's, Eq. 6 symbols and dequantised values of sampled slices against the
    oracle's quantiser (run on the slice with the global extrema appended);
  * the frequency table in the container against the oracle's normalisation of the histogram of ALL decoded
    symbols (counted by torch, not by the library);
  * sampled streams of sampled chunks (first, inner, last ragged): final state, word count and words against
    the oracle's single-stream coder run on oracle-quantised symbols (Eq. 2; the chunk layout of the container: states, word counts, words per stream);
  * the directory: monotone, ends at the container size;
  * CSR: decodes to exactly the symbols of the dense path, l_D = 2 nnz + N, table = normalised counts of
    v, c and r recomputed by torch.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_11664_amd import binding as B

pytestmark = pytest.mark.gpu

MAX_ELEMS = 1 << 30
SLAB = 1 << 26


def _fill(n, seed, shift, relu):
    """fp16 tensor of n elements on the GPU, seeded, generated slab by slab."""
    g = torch.Generator(device="cuda").manual_seed(seed)
    x = torch.empty(n, dtype=torch.float16, device="cuda")
    for i0 in range(0, n, SLAB):
        i1 = min(n, i0 + SLAB)
        t = torch.randn(i1 - i0, generator=g, device="cuda") + shift
        if relu:
            t = torch.relu(t)
        x[i0:i1] = t.to(torch.float16)
    return x


def _oracle_symbols(xs: np.ndarray, mn, mx, q_bits):
    """Eq. 6 on a sample with the tensor's extrema: the oracle quantises sample + [min, max]."""
    ext = np.concatenate([xs, np.array([mn, mx], xs.dtype)])
    sym, qi = oracle.quantize(ext, q_bits)
    return sym[:xs.size], qi


def _layout(stream, A, nc):
    payload_off = 128 + ((2 * A + 7) & ~7) + 8 * (nc + 1)
    head = stream[:payload_off].cpu().numpy()
    h = oracle.parse_header(head.tobytes())
    assert h.payload_off == payload_off
    f = head[h.table_off:h.table_off + 2 * A].view("<u2").copy()
    off = head[h.dir_off:h.dir_off + 8 * (nc + 1)].view("<u8").copy()
    return h, f, off


def _bincount_u8(sym, minlength):
    cnt = torch.zeros(minlength, dtype=torch.int64, device=sym.device)
    for i0 in range(0, sym.numel(), SLAB):
        cnt += torch.bincount(sym[i0:i0 + SLAB].to(torch.int32), minlength=minlength)
    return cnt


def _check_slices(x, sym, out, n, mn, mx, q_bits, seed):
    rng = np.random.default_rng(seed)
    starts = [0, n - 8192] + [int(s) for s in rng.integers(0, n - 8192, 8)]
    for s0 in starts:
        xs = x[s0:s0 + 8192].cpu().numpy()
        ref, qi = _oracle_symbols(xs, mn, mx, q_bits)
        assert np.array_equal(sym[s0:s0 + 8192].cpu().numpy(), ref), f"symbols differ in slice at {s0}"
        y_ref = oracle.dequantize(ref, qi, oracle.F16)
        assert np.array_equal(out[s0:s0 + 8192].cpu().numpy().view(np.uint16), y_ref.view(np.uint16)), s0
    return qi


@pytest.mark.parametrize("n,cs,what", [
    (MAX_ELEMS, 1 << 18, "the encoder places its words itself"),
    (MAX_ELEMS - 12345, 1 << 16, "separate size scan and gather kernels, ragged last chunk"),
])
def test_dense_maximum_size(n, cs, what):
    Q, M, S = 8, 14, 1024
    print(f"[case] dense n={n} cs={cs}: {what}", flush=True)
    rc, _, _ = B.rans_workspace_bytes(B.make_params(Q, M, MAX_ELEMS + 1, 1, B.MODE_DENSE, S, cs, B.F16), MAX_ELEMS + 1)
    assert rc == B.ERR_ARG  # one element more is refused on the host
    x = _fill(n, 20251, 0.3, relu=False)
    p = B.make_params(Q, M, n, 1, B.MODE_DENSE, S, cs, B.F16)
    codec = B.Codec(p, n)
    nbytes = codec.compress(x)
    hdr = codec.header(nbytes)
    assert hdr.n_elems == n and hdr.len_d == n
    mn, mx = float(x.min().item()), float(x.max().item())
    assert hdr.x_min == mn and hdr.x_max == mx
    nc = (n + cs - 1) // cs
    assert hdr.n_chunks == nc
    h, f, off = _layout(codec.stream, 256, nc)
    assert off[0] == 0 and np.all(np.diff(off.astype(np.int64)) >= 8 * S) and h.payload_off + int(off[nc]) == nbytes

    # decode: symbols and dequantised values on sampled slices
    sym = torch.empty(n, dtype=torch.uint8, device="cuda")
    codec.decode(nbytes, hdr, sym)
    out = torch.empty(n, dtype=torch.float16, device="cuda")
    codec.decompress(nbytes, hdr, out)
    qi = _check_slices(x, sym, out, n, mn, mx, Q, 5)
    q = codec.qinfo.cpu().numpy()
    assert np.array_equal(q.view(np.uint32), np.array(qi.as_tuple(), np.float32).view(np.uint32))
    # the dequantised tensor is a function of the symbols alone: 256 values, each checked above or here
    lut = torch.from_numpy(oracle.dequantize(np.arange(256, dtype=np.uint8), qi, oracle.F16).view(np.int16)).cuda()
    for i0 in range(0, n, SLAB):
        assert torch.equal(out[i0:i0 + SLAB].view(torch.int16), lut[sym[i0:i0 + SLAB].to(torch.int64)]), i0

    # the table: the oracle's normalisation of the histogram of all symbols
    cnt = _bincount_u8(sym, 256).cpu().numpy().astype(np.uint64)
    assert int(cnt.sum()) == n
    f_ref, _ = oracle.normalize(cnt, M)
    assert np.array_equal(f, f_ref)

    # sampled streams of sampled chunks against the oracle's coder
    rng = np.random.default_rng(11)
    for k in (0, int(rng.integers(1, nc - 1)), nc - 1):
        base = k * cs
        n_here = min(cs, n - base)
        ck = codec.stream[h.payload_off + int(off[k]):h.payload_off + int(off[k + 1])].cpu().numpy()
        states = ck[:4 * S].view("<u4")
        nwords = ck[4 * S:8 * S].view("<u4")
        used = 8 * S + 2 * int(nwords.sum())
        assert ck.size == (used + 3) & ~3 and not ck[used:].any()  # a chunk is zero-padded to 4 bytes
        wstart = 8 * S + 2 * np.concatenate([[0], np.cumsum(nwords.astype(np.int64))])
        xk = x[base:base + n_here].cpu().numpy()
        for j in (0, 1, 63, 64, 517, S - 1):
            xs = xk[j::S]
            d, _ = _oracle_symbols(xs, mn, mx, Q)
            st, words = oracle.encode_stream(d, f, M)
            assert st == int(states[j]), f"chunk {k} stream {j}: state"
            assert words.size == int(nwords[j]), f"chunk {k} stream {j}: word count"
            got = ck[int(wstart[j]):int(wstart[j + 1])].view("<u2")
            assert np.array_equal(got, words), f"chunk {k} stream {j}: words"


def test_csr_large_against_dense_path():
    """2^29 elements as [2^21, 256] with about 70 % zeros: l_D is about 3.2e8 symbols of D = v (+) c (+) r."""
    Q, M, S, cs = 8, 14, 1024, 1 << 18
    n, K = 1 << 29, 256
    N = n // K
    print(f"[case] CSR n={n} [{N}, {K}]", flush=True)
    x = _fill(n, 777, -0.52, relu=True)
    pd = B.make_params(Q, M, n, 1, B.MODE_DENSE, S, cs, B.F16)
    cd = B.Codec(pd, n)
    nb_d = cd.compress(x)
    sym_d = torch.empty(n, dtype=torch.uint8, device="cuda")
    cd.decode(nb_d, cd.header(nb_d), sym_d)
    mn, mx = float(x.min().item()), float(x.max().item())
    out = torch.empty(n, dtype=torch.float16, device="cuda")
    cd.decompress(nb_d, cd.header(nb_d), out)
    _check_slices(x, sym_d, out, n, mn, mx, Q, 6)
    del cd, out

    pc = B.make_params(Q, M, N, K, B.MODE_CSR, S, cs, B.F16)
    cc = B.Codec(pc, n)
    nb_c = cc.compress(x)
    hdr = cc.header(nb_c)
    nz = sym_d != 0
    nnz = int(nz.sum().item())
    assert hdr.len_d == 2 * nnz + N and hdr.n_elems == n
    assert hdr.x_min == mn and hdr.x_max == mx
    sym_c = torch.empty(n, dtype=torch.uint8, device="cuda")
    cc.decode(nb_c, hdr, sym_c)
    assert torch.equal(sym_c, sym_d)
    # the table over D: counts of the values, the column indices and the row counts
    A = oracle.alphabet(oracle.MODE_CSR, Q, K)
    assert hdr.alphabet == A
    cnt = torch.zeros(A, dtype=torch.int64, device="cuda")
    v_cnt = _bincount_u8(sym_d, 256)
    v_cnt[0] = 0
    cnt[:256] += v_cnt
    nz2 = nz.view(N, K)
    c_cnt = torch.zeros(K, dtype=torch.int64, device="cuda")
    for r0 in range(0, N, 1 << 18):
        c_cnt += nz2[r0:r0 + (1 << 18)].sum(0)
    cnt[:K] += c_cnt
    r = torch.cat([nz2[r0:r0 + (1 << 18)].sum(1) for r0 in range(0, N, 1 << 18)])
    cnt += torch.bincount(r, minlength=A)
    assert int(cnt.sum().item()) == 2 * nnz + N
    nc = (2 * nnz + N + cs - 1) // cs
    h, f, off = _layout(cc.stream, A, nc)
    f_ref, _ = oracle.normalize(cnt.cpu().numpy().astype(np.uint64), M)
    assert np.array_equal(f, f_ref)
    assert off[0] == 0 and np.all(np.diff(off.astype(np.int64)) >= 8 * S) and h.payload_off + int(off[nc]) == nb_c
    out = torch.empty(n, dtype=torch.float16, device="cuda")
    cc.decompress(nb_c, hdr, out)
    _, qi = _oracle_symbols(x[:16].cpu().numpy(), mn, mx, Q)
    lut = torch.from_numpy(oracle.dequantize(np.arange(256, dtype=np.uint8), qi, oracle.F16).view(np.int16)).cuda()
    for i0 in range(0, n, SLAB):
        assert torch.equal(out[i0:i0 + SLAB].view(torch.int16), lut[sym_d[i0:i0 + SLAB].to(torch.int64)]), i0
