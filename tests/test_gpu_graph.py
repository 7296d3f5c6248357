"""The entry points only enqueue kernels, so a caller may capture them into a HIP graph: replays, with eager
work and synchronisations between them, must write what the eager call writes (the oracle's container, the
oracle's dequantised tensor), and a replayed rans_compress must start from a clean status."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_11664_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def _oparams(p):
    return oracle.make_params(p.q_bits, p.freq_bits, p.rows, p.cols, p.mode, p.n_streams, p.chunk_syms, p.in_dtype)


@pytest.mark.parametrize("over", [{}, dict(mode=1, cols=4)])
def test_graph_replay_matches_eager_and_oracle(over):
    w = synth.workload("t1", 1, **over)
    x_cpu = synth.make(w)
    p = B.params_of(w)
    n = w.numel
    print(f"[case] graph replay t1 {over}", flush=True)
    ref, sym_ref = oracle.compress(x_cpu.numpy(), _oparams(p))
    _, qi = oracle.quantize(x_cpu.numpy(), p.q_bits)
    y_ref = torch.from_numpy(oracle.dequantize(sym_ref, qi, oracle.F32)).cuda()
    ref_d = torch.from_numpy(np.frombuffer(ref, np.uint8).copy()).cuda()
    x = x_cpu.cuda()
    codec = B.Codec(p, n)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    nbytes = codec.compress(x)
    hdr = codec.header(nbytes)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    g_enc, g_dec = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_enc, stream=s):
        assert B.rans_compress(x, n, p, codec.stream, codec.nbytes, codec.ws) == 0
    with torch.cuda.graph(g_dec, stream=s):
        assert B.rans_decompress(codec.stream, nbytes, hdr, B.F32, out, codec.ws) == 0
    torch.cuda.synchronize()
    for it in range(4):
        codec.stream.zero_()
        out.fill_(-1.0)
        g_enc.replay()
        torch.cuda.synchronize()
        assert B.rans_last_status(codec.ws) == 0
        assert int(codec.nbytes.item()) == len(ref), f"replay {it}"
        assert torch.equal(codec.stream[:nbytes], ref_d), f"replay {it}"
        _ = (x * 2).sum().item()  # the program's own eager work between replays
        g_dec.replay()
        torch.cuda.synchronize()
        assert B.rans_last_status(codec.ws) == 0
        assert torch.equal(out.view(torch.int32), y_ref.view(torch.int32)), f"replay {it}"

    # an error in one replay is not carried into the next: the tensor is captured by address, its values are not
    x[12345 % n] = float("nan")
    g_enc.replay()
    torch.cuda.synchronize()
    assert B.rans_last_status(codec.ws) == B.ERR_NONFINITE and int(codec.nbytes.item()) == 0
    x.copy_(x_cpu)
    g_enc.replay()
    torch.cuda.synchronize()
    assert B.rans_last_status(codec.ws) == 0
    assert int(codec.nbytes.item()) == len(ref) and torch.equal(codec.stream[:nbytes], ref_d)
