#!/usr/bin/env python3
"""Benchmark of the rANS intermediate-feature codec on one MI355X.

One step = the whole hot path over one tensor: rans_compress (min/max, quantise,
histogram, normalise, interleaved rANS encode, container) followed by
rans_decompress (table rebuild, rANS decode, dequantise), inputs and outputs
resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5a] [--mode 0|1] [--cols K]
                    [--q-bits Q] [--chunk-syms N] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5a")
    ap.add_argument("--chunk-syms", type=int, default=None)
    ap.add_argument("--mode", type=int, default=None)
    ap.add_argument("--cols", type=int, default=None)
    ap.add_argument("--q-bits", type=int, default=None)
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the codec has no cross-GPU step); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_11664_amd import binding as B, synth

    over = {}
    if args.chunk_syms is not None:
        over["chunk_syms"] = args.chunk_syms
    if args.mode is not None:
        over["mode"] = args.mode
    if args.cols is not None:
        over["cols"] = args.cols
    if args.q_bits is not None:
        over["q_bits"] = args.q_bits
    w = synth.workload(args.workload, 1, **over)
    x_cpu = synth.make(w)
    p = B.params_of(w)
    n = w.numel
    e = x_cpu.element_size()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    x = x_cpu.to(dev)
    codec = B.Codec(p, n)
    out = torch.empty(n, dtype=x.dtype, device=dev)

    nbytes = codec.compress(x)
    hdr = codec.header(nbytes)
    codec.decompress(nbytes, hdr, out)
    # a plain device copy of known size (reads and writes the input's byte count once): the reference
    # that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this script
    calib = torch.empty_like(x)
    calib.copy_(x)
    del calib

    def step():
        rc = B.rans_compress(x, n, p, codec.stream, codec.nbytes, codec.ws)
        rc |= B.rans_decompress(codec.stream, nbytes, hdr, w.in_dtype, out, codec.ws)
        return rc

    # warm-up; its last steps run with every kernel bracketed by events to find the dominant one
    for i in range(args.warmup):
        if i == max(0, args.warmup - 3):
            B.rans_profile_reset()
            B.rans_profile_enable("all")
        step()
    torch.cuda.synchronize()
    B.rans_profile_enable(None)
    prof_all = B.rans_profile_read()
    dom = max(prof_all, key=lambda k: prof_all[k]["total_ms"]) if prof_all else None

    # timed region: exactly K steps; the dominant kernel carries an event pair on every 5th launch (each
    # pair costs about 10 us of stream time, so bracketing every launch would distort the step time)
    B.rans_profile_reset()
    if dom:
        B.rans_profile_enable([dom], every=5)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        rc = step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    B.rans_profile_enable(None)
    assert rc == 0 and B.rans_last_status(codec.ws) == 0
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    prof = B.rans_profile_read()          # launch durations of the dominant kernel inside the timed region

    # encode and decode separately: p50 over per-call event pairs
    def p50_us(fn, reps):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:
            a.record()
            fn()
            b.record()
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        return ts[len(ts) // 2], ts[len(ts) // 10], ts[(9 * len(ts)) // 10]

    reps = max(args.steps, 20)
    enc_p50, enc_p10, enc_p90 = p50_us(lambda: B.rans_compress(x, n, p, codec.stream, codec.nbytes, codec.ws), reps)
    dec_p50, dec_p10, dec_p90 = p50_us(lambda: B.rans_decompress(codec.stream, nbytes, hdr, w.in_dtype, out, codec.ws), reps)

    # the four unfused entry points, for the record (symbols through a caller-side buffer)
    sym = torch.empty(n, dtype=torch.uint8, device=dev)
    unf = {}
    for name, fn in (("rans_quantize", lambda: B.rans_quantize(x, n, p, sym, codec.qinfo, codec.ws)),
                     ("rans_encode", lambda: B.rans_encode(sym, n, p, codec.qinfo, codec.stream, codec.nbytes, codec.ws)),
                     ("rans_decode", lambda: B.rans_decode(codec.stream, nbytes, hdr, sym, codec.qinfo, codec.ws)),
                     ("rans_dequantize", lambda: B.rans_dequantize(sym, n, codec.qinfo, w.in_dtype, out))):
        fn()
        unf[name] = round(p50_us(fn, 20)[0], 1)
    assert B.rans_last_status(codec.ws) == 0

    in_bytes = n * e
    # algorithmic bytes: three forced passes on the encode side (min/max reads X; quantise reads X and
    # writes xhat; the coder reads xhat and writes the container), one on the decode side.
    b_enc = 2 * e * n + 2 * n + nbytes
    b_dec = nbytes + e * n
    if w.mode == synth.MODE_CSR:
        # D = v (u8), c (u16), r (u16) is written and read back on both sides; the decoder also zero-fills and
        # scatters the symbol tensor
        nnz = (int(hdr.len_d) - w.rows) // 2
        d_bytes = 2 * (3 * nnz + 2 * w.rows)
        b_enc += d_bytes
        b_dec += d_bytes + n
    alg = {"k_encode": n + nbytes, "k_decode": nbytes + e * n, "k_quant_hist": e * n + n, "k_minmax": e * n,
           "k_gather": 2 * nbytes}
    # HBM-side bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary of this
    # same command (FETCH_SIZE / WRITE_SIZE scaled by a plain copy of known size); null if there is none
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"{w.name}_{'csr' if w.mode else 'dense'}_pmc_traffic.txt")
    if dom and os.path.exists(tfile) and not over:
        for line in open(tfile):
            if line.startswith(dom):
                traffic = int(line.split()[-1])
    roof = None
    if dom:
        avg_ms = prof[dom]["total_ms"] / prof[dom]["count"]
        achieved = alg.get(dom, 0) / (avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "avg_us": round(avg_ms * 1e3, 2),
                "algorithmic_bytes": alg.get(dom, 0),
                "all_kernels_avg_us_warmup": {k: round(v["total_ms"] / v["count"] * 1e3, 2) for k, v in prof_all.items()}}

    cpu = None
    if not args.no_cpu:
        import oracle
        # bounded sample: the whole tensor if it has at most 2^27 elements (about 5-10 s of single-thread work for
        # the Llama-shaped tensors), else its first 2^27 elements (same recipe, same parameters)
        cap = 1 << 27
        ns = n if n <= cap else (cap // w.cols * w.cols if w.mode == synth.MODE_CSR else cap)
        xs = x_cpu[:ns].numpy()
        op = oracle.make_params(w.q_bits, w.freq_bits, ns // w.cols if w.mode == synth.MODE_CSR else ns,
                                w.cols if w.mode == synth.MODE_CSR else 1, w.mode, w.n_streams, w.chunk_syms, w.in_dtype)
        t0 = time.perf_counter()
        buf, _ = oracle.compress(xs, op)
        t_enc = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.decompress(buf, w.in_dtype)
        t_dec = time.perf_counter() - t0
        cpu = {"value": round(ns * e / (t_enc + t_dec) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"first {ns} of {n} elements ({ns * e / 1e6:.1f} MB), compress {t_enc:.2f} s + decompress {t_dec:.2f} s",
               "encode_GBps": round(ns * e / t_enc / 1e9, 4), "decode_GBps": round(ns * e / t_dec / 1e9, 4)}

    line = {
        "metric": "encode+decode throughput of the input tensor (rans_compress followed by rans_decompress)",
        "value": round(in_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 state / f32 quantiser", "data": "synthetic",
        "config": {"workload": f"{w.name}: {'fp16' if e == 2 else 'fp32'} {'x'.join(map(str, w.shape))}, Q={w.q_bits}, M={w.freq_bits}, "
                               f"S={w.n_streams}, chunk_syms={w.chunk_syms}, mode={'CSR' if w.mode else 'DENSE'}"
                               + (f" N={w.rows} K={w.cols}" if w.mode else ""),
                   "input_bytes": in_bytes, "container_bytes": nbytes,
                   "compression_ratio": round(in_bytes / nbytes, 3), "bits_per_element": round(8 * nbytes / n, 3)},
        "encode": {"p50_us": round(enc_p50, 1), "p10_us": round(enc_p10, 1), "p90_us": round(enc_p90, 1),
                   "GBps_input": round(in_bytes / enc_p50 / 1e3, 1), "GBps_fp32_equiv": round(4 * n / enc_p50 / 1e3, 1),
                   "algorithmic_bytes": b_enc, "roofline_frac": round(b_enc / (enc_p50 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
        "decode": {"p50_us": round(dec_p50, 1), "p10_us": round(dec_p10, 1), "p90_us": round(dec_p90, 1),
                   "GBps_output": round(in_bytes / dec_p50 / 1e3, 1), "GBps_fp32_equiv": round(4 * n / dec_p50 / 1e3, 1),
                   "algorithmic_bytes": b_dec, "roofline_frac": round(b_dec / (dec_p50 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
        "unfused_p50_us": unf,
        "roofline": roof,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
