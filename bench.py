#!/usr/bin/env python3
"""Benchmark of the rANS intermediate-feature codec on one MI355X.

One step = the whole hot path over one tensor: rans_compress (min/max, quantise,
histogram, normalise, interleaved rANS encode, container) followed by
rans_decompress (table rebuild, rANS decode, dequantise), inputs and outputs
resident in HBM.  Prints ONE JSON line.  Besides the headline figures of the
timed workload the line carries
  roofline      the dominant kernel against the HBM peak (durations measured in this run)
  cpu_baseline  the CPU oracle on the same tensor: one core, and all host cores
  configs       encode / decode p50, GB/s, roofline fraction and ratio for every
                configuration of synth.BENCH_CONFIGS (the rows the full-size parity tests check)
  eq8           the terms of the paper's Eq. 8 over the reshape domain of Algorithm 1 on the
                Table-1-shaped tensor, next to a plain copy ("binary serialisation")

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c5a] [--mode 0|1] [--cols K]
                    [--q-bits Q] [--chunk-syms N] [--no-cpu] [--no-configs] [--configs a,b,...]

Two further measurements print a JSON object of their own instead of that line:

    python bench.py --sweep bits [--workload t1]      size and latency per bit width Q (layout of the paper's Table 1 / 3)
    python bench.py --sweep reshape [--workload t1]   Eq. 8: size, encode and decode time for every reshape N of
                                                      Algorithm 1's domain, next to a plain copy of the tensor
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak


def _p50(torch, fn, reps=30, warm=3):
    """p50 / p10 / p90 in microseconds of fn() on the current stream, one event pair per call."""
    for _ in range(warm):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
    return ts[len(ts) // 2], ts[len(ts) // 10], ts[(9 * len(ts)) // 10]


def _describe(w):
    e = 2 if w.in_dtype else 4
    return (f"{w.name}: {'fp16' if e == 2 else 'fp32'} {'x'.join(map(str, w.shape))}, Q={w.q_bits}, M={w.freq_bits}, "
            f"S={w.n_streams}, chunk_syms={w.chunk_syms}, mode={'CSR' if w.mode else 'DENSE'}"
            + (f" N={w.rows} K={w.cols}" if w.mode else ""))


def _alg_bytes(w, nbytes, len_d):
    """Algorithmic bytes of the two directions: three forced passes on the encode side (min/max reads X; quantise
    reads X and writes xhat; the coder reads xhat and writes the container), one on the decode side.  CSR: D = v (u8),
    c (u16), r (u16) is written and read back on both sides; the decoder also zero-fills and scatters the symbols."""
    n, e = w.numel, (2 if w.in_dtype else 4)
    b_enc = 2 * e * n + 2 * n + nbytes
    b_dec = nbytes + e * n
    if w.mode:
        nnz = (len_d - w.rows) // 2
        d_bytes = 2 * (3 * nnz + 2 * w.rows)
        b_enc += d_bytes
        b_dec += d_bytes + n
    return b_enc, b_dec


def measure_config(torch, B, synth, label, name, over, reps):
    """One row of the configs table: whole-call p50 of rans_compress and rans_decompress."""
    w = synth.workload(name, 1, **over)
    x = synth.make(w).cuda()
    n = w.numel
    e = x.element_size()
    p = B.params_of(w)
    codec = B.Codec(p, n)
    out = torch.empty(n, dtype=x.dtype, device=x.device)
    nbytes = codec.compress(x)
    hdr = codec.header(nbytes)
    codec.decompress(nbytes, hdr, out)
    enc = _p50(torch, lambda: B.rans_compress(x, n, p, codec.stream, codec.nbytes, codec.ws), reps)
    assert B.rans_last_status(codec.ws) == 0 and int(codec.nbytes.item()) == nbytes
    dec = _p50(torch, lambda: B.rans_decompress(codec.stream, nbytes, hdr, w.in_dtype, out, codec.ws), reps)
    assert B.rans_last_status(codec.ws) == 0
    b_enc, b_dec = _alg_bytes(w, nbytes, int(hdr.len_d))
    in_bytes = n * e
    return {"label": label, "workload": _describe(w), "input_MB": round(in_bytes / 1e6, 3),
            "ratio": round(in_bytes / nbytes, 3), "bits_per_elem": round(8 * nbytes / n, 3),
            "enc_p50_us": round(enc[0], 1), "enc_GBps": round(in_bytes / enc[0] / 1e3, 1),
            "enc_frac": round(b_enc / (enc[0] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
            "dec_p50_us": round(dec[0], 1), "dec_GBps": round(in_bytes / dec[0] / 1e3, 1),
            "dec_frac": round(b_dec / (dec[0] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}


def eq8_terms(torch, B, synth, name="t1", reps=20):
    """Eq. 8, T(N) = alpha_enc T_enc(N) + alpha_dec T_dec(N) + T_tot(N), over the whole domain of Algorithm 1."""
    import ctypes as C
    w = synth.workload(name, 1)
    x = synth.make(w).cuda()
    n = w.numel
    pd = B.params_of(w)
    cq = B.Codec(pd, n)
    sym = torch.empty(n, dtype=torch.uint8, device="cuda")
    cq.quantize(x.reshape(-1), sym)
    res = B.search_reshape(sym, w.q_bits)
    out = torch.empty(n, dtype=x.dtype, device="cuda")
    rows = []
    for k in range(res.n_candidates):
        N = int(res.cand_rows[k])
        p = B.make_params(w.q_bits, w.freq_bits, N, n // N, B.MODE_CSR, w.n_streams, w.chunk_syms, w.in_dtype)
        ce = B.Codec(p, n)
        ce.qinfo.copy_(cq.qinfo)
        nb = ce.encode(sym)
        hc = ce.header(nb)
        rows.append({"N": N, "K": n // N, "len_D": int(hc.len_d), "T_tot_bits": round(float(res.cand_cost[k]), 1),
                     "container_bytes": nb,
                     "T_enc_us": round(_p50(torch, lambda: B.rans_encode(sym, n, p, ce.qinfo, ce.stream, ce.nbytes, ce.ws), reps)[0], 1),
                     "T_dec_us": round(_p50(torch, lambda: B.rans_decompress(ce.stream, nb, hc, w.in_dtype, out, ce.ws), reps)[0], 1)})
    calib = torch.empty_like(x)
    copy_us = round(_p50(torch, lambda: calib.copy_(x), reps)[0], 1)
    rc, wsb = B.rans_search_workspace_bytes(n, w.q_bits)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    rr = torch.zeros(C.sizeof(B.ReshapeResult), dtype=torch.uint8, device="cuda")
    search_us = round(_p50(torch, lambda: B.rans_search_reshape(sym, n, w.q_bits, rr, ws), reps)[0], 1)
    best = {}
    for alpha in (0.0, 100.0, 10000.0):  # bits per microsecond of coding time (the rate of the link)
        best[str(alpha)] = min(rows, key=lambda r: r["T_tot_bits"] + alpha * (r["T_enc_us"] + r["T_dec_us"]))["N"]
    return {"workload": name, "q_bits": w.q_bits, "chosen_by_algorithm_1": int(res.rows), "n_evaluated": int(res.n_evaluated),
            "search_us": search_us, "argmin_N_for_alpha_bits_per_us": best,
            "binary_serialisation": {"bytes": n * x.element_size(), "copy_us": copy_us}, "rows": rows}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


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
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration table and the Eq. 8 terms")
    ap.add_argument("--configs", default=None, help="comma-separated labels of synth.BENCH_CONFIGS (default: all)")
    ap.add_argument("--sweep", choices=["bits", "reshape"], default=None)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the codec has no cross-GPU step); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2511_11664_amd import binding as B, synth

    if args.sweep:
        return sweep(args, np, torch, B, synth)

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
    # the status is sticky: the first error of any of the 2 K calls would still be there
    assert rc == 0 and B.rans_last_status(codec.ws) == 0 and int(codec.nbytes.item()) == nbytes
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    prof = B.rans_profile_read()          # launch durations of the dominant kernel inside the timed region

    # encode and decode separately: p50 over per-call event pairs
    reps = max(args.steps, 20)
    enc_p50, enc_p10, enc_p90 = _p50(torch, lambda: B.rans_compress(x, n, p, codec.stream, codec.nbytes, codec.ws), reps, 0)
    assert B.rans_last_status(codec.ws) == 0 and int(codec.nbytes.item()) == nbytes
    dec_p50, dec_p10, dec_p90 = _p50(torch, lambda: B.rans_decompress(codec.stream, nbytes, hdr, w.in_dtype, out, codec.ws), reps, 0)
    assert B.rans_last_status(codec.ws) == 0

    # the four unfused entry points, for the record (symbols through a caller-side buffer)
    sym = torch.empty(n, dtype=torch.uint8, device=dev)
    unf = {}
    for name, fn in (("rans_quantize", lambda: B.rans_quantize(x, n, p, sym, codec.qinfo, codec.ws)),
                     ("rans_encode", lambda: B.rans_encode(sym, n, p, codec.qinfo, codec.stream, codec.nbytes, codec.ws)),
                     ("rans_decode", lambda: B.rans_decode(codec.stream, nbytes, hdr, sym, codec.qinfo, codec.ws)),
                     ("rans_dequantize", lambda: B.rans_dequantize(sym, n, codec.qinfo, w.in_dtype, out))):
        unf[name] = round(_p50(torch, fn, 20, 1)[0], 1)
    assert B.rans_last_status(codec.ws) == 0

    in_bytes = n * e
    # the measured ceiling of this machine: a plain device-to-device copy of the input (reads and writes its bytes once)
    calib = torch.empty_like(x)
    copy_p50 = _p50(torch, lambda: calib.copy_(x), 20, 1)[0]
    del calib
    copy_ceiling = {"p50_us": round(copy_p50, 1), "GBps": round(2 * in_bytes / copy_p50 / 1e3, 1),
                    "frac_of_peak": round(2 * in_bytes / copy_p50 / 1e3 / HBM_PEAK_GBPS, 4)}
    # bits per symbol next to the entropy H of the symbols and the cross entropy CE against the stored table
    # (Eq. 1); DENSE mode only, where D is the symbol tensor itself
    coding = None
    if w.mode != synth.MODE_CSR and n:
        hist = torch.bincount(sym.to(torch.int64), minlength=1 << w.q_bits).double().cpu().numpy()
        pr = hist / hist.sum()
        f = np.frombuffer(codec.stream[128:128 + 2 * (1 << w.q_bits)].cpu().numpy().tobytes(), dtype="<u2").astype(np.float64)
        nzm = pr > 0
        H = float(-(pr[nzm] * np.log2(pr[nzm])).sum())
        CE = float(-(pr[nzm] * np.log2(f[nzm] / float(1 << w.freq_bits))).sum())
        coding = {"bits_per_symbol": round(8 * nbytes / n, 4), "entropy_H": round(H, 4), "cross_entropy_CE": round(CE, 4)}
    b_enc, b_dec = _alg_bytes(w, nbytes, int(hdr.len_d))
    # algorithmic bytes per launch of the kernels that can dominate (per-unit figure x units of one launch)
    alg = {"k_encode": n + nbytes, "k_decode": nbytes + e * n, "k_quant_hist": e * n + n, "k_minmax": e * n,
           "k_gather": 2 * nbytes}
    # HBM-side bytes per launch of the dominant kernel: NOT measured by this run (counters need rocprofv3); the figure
    # is the one recorded by the rocprofv3 --pmc runs of this same command whose summary is committed under profiles/
    # (FETCH_SIZE + WRITE_SIZE, each scaled by what the counter reads for the plain copy above), null if there is none
    traffic, traffic_source = None, None
    tfile = os.path.join(ROOT, "profiles", f"{w.name}_{'csr' if w.mode else 'dense'}_pmc_traffic.txt")
    if dom and os.path.exists(tfile) and not over:
        # the summary has one line per template instantiation; the timed loop runs the fused encoder and the
        # decoder that writes the caller's dtype, the other instantiations belong to the unfused entry points
        want = {"k_encode": f"k_encode<{'SrcCsr' if w.mode else 'SrcDense'},2,{'true' if w.freq_bits >= 8 else 'false'},true>",
                "k_decode": "k_decode_fast<FSink" + ("U16" if w.mode else "Float")}.get(dom, dom + "<")
        hits = [line.split() for line in open(tfile) if line.startswith(want)]
        if len(hits) == 1:
            traffic = int(hits[0][-1])
            traffic_source = (os.path.relpath(tfile, ROOT) + f" line {hits[0][0]}"
                              + " (rocprofv3 --pmc runs of this command, recorded earlier; not measured in this run)")
    roof = None
    if dom:
        avg_ms = prof[dom]["total_ms"] / prof[dom]["count"]
        achieved = alg.get(dom, 0) / (avg_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                "avg_us": round(avg_ms * 1e3, 2), "algorithmic_bytes": alg.get(dom, 0),
                "all_kernels_avg_us_warmup": {k: round(v["total_ms"] / v["count"] * 1e3, 2) for k, v in prof_all.items()}}

    cpu = None
    if not args.no_cpu:
        import oracle
        # bounded sample: the whole tensor if it has at most 2^27 elements (about 15-20 s of single-thread work for
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
        # all host cores this process may run on: the same oracle routines on slices / row blocks / chunks, one
        # std::thread per core (oracle/rans_oracle_mt.cpp)
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count() or 1
        cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
        buf_np = np.frombuffer(buf, np.uint8)
        oracle.lib_mt()
        t0 = time.perf_counter()
        buf_mt = oracle.compress_mt(xs, op, cores)
        t_enc_mt = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.decompress_mt(buf_np, w.in_dtype, cores)
        t_dec_mt = time.perf_counter() - t0
        assert buf_mt == buf
        sample = f"first {ns} of {n} elements ({ns * e / 1e6:.1f} MB)"
        cpu = {"value": round(ns * e / (t_enc + t_dec) / 1e9, 4), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"{sample}, compress {t_enc:.2f} s + decompress {t_dec:.2f} s", "cpu_model": cpu_model(),
               "encode_GBps": round(ns * e / t_enc / 1e9, 4), "decode_GBps": round(ns * e / t_dec / 1e9, 4),
               "all_cores": {"value": round(ns * e / (t_enc_mt + t_dec_mt) / 1e9, 4), "unit": "GB/s", "cores": cores,
                             "kind": "oracle routines under a chunk-parallel std::thread driver",
                             "sample": f"{sample}, compress {t_enc_mt:.2f} s + decompress {t_dec_mt:.2f} s",
                             "encode_GBps": round(ns * e / t_enc_mt / 1e9, 4), "decode_GBps": round(ns * e / t_dec_mt / 1e9, 4)}}

    configs, eq8 = None, None
    if not args.no_configs:
        del x, out, sym, codec
        torch.cuda.empty_cache()
        want = set(args.configs.split(",")) if args.configs else None
        configs = []
        for label, name, cover in synth.BENCH_CONFIGS:
            if want is None or label in want:
                configs.append(measure_config(torch, B, synth, label, name, cover, 20))
                torch.cuda.empty_cache()
        eq8 = eq8_terms(torch, B, synth)

    line = {
        "metric": "encode+decode throughput of the input tensor (rans_compress followed by rans_decompress)",
        "value": round(in_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 state / f32 quantiser", "data": "synthetic",
        "config": {"workload": _describe(w), "input_bytes": in_bytes, "container_bytes": nbytes,
                   "compression_ratio": round(in_bytes / nbytes, 3), "bits_per_element": round(8 * nbytes / n, 3)},
        "encode": {"p50_us": round(enc_p50, 1), "p10_us": round(enc_p10, 1), "p90_us": round(enc_p90, 1),
                   "GBps_input": round(in_bytes / enc_p50 / 1e3, 1), "GBps_fp32_equiv": round(4 * n / enc_p50 / 1e3, 1),
                   "algorithmic_bytes": b_enc, "roofline_frac": round(b_enc / (enc_p50 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
        "decode": {"p50_us": round(dec_p50, 1), "p10_us": round(dec_p10, 1), "p90_us": round(dec_p90, 1),
                   "GBps_output": round(in_bytes / dec_p50 / 1e3, 1), "GBps_fp32_equiv": round(4 * n / dec_p50 / 1e3, 1),
                   "algorithmic_bytes": b_dec, "roofline_frac": round(b_dec / (dec_p50 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
        "unfused_p50_us": unf,
        "copy_ceiling": copy_ceiling,
        "coding": coding,
        "roofline": roof,
        "cpu_baseline": cpu,
        "configs": configs,
        "eq8": eq8,
    }
    print(json.dumps(line))


def sweep(args, np, torch, B, synth):
    """--sweep bits / reshape: see the module docstring."""
    import ctypes as C
    name = args.workload if args.workload != "c5a" or args.sweep == "bits" else "t1"
    torch.cuda.set_device(0)
    rows = []
    p50 = lambda fn: round(_p50(torch, fn)[0], 1)  # noqa: E731
    if args.sweep == "bits":
        for Q in (2, 3, 4, 6, 8):
            w = synth.workload(name, 1, q_bits=Q, mode=synth.MODE_DENSE)
            x = synth.make(w).cuda()
            n = w.numel
            pd = B.params_of(w)
            cd = B.Codec(pd, n)
            nb_d = cd.compress(x)
            hd = cd.header(nb_d)
            out = torch.empty(n, dtype=x.dtype, device="cuda")
            row = {"Q": Q, "raw_bytes": n * x.element_size(), "dense_bytes": nb_d,
                   "dense_compress_us": p50(lambda: B.rans_compress(x, n, pd, cd.stream, cd.nbytes, cd.ws)),
                   "dense_decompress_us": p50(lambda: B.rans_decompress(cd.stream, nb_d, hd, w.in_dtype, out, cd.ws))}
            if n <= 1 << 24 and n >= 4:  # the searched CSR form too (the search result comes back to the host)
                stream, p, res = B.compress_with_search(x, Q, w.freq_bits, w.n_streams, w.chunk_syms)
                sym = torch.empty(n, dtype=torch.uint8, device="cuda")
                cq = B.Codec(pd, n)
                row["quantise_us"] = p50(lambda: B.rans_quantize(x, n, pd, sym, cq.qinfo, cq.ws))
                rc, wsb = B.rans_search_workspace_bytes(n, Q)
                ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
                rr = torch.zeros(C.sizeof(B.ReshapeResult), dtype=torch.uint8, device="cuda")
                row["search_us"] = p50(lambda: B.rans_search_reshape(sym, n, Q, rr, ws))
                ce = B.Codec(p, n)
                ce.qinfo.copy_(cq.qinfo)
                row["csr_encode_us"] = p50(lambda: B.rans_encode(sym, n, p, ce.qinfo, ce.stream, ce.nbytes, ce.ws))
                nb = int(ce.nbytes.item())
                hc = ce.header(nb)
                row["csr_decompress_us"] = p50(lambda: B.rans_decompress(ce.stream, nb, hc, w.in_dtype, out, ce.ws))
                row.update({"csr_bytes": stream.numel(), "csr_rows": int(res.rows), "csr_cols": int(res.cols)})
            rows.append(row)
        print(json.dumps({"sweep": "bits", "workload": name, "rows": rows}))
        return
    res = eq8_terms(torch, B, synth, name, 30)
    res["sweep"] = "reshape"
    print(json.dumps(res))


if __name__ == "__main__":
    main()
