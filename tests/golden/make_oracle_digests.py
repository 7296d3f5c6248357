"""Writes tests/golden/oracle_container_digests.txt: SHA-256 of the oracle's container for a few small inputs
given by closed formulas (no random generator), so that an unintended change of the oracle's arithmetic or of
the container layout (the readings of the paper listed with the oracle) shows up as a changed digest.
Calls only the oracle.  Run from the repository root:  python tests/golden/make_oracle_digests.py
"""
import hashlib
import os
import sys

import numpy as np

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", ".."))
import oracle  # noqa: E402


def cases():
    """(name, tensor, q_bits, freq_bits, rows, cols, mode, n_streams, chunk_syms)"""
    # integer hashes only (exact in every arithmetic): two 12-bit values per index, their sum is triangular
    i = np.arange(6000, dtype=np.uint64)
    h1 = ((i * np.uint64(2654435761)) % np.uint64(1 << 32)) >> np.uint64(20)
    h2 = (((i + np.uint64(12345)) * np.uint64(40503)) % np.uint64(1 << 16)) >> np.uint64(4)
    wave = ((h1 + h2).astype(np.float64) / 512.0 - 8.0).astype(np.float32)   # multiples of 2^-9 in [-8, 8)
    relu = np.maximum(wave - 1.0, 0.0).astype(np.float32)
    saw = ((i % np.uint64(97)).astype(np.float64) / 8.0 - 3.0).astype(np.float16)
    return [
        ("dense_f32_q8_m12_s32_onechunk", wave, 8, 12, 6000, 1, oracle.MODE_DENSE, 32, 0),
        ("dense_f32_q8_m12_s32_chunks", wave, 8, 12, 6000, 1, oracle.MODE_DENSE, 32, 640),
        ("dense_f16_q6_m14_s64", saw, 6, 14, 6000, 1, oracle.MODE_DENSE, 64, 1280),
        ("dense_f32_q2_m8_s5", relu, 2, 8, 6000, 1, oracle.MODE_DENSE, 5, 50),
        ("csr_f32_q8_m12_100x60_s32", relu, 8, 12, 100, 60, oracle.MODE_CSR, 32, 0),
        ("csr_f32_q4_m10_1500x4_s16_chunks", relu, 4, 10, 1500, 4, oracle.MODE_CSR, 16, 160),
        ("csr_f16_q8_m13_12x500_s64", relu.astype(np.float16), 8, 13, 12, 500, oracle.MODE_CSR, 64, 1280),
        ("constant_f32", np.full(1000, -2.5, np.float32), 8, 12, 1000, 1, oracle.MODE_DENSE, 8, 0),
        ("empty_csr", np.zeros(0, np.float32), 8, 12, 0, 4, oracle.MODE_CSR, 32, 0),
    ]


def digests():
    out = []
    for name, x, q, m, rows, cols, mode, s, cs in cases():
        dt = oracle.F16 if x.dtype == np.float16 else oracle.F32
        p = oracle.make_params(q, m, rows, cols, mode, s, cs, dt)
        buf, _ = oracle.compress(x, p)
        out.append((name, len(buf), hashlib.sha256(buf).hexdigest()))
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_container_digests.txt")
    with open(path, "w") as f:
        f.write("# name, container bytes, SHA-256 of the oracle's container; written by make_oracle_digests.py\n")
        f.write("# (format and arithmetic are this build's readings of Sec. 2.1 and Sec. 3.1: Eq. 2-7)\n")
        for name, n, h in digests():
            f.write(f"{name} {n} {h}\n")
    print(open(path).read())
