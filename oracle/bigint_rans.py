"""Unbounded-state rANS written directly from Eq. 2-4 (Sec. 2.1) -- TEST INFRASTRUCTURE ONLY.

Python integers never overflow, so no renormalisation is needed: the whole
message is one state.  This is the paper's coder with nothing added, and serves
as an independent check of the 32-bit, word-renormalised coder in
``rans_oracle.c``: both must decode to the same symbols, and their code lengths
must agree up to the truncation loss of the 32-bit state.
"""
from __future__ import annotations

import math
from typing import Sequence


def cumulative(f: Sequence[int]) -> list[int]:
    """F(x) = sum of f(y) for y < x, with one extra entry F(A) = sum f."""
    F = [0]
    for fx in f:
        F.append(F[-1] + int(fx))
    return F


def encode(symbols: Sequence[int], f: Sequence[int], n_bits: int, s0: int = 1 << 16) -> int:
    """Eq. 2 applied to the symbols last to first, so that decoding yields them first to last."""
    F = cumulative(f)
    assert F[-1] == 1 << n_bits
    s = s0
    for x in reversed(list(symbols)):
        fx = int(f[x])
        assert fx > 0
        s = (s // fx) * (1 << n_bits) + F[x] + (s % fx)
    return s


def decode(s: int, count: int, f: Sequence[int], n_bits: int):
    """Eq. 3 (symbol selection) and Eq. 4 (state update), ``count`` times. Returns (symbols, final state)."""
    F = cumulative(f)
    out = []
    for _ in range(count):
        slot = s % (1 << n_bits)
        x = next(t for t in range(len(f)) if F[t] <= slot < F[t + 1])
        s = int(f[x]) * (s // (1 << n_bits)) + slot - F[x]
        out.append(x)
    return out, s


def code_length_bits(s: int) -> float:
    """log2 of the final state: the information the state carries."""
    return math.log2(s) if s > 0 else 0.0
