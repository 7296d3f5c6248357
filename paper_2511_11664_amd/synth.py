"""Seeded synthetic activation tensors shaped like the paper's workloads.

The paper measures on real intermediate features (ResNet / VGG16 / SwinT on
CIFAR100 and ImageNet, Llama2 hidden states on seven NLP suites, Sec. 4.1);
none of those models or datasets ship with this repository, so these
generators stand in for them: same shapes, similar sparsity and value
distributions.  This module only draws numbers -- it holds none of the codec's
arithmetic -- and is the single source of inputs for the tests, the smoke check
and the benchmark, for both the CPU oracle and the GPU library.

All tensors are generated on the CPU with ``torch.Generator().manual_seed``.
``shrink`` divides the leading (batch) dimension so that parity tests can use
the same recipe at a size the oracle finishes in seconds.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch

MODE_DENSE, MODE_CSR = 0, 1
F32, F16 = 0, 1


@dataclass
class Workload:
    name: str
    shape: tuple
    dtype: torch.dtype
    seed: int
    q_bits: int
    freq_bits: int
    n_streams: int
    chunk_syms: int
    mode: int
    cols: int                      # K of the reshape; rows = numel // cols
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def numel(self) -> int:
        n = 1
        for d in self.shape:
            n *= d
        return n

    @property
    def rows(self) -> int:
        return self.numel // self.cols

    @property
    def in_dtype(self) -> int:
        return F16 if self.dtype == torch.float16 else F32


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def _c1(shape, g):
    # post-ReLU unit normal: about half exact zeros
    return torch.relu(torch.randn(shape, generator=g))


def _c2(shape, g):
    # ResNet-style post-ReLU features: ReLU(N(0, 0.5)) and 40 % of the entries
    # dropped on top, so that about 70 % of all entries are exact zeros
    x = torch.relu(0.5 * torch.randn(shape, generator=g))
    keep = torch.rand(shape, generator=g) < 0.6
    return x * keep


def _c3(shape, g):
    # VGG16-style: ReLU(N(-0.3, 1)) with a per-channel scale U(0.2, 3) on dim 1
    x = torch.relu(torch.randn(shape, generator=g) - 0.3)
    scale = 0.2 + 2.8 * torch.rand(shape[1], generator=g)
    view = [1] * len(shape)
    view[1] = shape[1]
    return x * scale.view(view)


def _c4(shape, g):
    # SwinT-style token features: exact-erf GELU of a unit normal (dense, small negative tail)
    return torch.nn.functional.gelu(torch.randn(shape, generator=g))


def _c5(shape, g):
    # Llama2-style hidden states: unit normal, 1 % of the hidden channels scaled x20, stored as fp16
    x = torch.randn(shape, generator=g)
    hidden = shape[-1]
    k = max(1, hidden // 100)
    idx = torch.randperm(hidden, generator=g)[:k]
    x[..., idx] *= 20.0
    return x.to(torch.float16)


_RECIPES = {
    # name: (full shape, dtype, seed, fn, Q, M, S, chunk_syms, mode, cols)
    # The post-ReLU (sparse) tensors default to the paper's own path, the modified CSR of Sec. 3.1, with the
    # reshape their configuration names; the dense ones (GELU tokens, hidden states) to D = xhat.
    # c1 as configured: reshape 64 x 3136, 32 streams, all of D in one chunk
    "c1": ((1, 64, 56, 56), torch.float32, 0, _c1, 8, 12, 32, 0, MODE_CSR, 3136),
    # the shape of the features in the paper's Table 1 (128 x 28 x 28 fp32, 401 408 bytes), post-ReLU
    "t1": ((1, 128, 28, 28), torch.float32, 6, _c1, 8, 12, 64, 64 * 64, MODE_DENSE, 784),
    # c2: the configured "rows = 256" would need 100 352 column symbols (more than the 65 535 a 16-bit symbol
    # allows, and than any 2^12 table holds); it is run as N x 256 instead
    "c2": ((32, 256, 56, 56), torch.float32, 1, _c2, 8, 12, 1024, 80 * 1024, MODE_CSR, 256),
    "c3": ((64, 512, 28, 28), torch.float32, 2, _c3, 8, 14, 1024, 80 * 1024, MODE_CSR, 256),
    "c4": ((16, 3136, 96), torch.float32, 3, _c4, 8, 12, 1024, 1 << 18, MODE_DENSE, 96),
    "c5a": ((8, 2048, 4096), torch.float16, 4, _c5, 8, 14, 1024, 1 << 18, MODE_DENSE, 4096),
    "c5b": ((8, 2048, 5120), torch.float16, 5, _c5, 8, 14, 1024, 320 * 1024, MODE_DENSE, 5120),  # 256 chunks: one per CU
}

# The rows of the benchmark's per-configuration table: (label, recipe, overrides).  The full-size parity tests
# run the same list, so every reported row is also compared with the oracle byte by byte.
BENCH_CONFIGS = (
    ("c1_csr3136_onechunk", "c1", {}),                                        # the configuration as written
    ("c1_csr7", "c1", dict(cols=7, chunk_syms=2048)),                         # a reshape of the paper's search domain
    ("c1_dense_onechunk", "c1", dict(mode=MODE_DENSE)),
    ("c1_dense", "c1", dict(mode=MODE_DENSE, chunk_syms=2048)),
    ("t1_dense", "t1", {}),
    ("t1_csr4", "t1", dict(mode=MODE_CSR, cols=4)),
    ("c2_csr256", "c2", {}),
    ("c2_csr7", "c2", dict(cols=7, chunk_syms=80 * 1024)),
    ("c2_csr4", "c2", dict(cols=4, chunk_syms=96 * 1024)),  # l_D = 21.8 M: 223 chunks, one round of the decoder
    ("c2_dense", "c2", dict(mode=MODE_DENSE, chunk_syms=100352)),
    ("c3_csr256_q8", "c3", {}),
    ("c3_csr64_q6", "c3", dict(q_bits=6, cols=64)),
    ("c3_dense_q8", "c3", dict(mode=MODE_DENSE, chunk_syms=1 << 18)),
    ("c3_dense_q6", "c3", dict(mode=MODE_DENSE, q_bits=6, chunk_syms=1 << 18)),
    ("c4_dense", "c4", {}),
    ("c4_dense_cs18432", "c4", dict(chunk_syms=18432)),
    ("c5a_dense", "c5a", {}),
    ("c5b_dense", "c5b", {}),
)

NAMES = tuple(_RECIPES)


def workload(name: str, shrink: int = 1, **over) -> Workload:
    """Describe a workload; keyword overrides replace codec parameters (mode, cols, q_bits, ...)."""
    shape, dtype, seed, _, q, m, s, cs, mode, cols = _RECIPES[name]
    shape = (max(1, shape[0] // shrink),) + tuple(shape[1:])
    if name == "c1" and shrink > 1:
        shape = (1, max(1, 64 // shrink), 56, 56)
    if name == "t1" and shrink > 1:
        shape = (1, max(1, 128 // shrink), 28, 28)
    w = Workload(name=name, shape=shape, dtype=dtype, seed=seed, q_bits=q, freq_bits=m, n_streams=s,
                 chunk_syms=cs, mode=mode, cols=cols)
    for k, v in over.items():
        setattr(w, k, v)
    assert w.numel % w.cols == 0, "cols must divide the element count"
    return w


def make(w: Workload) -> torch.Tensor:
    """Generate the tensor of a workload on the CPU (flat, contiguous)."""
    fn = _RECIPES[w.name][3]
    return fn(w.shape, _gen(w.seed)).contiguous().view(-1)
