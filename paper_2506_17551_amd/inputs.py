"""Seeded synthetic inputs for the gradient-compression workloads.

This module only DRAWS numbers and lists tensor shapes. It contains none of the
method's arithmetic (no accumulate, no selection, no quantization), so it can
serve the HIP path and the CPU oracle alike: a test generates an input once and
hands the SAME bytes to both sides.

The paper trains on a public e-commerce interaction dataset that is not
available here; nothing in this path depends on its content, only on gradient
shapes and value distributions, which the workload list below fixes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch

BASE_SEED = 20250617
_CHUNK = 1 << 27  # elements drawn per call, bounds temporaries at large n


def seed_for(config: int, worker: int = 0, step: int = 0, tensor: int = 0, stream: int = 0) -> int:
    """One independent stream per (config, worker, step, tensor, stream)."""
    x = BASE_SEED
    for v in (config, worker, step, tensor, stream):
        x = (x * 6364136223846793005 + 1442695040888963407 + int(v) * 0x9E3779B97F4A7C15) % (1 << 63)
    return x


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def normal(n: int, std: float, seed: int, device="cpu", out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """n fp32 draws from N(0, std^2)."""
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=device)
    g = _gen(seed, out.device)
    for a in range(0, n, _CHUNK):
        b = min(n, a + _CHUNK)
        out[a:b].normal_(0.0, std, generator=g)
    return out


def outlier_mixture(n: int, std: float, p_outlier: float, factor: float, seed: int, device="cpu",
                    out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """N(0, std^2) with each entry independently multiplied by `factor` with prob. p_outlier."""
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=device)
    g = _gen(seed, out.device)
    for a in range(0, n, _CHUNK):
        b = min(n, a + _CHUNK)
        sl = out[a:b]
        sl.normal_(0.0, std, generator=g)
        u = torch.empty(b - a, dtype=torch.float32, device=out.device).uniform_(0.0, 1.0, generator=g)
        sl.mul_(torch.where(u < p_outlier, float(factor), 1.0))
        del u
    return out


def student_t3(n: int, scale: float, seed: int, device="cpu", out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scale * Student-t with 3 degrees of freedom: Z / sqrt((A^2+B^2+C^2)/3)."""
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=device)
    g = _gen(seed, out.device)
    chunk = _CHUNK // 4
    for a in range(0, n, chunk):
        b = min(n, a + chunk)
        z = torch.empty((4, b - a), dtype=torch.float32, device=out.device).normal_(0.0, 1.0, generator=g)
        chi = (z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0
        out[a:b] = scale * z[0] / torch.sqrt(chi)
        del z, chi
    return out


def tie_alphabet(n: int, symbols, seed: int, device="cpu") -> torch.Tensor:
    """n fp32 values drawn uniformly from a small alphabet (forces ties, may hold +0/-0)."""
    sym = torch.tensor(list(symbols), dtype=torch.float32, device=device)
    g = _gen(seed, device)
    pick = torch.randint(0, sym.numel(), (n,), generator=g, device=device)
    return sym[pick].contiguous()


def bf16_bits(x: torch.Tensor) -> np.ndarray:
    """Bit patterns (uint16) of a torch.bfloat16 tensor, for the oracle."""
    assert x.dtype == torch.bfloat16
    return x.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def decoder_125m_shapes(context: int = 1024) -> List[Tuple[str, int]]:
    """Tensor list of a 12-layer pre-LN decoder, d=768, ffn=3072, vocab 50,257, biases,
    tied output head, learned positions (context length is an assumption): 148 tensors,
    124,439,808 parameters."""
    d, ffn, vocab, layers = 768, 3072, 50257, 12
    t = [("tok_emb", vocab * d), ("pos_emb", context * d)]
    for l in range(layers):
        t += [(f"l{l}.ln1.w", d), (f"l{l}.ln1.b", d),
              (f"l{l}.qkv.w", d * 3 * d), (f"l{l}.qkv.b", 3 * d),
              (f"l{l}.proj.w", d * d), (f"l{l}.proj.b", d),
              (f"l{l}.ln2.w", d), (f"l{l}.ln2.b", d),
              (f"l{l}.up.w", d * ffn), (f"l{l}.up.b", ffn),
              (f"l{l}.down.w", ffn * d), (f"l{l}.down.b", d)]
    t += [("lnf.w", d), ("lnf.b", d)]
    return t


def offsets_of(sizes) -> np.ndarray:
    off = np.zeros(len(sizes) + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.asarray(sizes, dtype=np.int64))
    return off


_ZIPF_CDF = {}


def _zipf_cdf(num_rows: int, s: float) -> np.ndarray:
    key = (int(num_rows), float(s))
    if key not in _ZIPF_CDF:
        w = np.arange(1, num_rows + 1, dtype=np.float64) ** (-s)
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        _ZIPF_CDF.clear()          # one table at a time (80 MB at 10M rows)
        _ZIPF_CDF[key] = cdf
    return _ZIPF_CDF[key]


def zipf_unique_rows(num_lookups: int, num_rows: int, s: float, seed: int) -> np.ndarray:
    """Sorted unique row ids hit by `num_lookups` draws from Zipf(s) over 1..num_rows
    (inverse CDF in double precision on the host)."""
    cdf = _zipf_cdf(num_rows, s)
    rng = np.random.Generator(np.random.Philox(key=int(seed) % (1 << 64)))
    u = rng.random(num_lookups)
    ids = np.searchsorted(cdf, u, side="left")
    return np.unique(np.minimum(ids, num_rows - 1)).astype(np.int64)


@dataclass
class Workload:
    """One of the five benchmark workloads: sizes only, inputs come from `grad`/`residual0`."""
    name: str
    config: int
    n: int
    density: float
    block: int
    W: int
    steps: int = 1
    grad_dtype: str = "f32"
    index_bits: int = 32
    sizes: Optional[List[int]] = None  # per-tensor sizes for the multi-tensor workloads
    note: str = ""

    def grad(self, worker: int, step: int, device, out=None) -> torch.Tensor:
        sd = seed_for(self.config, worker, step)
        if self.config == 1:
            return normal(self.n, 1.0, sd, device, out)
        if self.config == 2:
            return normal(self.n, 0.02, sd, device, out)
        if self.config == 3:
            return normal(self.n, 0.01, sd, device, out)
        if self.config == 4:
            x = student_t3(self.n, 1e-3, sd, device, out)
            return x.to(torch.bfloat16)
        if self.config == 5:
            return outlier_mixture(self.n, 1e-3, 0.01, 100.0, sd, device, out)
        raise ValueError(self.config)

    def residual0(self, worker: int, device, out=None) -> torch.Tensor:
        if self.config == 5:  # the residual is drawn from the same mixture as the gradient
            return outlier_mixture(self.n, 1e-3, 0.01, 100.0, seed_for(5, worker, 0, 0, 1), device, out)
        if out is None:
            return torch.zeros(self.n, dtype=torch.float32, device=device)
        return out.zero_()


def workload(config: int, scale: float = 1.0) -> Workload:
    """The five workloads. `scale` < 1 shrinks n (same distribution, density, block) so that the
    CPU oracle can follow; scale == 1 is the size the benchmark names."""
    def sc(n, mult=1):
        if scale >= 1.0:
            return n
        return max(mult, int(n * scale) // mult * mult)

    if config == 1:
        return Workload("flat-1M-f32", 1, sc(1 << 20), 0.01, 256, 1, steps=3)
    if config == 2:
        sizes = [sz for _, sz in decoder_125m_shapes()]
        if scale < 1.0:
            sizes = [max(1, int(sz * scale)) for sz in sizes]
        return Workload("decoder-125M-f32", 2, int(sum(sizes)), 0.001, 256, 8, sizes=sizes,
                        note="context length 1024 assumed; per-tensor top-k")
    if config == 3:
        return Workload("recsys-mlp-100M-f32", 3, sc(100_000_000), 0.01, 256, 8,
                        note="dense MLP tower part; the embedding gradient is row-sparse (touched rows of a 10M x 128 table)")
    if config == 4:
        return Workload("flat-1.3B-bf16", 4, sc(1_300_000_000, 8), 0.005, 1024, 16, steps=10,
                        grad_dtype="bf16")
    if config == 5:
        n = sc(7_000_000_000, 8)
        return Workload("flat-7B-f32", 5, n, 0.001, 2048, 16,
                        index_bits=64 if n > (1 << 32) else 32)
    raise ValueError(config)


def embedding_rows_workload(worker: int, device="cpu", step: int = 0):
    """Config 3's row-sparse embedding gradient: sorted unique rows hit by 65,536 Zipf(1.1)
    lookups over a 10M-row table, and an (U x 128) fp32 value block ~ N(0, 0.01). Every
    (worker, step) draws its own batch, so the number of touched rows changes from step to step."""
    rows = zipf_unique_rows(65536, 10_000_000, 1.1, seed_for(3, worker, step, 1))
    vals = normal(rows.shape[0] * 128, 0.01, seed_for(3, worker, step, 2), device)
    return rows, vals
