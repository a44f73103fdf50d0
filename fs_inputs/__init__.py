"""Seeded synthetic inputs for the tiered sequence-embedding lookup.

Serves both the HIP library's callers (tests, bench) and the CPU oracle's
tests.  It holds none of the method's arithmetic: it only draws jagged batches,
tables, gradients and builds placement tables in the documented bit layout
(tier in bits 31..30, owner in bits 29..0).

Everything is drawn with torch on the device asked for (CPU here, the GPU for
the large configurations), from generators seeded by (config, purpose), and is
then handed, unchanged, to whichever side consumes it.  The paper's workloads
are private production data with power-law row popularity (Section 5,
"Dataset"; Section 4.1); Zipf-over-a-random-permutation ids stand in for them.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import torch

MASTER_SEED = 2959

TIER_GLOBAL, TIER_GROUP, TIER_SHARDED = 0, 1, 2
TIER_SHIFT = 30

_TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}
ELEM_BYTES = {"f32": 4, "f16": 2, "bf16": 2}


@dataclasses.dataclass(frozen=True)
class Config:
    """One workload: T tables of E rows x D, batch B, a length law, Zipf(alpha) ids."""
    name: str
    index: int            # position in the list of configurations, seeds the streams
    T: int
    E: int
    D: int
    dtype: str            # "f32" | "f16" | "bf16"
    B: int
    length_law: str       # "fixed" | "uniform" | "geometric" | "lognormal"
    length_args: tuple
    alpha: float
    U: int
    W: int
    f_global: float       # fraction of each table's rows (by popularity rank) in tier 0
    f_group: float        # next fraction in tier 1
    self_bucket: int = 0

    @property
    def R(self) -> int:
        return self.T * self.E

    @property
    def row_bytes(self) -> int:
        return self.D * ELEM_BYTES[self.dtype]

    @property
    def torch_dtype(self):
        return _TORCH_DTYPE[self.dtype]

    def scaled(self, E: Optional[int] = None, B: Optional[int] = None, T: Optional[int] = None,
               name: Optional[str] = None) -> "Config":
        """Same laws, fewer rows / samples / tables (for runs the CPU oracle finishes fast)."""
        return dataclasses.replace(self, E=E or self.E, B=B or self.B, T=T or self.T,
                                   name=name or (self.name + "-scaled"))


CONFIGS: Dict[str, Config] = {
    "c1": Config("c1", 1, T=1, E=100_000, D=64, dtype="f32", B=256, length_law="fixed",
                 length_args=(32,), alpha=1.05, U=8, W=8, f_global=0.01, f_group=0.0),
    "c2": Config("c2", 2, T=8, E=10_000_000, D=128, dtype="f16", B=4096, length_law="uniform",
                 length_args=(1, 256), alpha=1.1, U=64, W=64, f_global=0.005, f_group=0.0),
    "c3": Config("c3", 3, T=16, E=5_000_000, D=256, dtype="bf16", B=8192, length_law="geometric",
                 length_args=(120.0, 1024), alpha=1.2, U=64, W=8, f_global=0.002, f_group=0.02),
    "c4": Config("c4", 4, T=16, E=20_000_000, D=256, dtype="f16", B=16384, length_law="lognormal",
                 length_args=(5.3, 0.8, 1, 2048), alpha=1.1, U=128, W=128, f_global=0.01, f_group=0.0),
    # c5: the planning sample is drawn by make_profile_sample; the batch below is its backward leg
    "c5": Config("c5", 5, T=4, E=50_000_000, D=128, dtype="f16", B=8192, length_law="uniform",
                 length_args=(1, 512), alpha=1.3, U=64, W=64, f_global=0.0, f_group=0.0),
}


def _generator(cfg: Config, purpose: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((MASTER_SEED * 1_000_003 + cfg.index * 10_007 + purpose) & 0x7FFFFFFFFFFF)
    return g


def make_lengths(cfg: Config, device="cpu") -> torch.Tensor:
    """Sequence length of each of the T*B segments (int64)."""
    S = cfg.T * cfg.B
    gen = _generator(cfg, 1, device)
    law, a = cfg.length_law, cfg.length_args
    if law == "fixed":
        return torch.full((S,), int(a[0]), dtype=torch.int64, device=device)
    if law == "uniform":
        lo, hi = a
        return torch.randint(lo, hi + 1, (S,), generator=gen, device=device, dtype=torch.int64)
    if law == "geometric":
        mean, cap = a
        u = torch.rand(S, generator=gen, device=device, dtype=torch.float64).clamp_min(1e-300)
        ln = 1 + torch.floor(torch.log(u) / math.log(1.0 - 1.0 / mean))
        return ln.clamp_max(cap).to(torch.int64)
    if law == "lognormal":
        mu, sigma, lo, hi = a
        z = torch.randn(S, generator=gen, device=device, dtype=torch.float64)
        return torch.round(torch.exp(mu + sigma * z)).clamp(lo, hi).to(torch.int64)
    raise ValueError(law)


class ZipfTable:
    """Finite Zipf over ranks 1..E, P(r) ~ r^-alpha, drawn by inverse CDF; id = perm[rank - 1]."""

    def __init__(self, E: int, alpha: float, gen: torch.Generator, device):
        r = torch.arange(1, E + 1, dtype=torch.float64, device=device)
        self.cdf = torch.cumsum(r.pow_(-alpha), 0)
        self.total = float(self.cdf[-1])
        self.perm = torch.randperm(E, generator=gen, device=device)
        self.E = E

    def draw(self, count: int, gen: torch.Generator) -> torch.Tensor:
        u = torch.rand(count, generator=gen, device=self.cdf.device, dtype=torch.float64) * self.total
        rank = torch.searchsorted(self.cdf, u, right=True).clamp_max_(self.E - 1)
        return self.perm[rank]


def make_batch(cfg: Config, device="cpu", keep_perms: bool = True) -> dict:
    """Jagged batch: ids[n] (table-local), offsets[T*B+1], row_base[T+1]; plus the
    popularity permutations perms[t] (rank -> table-local id) used to tag tiers."""
    lengths = make_lengths(cfg, device)
    offsets = torch.zeros(cfg.T * cfg.B + 1, dtype=torch.int64, device=device)
    torch.cumsum(lengths, 0, out=offsets[1:])
    n = int(offsets[-1])
    ids = torch.empty(n, dtype=torch.int64, device=device)
    perms: List[torch.Tensor] = []
    for t in range(cfg.T):
        gen = _generator(cfg, 100 + t, device)
        z = ZipfTable(cfg.E, cfg.alpha, gen, device)
        lo, hi = int(offsets[t * cfg.B]), int(offsets[(t + 1) * cfg.B])
        ids[lo:hi] = z.draw(hi - lo, gen)
        perms.append(z.perm if keep_perms else z.perm[: max(1, int((cfg.f_global + cfg.f_group) * cfg.E))].clone())
        del z
    row_base = torch.arange(cfg.T + 1, dtype=torch.int64, device=device) * cfg.E
    return {"ids": ids, "offsets": offsets, "row_base": row_base, "perms": perms, "n": n}


def make_placement(cfg: Config, perms: List[torch.Tensor], device="cpu") -> torch.Tensor:
    """placement[R] as int32 bit patterns (reinterpret as uint32).  Per table, by popularity
    rank: the first f_global*E rows are tier 0, the next f_group*E tier 1 (owner = id mod W),
    the rest tier 2 (owner = id mod U)."""
    out = torch.empty(cfg.R, dtype=torch.int32, device=device)
    n0 = int(cfg.f_global * cfg.E)
    n1 = int(cfg.f_group * cfg.E)
    for t in range(cfg.T):
        local = torch.arange(cfg.E, dtype=torch.int64, device=device)
        entry = (TIER_SHARDED << TIER_SHIFT) | (local % cfg.U)
        if n1 > 0:
            rows1 = perms[t][n0:n0 + n1]
            entry[rows1] = (TIER_GROUP << TIER_SHIFT) | (rows1 % cfg.W)
        if n0 > 0:
            rows0 = perms[t][:n0]
            entry[rows0] = (TIER_GLOBAL << TIER_SHIFT)
        out[t * cfg.E:(t + 1) * cfg.E] = entry.to(torch.int32)   # wraps: bit pattern kept
    return out


def make_table(cfg: Config, device="cpu", std: float = 0.1, purpose: int = 7,
               rows: Optional[int] = None) -> torch.Tensor:
    """Embedding table [R, D] ~ N(0, std^2) in the config's dtype, drawn in chunks."""
    R = cfg.R if rows is None else rows
    return _normal((R, cfg.D), cfg.torch_dtype, std, _generator(cfg, purpose, device), device)


def make_grad(cfg: Config, n: int, device="cpu") -> torch.Tensor:
    """Upstream gradient [n, D] ~ N(0, 1) in the table's dtype."""
    return _normal((n, cfg.D), cfg.torch_dtype, 1.0, _generator(cfg, 9, device), device)


def _normal(shape, dtype, std, gen, device, chunk_elems: int = 1 << 28) -> torch.Tensor:
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    total = flat.numel()
    for lo in range(0, total, chunk_elems):
        hi = min(total, lo + chunk_elems)
        flat[lo:hi] = (torch.randn(hi - lo, generator=gen, device=device, dtype=torch.float32) * std).to(dtype)
    return out


def make_profile_sample(cfg: Config, per_table: int, device="cpu", chunk: int = 1 << 26):
    """Profiling sample for the replication plan: `per_table` ids per table, one segment per
    table (B = 1).  Yields (t, ids_chunk) so a billion ids need not be resident at once."""
    for t in range(cfg.T):
        gen = _generator(cfg, 100 + t, device)
        z = ZipfTable(cfg.E, cfg.alpha, gen, device)
        gen2 = _generator(cfg, 500 + t, device)
        done = 0
        while done < per_table:
            c = min(chunk, per_table - done)
            yield t, z.draw(c, gen2)
            done += c
        del z


def as_numpy_bits(t: torch.Tensor):
    """Host numpy view of a tensor; bfloat16 comes back as its uint16 bit pattern."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
