"""Seeded synthetic inputs for example-selection tests and benchmarks.

This module only *makes inputs*: clustered unit embeddings, utilities, validity
masks and queries.  It holds none of the search arithmetic and is imported by
the tests and the benchmark, which hand the same arrays to the GPU library and
to the CPU reference.

The pools stand in for embedded request/response pools such as those the
IC-Cache paper evaluates (Table 1: 7.5 k to 0.8 M examples; Sec. 2.3: most
requests have a neighbour with cosine above 0.8).  Nothing of those datasets is
used.  Recipe:

* ``C`` cluster centres: unit vectors, directions of i.i.d. Gaussians.
* a row picks a cluster (uniform, or Zipf with exponent ``zipf`` over cluster
  rank) and is ``normalize(centre + sigma * g / sqrt(d))`` with ``g`` standard
  normal, so the noise has norm ~``sigma`` and same-cluster cosines sit near
  ``1 / (1 + sigma^2)`` (0.917 for sigma = 0.3); cross-cluster cosines are
  ~``N(0, 1/d)``.
* queries are drawn the same way (requests and cached examples come from one
  stream).
* utility: none, Uniform[0,1], or Beta(2,5) taken as the 2nd smallest of six
  uniforms; mask: Bernoulli(``p_valid``) per row, 1 = valid.

Values are a pure function of (config seed, stream, block index, device type):
rows are produced in fixed blocks of ``BLOCK`` rows, each from its own seeded
``torch.Generator``, so any row range can be regenerated without the rest.  CPU
and GPU generators give different values for one seed; a test generates once on
one device and copies.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Optional, Tuple

import torch

BLOCK = 65536

_STREAM_CENTRES, _STREAM_ROWS, _STREAM_QUERIES, _STREAM_UTIL, _STREAM_MASK = range(5)


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    N: int
    d: int
    clusters: int
    Q: int
    k: int
    store: str = "bf16"          # "bf16" | "fp8"
    zipf: float = 0.0            # 0 = uniform over clusters
    sigma: float = 0.3
    lam: float = 0.0
    util: str = "none"           # "none" | "uniform" | "beta25"
    p_valid: float = 1.0         # 1.0 = no mask
    seed: int = 0

    def scaled(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations.
C1 = Config("C1", N=100_000, d=384, clusters=256, Q=64, k=10, seed=126891)
C2 = Config("C2", N=1_000_000, d=768, clusters=1024, Q=256, k=32, lam=0.1, util="uniform",
            p_valid=0.95, seed=126892)
C3 = Config("C3", N=10_000_000, d=768, clusters=4096, Q=64, k=64, zipf=1.1, seed=126893)
C4 = Config("C4", N=4_000_000, d=1024, clusters=2048, Q=4096, k=16, lam=0.2, util="beta25",
            p_valid=0.90, seed=126894)
C5 = Config("C5", N=20_000_000, d=1024, clusters=8192, Q=64, k=100, store="fp8", zipf=1.1,
            seed=126895)
CONFIGS = {c.name: c for c in (C1, C2, C3, C4, C5)}


def _gen(cfg: Config, stream: int, block: int, device: torch.device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((cfg.seed * 1_000_003 + stream) * 1_000_033 + block)
    return g


class Workload:
    """Row/query factory for one configuration on one device."""

    def __init__(self, cfg: Config, device="cpu"):
        self.cfg = cfg
        self.device = torch.device(device)
        g = _gen(cfg, _STREAM_CENTRES, 0, self.device)
        c = torch.randn(cfg.clusters, cfg.d, generator=g, device=self.device, dtype=torch.float32)
        self.centres = c / c.norm(dim=1, keepdim=True)
        if cfg.zipf > 0:
            w = torch.arange(1, cfg.clusters + 1, dtype=torch.float64) ** (-cfg.zipf)
        else:
            w = torch.ones(cfg.clusters, dtype=torch.float64)
        cdf = torch.cumsum(w / w.sum(), 0)
        cdf[-1] = 1.0
        self.cdf = cdf.to(torch.float32).to(self.device)

    # -- helpers -----------------------------------------------------------
    def _draw(self, stream: int, block: int, n: int) -> torch.Tensor:
        cfg = self.cfg
        g = _gen(cfg, stream, block, self.device)
        u = torch.rand(n, generator=g, device=self.device, dtype=torch.float32)
        cl = torch.searchsorted(self.cdf, u).clamp_(max=cfg.clusters - 1)
        noise = torch.randn(n, cfg.d, generator=g, device=self.device, dtype=torch.float32)
        x = self.centres[cl] + noise * (cfg.sigma / math.sqrt(cfg.d))
        return x / x.norm(dim=1, keepdim=True)

    def _block(self, b: int):
        cfg = self.cfg
        E = self._draw(_STREAM_ROWS, b, BLOCK)
        U = None
        if cfg.util == "uniform":
            g = _gen(cfg, _STREAM_UTIL, b, self.device)
            U = torch.rand(BLOCK, generator=g, device=self.device, dtype=torch.float32)
        elif cfg.util == "beta25":
            g = _gen(cfg, _STREAM_UTIL, b, self.device)
            six = torch.rand(BLOCK, 6, generator=g, device=self.device, dtype=torch.float32)
            U = six.sort(dim=1).values[:, 1].contiguous()
        M = None
        if cfg.p_valid < 1.0:
            g = _gen(cfg, _STREAM_MASK, b, self.device)
            M = (torch.rand(BLOCK, generator=g, device=self.device) < cfg.p_valid).to(torch.uint8)
        return E, U, M

    # -- public ------------------------------------------------------------
    def rows(self, start: int, n: int) -> Tuple[torch.Tensor, Optional[torch.Tensor], Optional[torch.Tensor]]:
        """Rows [start, start+n): (E fp32 [n,d], U fp32 [n] | None, mask u8 [n] | None)."""
        assert 0 <= start and n >= 0
        Es, Us, Ms = [], [], []
        b0, b1 = start // BLOCK, (start + n + BLOCK - 1) // BLOCK
        for b in range(b0, max(b1, b0)):
            lo = max(start, b * BLOCK) - b * BLOCK
            hi = min(start + n, (b + 1) * BLOCK) - b * BLOCK
            E, U, M = self._block(b)
            Es.append(E[lo:hi])
            if U is not None:
                Us.append(U[lo:hi])
            if M is not None:
                Ms.append(M[lo:hi])
        if not Es:
            E = torch.empty(0, self.cfg.d, device=self.device)
            U = torch.empty(0, device=self.device) if self.cfg.util != "none" else None
            M = torch.empty(0, dtype=torch.uint8, device=self.device) if self.cfg.p_valid < 1 else None
            return E, U, M
        E = torch.cat(Es).contiguous()
        U = torch.cat(Us).contiguous() if Us else None
        M = torch.cat(Ms).contiguous() if Ms else None
        return E, U, M

    def queries(self, Q: Optional[int] = None, batch: int = 0) -> torch.Tensor:
        """Query batch number ``batch``: fp32 [Q,d], unit rows near cluster centres."""
        Q = self.cfg.Q if Q is None else Q
        return self._draw(_STREAM_QUERIES, batch, Q).contiguous()


# ---------------------------------------------------------------------------------------------
# Rows that land exactly on rounding ties of the store formats.
# ---------------------------------------------------------------------------------------------

def _two_squares(n: int):
    a = math.isqrt(n)
    while a * a * 2 >= n:
        b2 = n - a * a
        b = math.isqrt(b2)
        if b * b == b2:
            return a, b
        a -= 1
    return None


def _four_squares(n: int, limit: int):
    """Non-negative integers (a, b, c, e), each <= limit, with a^2 + b^2 + c^2 + e^2 == n (Lagrange)."""
    a = min(math.isqrt(n), limit)
    while a >= 0:
        r1 = n - a * a
        b = min(math.isqrt(r1), limit)
        while b >= 0 and 3 * b * b >= r1:      # b is the largest of the remaining three
            two = _two_squares(r1 - b * b)
            if two and max(two) <= limit:
                return a, b, two[0], two[1]
            b -= 1
        a -= 1
    raise ValueError(f"no decomposition of {n} within {limit}")


def tie_rows(fmt: str, n: int, d: int, seed: int) -> torch.Tensor:
    """fp32 rows [n, d] with integer entries (times a power of two per row) whose Euclidean norm is
    an exact power of two, so that every ``x / |x|`` is exact in binary, and many of which sit exactly
    half-way between two neighbouring codes of the store format ``fmt``:

    * ``"bf16"``: entries ``m * 2^e`` with ``m`` odd in [257, 511] (a 9-bit significand, one bit more than
      bfloat16 keeps) in a row of norm 4096;
    * ``"fp8"``: a row of norm 1024 whose largest magnitude is 448, so the per-row scale is exactly
      2^-10 and ``unit / scale`` is the integer entry itself; entries ``m * 2^e`` with ``m`` odd in
      [17, 31] (a 5-bit significand, one more than E4M3 keeps).

    Both rounding directions occur (the neighbour with the even last bit lies below for some entries,
    above for others).  The rest of the row is what makes the sum of squares come out, then zeros.
    """
    assert fmt in ("bf16", "fp8") and d >= 32
    rng = torch.Generator().manual_seed(seed)
    ri = lambda lo, hi: int(torch.randint(lo, hi + 1, (1,), generator=rng))   # inclusive
    rows = torch.zeros(n, d, dtype=torch.float64)
    for i in range(n):
        if fmt == "bf16":
            target, limit, vals = 4096 ** 2, 4096, []
            tie = lambda: (2 * ri(128, 255) + 1) << ri(0, 2)
        else:
            target, limit, vals = 1024 ** 2, 448, [448, 448, 448, 448]
            tie = lambda: min((2 * ri(8, 15) + 1) << ri(0, 4), 432)   # 27 * 16: the largest tie below 448
        rem = target - sum(v * v for v in vals)
        floor_rem = 20_000 if fmt == "fp8" else 200_000
        while len(vals) < d - 4:
            t = tie()
            if rem - t * t < floor_rem:
                if fmt == "fp8" and rem > limit * limit:
                    continue       # what is left has to fit four entries of at most 448
                break
            vals.append(t)
            rem -= t * t
        vals.extend(_four_squares(rem, limit))
        assert sum(v * v for v in vals) == target and len(vals) <= d
        v = torch.tensor(vals, dtype=torch.float64)
        v = v * (torch.randint(0, 2, (len(vals),), generator=rng).to(torch.float64) * 2 - 1)
        pos = torch.randperm(d, generator=rng)[: len(vals)]
        rows[i, pos] = v * 2.0 ** ri(-3, 3)
    return rows.to(torch.float32)
