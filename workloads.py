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
