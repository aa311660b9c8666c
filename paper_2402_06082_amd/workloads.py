"""Seeded synthetic input generators for the SubGen decode path.

This module holds no arithmetic of the method: it only draws keys, values and
queries.  Both the HIP library (through the binding) and the CPU oracle (in
tests) are fed the bytes produced here, so neither depends on the other.

The generators imitate the structure the paper reports for LLM caches
(Section 3.1: keys cluster, values do not, rotary embeddings make key
clusters drift over time): per stream, keys are a mixture of isotropic
Gaussians around random centers, values are unstructured Gaussians with a
per-token scale, queries are N(0, I)/sqrt(d).  They stand in for the model
caches of the paper's experiments, which are not available here.

Tokens are produced in fixed blocks of ``BLOCK`` positions, each block seeded
by (seed, block index), so any range [t0, t1) is reproducible regardless of
how a caller chunks its requests.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import torch

BLOCK = 256            # token positions per random-number block
DRIFT_PERIOD = 1024    # tokens between two random-walk steps of the mixture centers


@dataclass(frozen=True)
class Config:
    name: str
    batch: int
    layers: int
    kv_heads: int
    g: int                 # queries per KV stream
    d: int
    dtype: str             # "fp32" | "bf16"
    prefix: int            # tokens ingested before decoding
    decode_steps: int
    s: int                 # sample budget
    w: int                 # recent window
    components: int        # mixture components per stream
    norm_mode: str         # "halfnormal4": 4*abs(N(0,1)); "normal8": N(8,1)
    sigma: float           # within-component std
    weights: str           # "uniform" | "zipf1.1"
    value_scale: str       # "none" | "lognormal0.5"
    drift: float = 0.0     # per-coordinate std of the center random walk per DRIFT_PERIOD tokens
    delta: Optional[float] = None      # fixed threshold, or None: tuned to target_centers
    target_centers: Optional[int] = None
    data_seed: int = 0

    @property
    def streams(self) -> int:
        return self.batch * self.layers * self.kv_heads

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "fp32" else torch.bfloat16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


# The five workloads of the benchmark definition (+ a companion of the first
# one whose threshold makes tokens merge, so the join branch is exercised at
# that size).
CONFIGS = {
    "cfg1": Config("cfg1", 1, 1, 1, 1, 64, "fp32", 1024, 256, 64, 32, 16, "halfnormal4", 0.3, "uniform", "none",
                   delta=1.0, data_seed=0),
    "cfg1b": Config("cfg1b", 1, 1, 1, 1, 64, "fp32", 1024, 256, 64, 32, 16, "halfnormal4", 0.3, "uniform", "none",
                    delta=3.6, data_seed=0),
    "cfg2": Config("cfg2", 1, 1, 32, 1, 128, "bf16", 4096, 512, 256, 64, 64, "normal8", 0.5, "zipf1.1",
                   "lognormal0.5", target_centers=300, data_seed=1),
    "cfg3": Config("cfg3", 8, 32, 32, 1, 128, "bf16", 16384, 256, 512, 128, 128, "normal8", 0.5, "zipf1.1",
                   "lognormal0.5", target_centers=600, data_seed=2),
    "cfg4": Config("cfg4", 4, 32, 32, 1, 128, "bf16", 131072, 128, 1024, 256, 512, "normal8", 0.5, "zipf1.1",
                   "lognormal0.5", drift=0.01, target_centers=2400, data_seed=3),
    "cfg5": Config("cfg5", 32, 32, 8, 4, 128, "bf16", 32768, 256, 512, 128, 128, "normal8", 0.5, "zipf1.1",
                   "lognormal0.5", target_centers=600, data_seed=4),
}


def _mix(*xs: int) -> int:
    """Deterministic 63-bit seed from a tuple of small integers (splitmix-style)."""
    h = 0x9E3779B97F4A7C15
    for x in xs:
        h ^= (int(x) + 0x9E3779B97F4A7C15 + ((h << 6) & 0xFFFFFFFFFFFFFFFF) + (h >> 2)) & 0xFFFFFFFFFFFFFFFF
        h = (h * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        h ^= h >> 31
    return h & 0x7FFFFFFFFFFFFFFF


class Workload:
    """Synthetic streams for one config on one device.

    ``streams`` overrides the config's stream count (tests use a few streams
    of a large config's shape).
    """

    def __init__(self, cfg: Config, device="cpu", streams: Optional[int] = None):
        self.cfg = cfg
        self.device = torch.device(device)
        self.S = int(streams) if streams is not None else cfg.streams
        g = self._gen("centers")
        S, Cn, d = self.S, cfg.components, cfg.d
        direction = torch.randn(S, Cn, d, generator=g, device=self.device)
        direction = direction / direction.norm(dim=-1, keepdim=True)
        z = torch.randn(S, Cn, 1, generator=g, device=self.device)
        if cfg.norm_mode == "halfnormal4":
            norm = 4.0 * z.abs()
        elif cfg.norm_mode == "normal8":
            norm = 8.0 + z
        else:
            raise ValueError(cfg.norm_mode)
        self.centers0 = direction * norm
        if cfg.weights == "uniform":
            wts = torch.ones(Cn)
        elif cfg.weights == "zipf1.1":
            wts = torch.arange(1, Cn + 1, dtype=torch.float64).pow(-1.1).float()
        else:
            raise ValueError(cfg.weights)
        self.weights = (wts / wts.sum()).to(self.device)
        self._drift_epoch = 0
        self._drift_centers = self.centers0

    def _gen(self, kind: str, idx: int = 0) -> torch.Generator:
        g = torch.Generator(device=self.device)
        g.manual_seed(_mix(self.cfg.data_seed, sum(ord(c) << (8 * i) for i, c in enumerate(kind[:6])), idx))
        return g

    def _centers_at(self, epoch: int) -> torch.Tensor:
        if self.cfg.drift == 0.0 or epoch == 0:
            return self.centers0
        if epoch < self._drift_epoch:
            self._drift_epoch, self._drift_centers = 0, self.centers0
        while self._drift_epoch < epoch:
            self._drift_epoch += 1
            g = self._gen("drift", self._drift_epoch)
            step = torch.randn(self.centers0.shape, generator=g, device=self.device)
            self._drift_centers = self._drift_centers + self.cfg.drift * step
        return self._drift_centers

    def _block(self, b: int) -> Tuple[torch.Tensor, torch.Tensor]:
        cfg, S, d = self.cfg, self.S, self.cfg.d
        g = self._gen("kv", b)
        comp = torch.multinomial(self.weights.expand(S, -1), BLOCK, replacement=True, generator=g)
        centers = self._centers_at((b * BLOCK) // DRIFT_PERIOD)
        mean = torch.gather(centers, 1, comp.unsqueeze(-1).expand(S, BLOCK, d))
        K = mean + cfg.sigma * torch.randn(S, BLOCK, d, generator=g, device=self.device)
        V = torch.randn(S, BLOCK, d, generator=g, device=self.device)
        if cfg.value_scale == "lognormal0.5":
            V = V * torch.exp(0.5 * torch.randn(S, BLOCK, 1, generator=g, device=self.device))
        return K.to(cfg.torch_dtype), V.to(cfg.torch_dtype)

    def tokens(self, t0: int, t1: int) -> Tuple[torch.Tensor, torch.Tensor]:
        """Keys and values of token positions [t0, t1): two [S, t1-t0, d] tensors in the config dtype."""
        assert 0 <= t0 <= t1
        Ks, Vs = [], []
        for b in range(t0 // BLOCK, (t1 + BLOCK - 1) // BLOCK if t1 > t0 else t0 // BLOCK):
            K, V = self._block(b)
            lo, hi = max(t0 - b * BLOCK, 0), min(t1 - b * BLOCK, BLOCK)
            Ks.append(K[:, lo:hi])
            Vs.append(V[:, lo:hi])
        if not Ks:
            e = torch.empty(self.S, 0, self.cfg.d, dtype=self.cfg.torch_dtype, device=self.device)
            return e, e.clone()
        return torch.cat(Ks, 1).contiguous(), torch.cat(Vs, 1).contiguous()

    def queries(self, t0: int, t1: int) -> torch.Tensor:
        """Queries for decode positions [t0, t1): [S, t1-t0, g, d], N(0, I)/sqrt(d) in the config dtype."""
        cfg = self.cfg
        out = []
        for b in range(t0 // BLOCK, (t1 + BLOCK - 1) // BLOCK if t1 > t0 else t0 // BLOCK):
            g = self._gen("q", b)
            Q = torch.randn(self.S, BLOCK, cfg.g, cfg.d, generator=g, device=self.device) / (cfg.d ** 0.5)
            lo, hi = max(t0 - b * BLOCK, 0), min(t1 - b * BLOCK, BLOCK)
            out.append(Q[:, lo:hi].to(cfg.torch_dtype))
        if not out:
            return torch.empty(self.S, 0, cfg.g, cfg.d, dtype=cfg.torch_dtype, device=self.device)
        return torch.cat(out, 1).contiguous()


def clusterable_streams(streams: int, n: int, d: int, m: int, delta: float, r: float, g: int = 1, seed: int = 0,
                        device="cpu", dtype=torch.float32, center_norm: float = 0.0):
    """Streams whose keys are (m, delta)-clusterable in the sense of Definition 1 of the paper.

    Per stream: m centers of norm ``center_norm`` (default 4*delta) in random directions; every key lies within
    0.45*delta of its center, so two keys of one cluster are at most 0.9*delta apart (the slack absorbs the
    rounding to ``dtype``); cluster membership is uniform.  Values are N(0, I) with a per-token log-normal
    scale, queries have norm r (scaled by 1 - 2^-7 so that rounding cannot push them above r).
    Returns K [S, n, d], V [S, n, d], Q [S, g, d] in ``dtype`` and the membership [S, n] (int64).
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(_mix(seed, 0xC1, streams, n, d, m))
    cn = center_norm if center_norm > 0.0 else 4.0 * delta
    cent = torch.randn(streams, m, d, generator=gen, device=dev)
    cent = cn * cent / cent.norm(dim=-1, keepdim=True)
    member = torch.randint(0, m, (streams, n), generator=gen, device=dev)
    off = torch.randn(streams, n, d, generator=gen, device=dev)
    off = off / off.norm(dim=-1, keepdim=True)
    off = off * (0.45 * delta * torch.rand(streams, n, 1, generator=gen, device=dev))
    K = torch.gather(cent, 1, member.unsqueeze(-1).expand(streams, n, d)) + off
    V = torch.randn(streams, n, d, generator=gen, device=dev)
    V = V * torch.exp(0.5 * torch.randn(streams, n, 1, generator=gen, device=dev))
    Q = torch.randn(streams, g, d, generator=gen, device=dev)
    Q = Q / Q.norm(dim=-1, keepdim=True) * (r * (1.0 - 2.0 ** -7))
    return K.to(dtype).contiguous(), V.to(dtype).contiguous(), Q.to(dtype).contiguous(), member
