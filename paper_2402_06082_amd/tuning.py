"""Threshold selection for the synthetic workloads: bisection on delta until the mean number of
centers per stream at the end of the prefix reaches the config's target.  Runs the library
itself (prefix ingest on a few probe streams); no arithmetic of the method lives here."""
from __future__ import annotations

from typing import Tuple

from . import binding
from .workloads import Config, Workload


def mean_centers(cfg: Config, delta: float, K, V, max_centers: int) -> float:
    sg = binding.SubGen(K.shape[0], cfg.d, delta, 4, cfg.w, dtype=cfg.torch_dtype, max_centers=max_centers,
                        device=K.device)
    try:
        sg.ingest_prefix(K, V)
        return float(sg.center_counts().mean())
    finally:
        sg.close()


def tune_delta(cfg: Config, device="cuda:0", probe_streams: int = 16, prefix: int | None = None,
               lo: float = 0.0, hi: float = 0.0, iters: int = 14, rel_tol: float = 0.02) -> Tuple[float, float]:
    """Returns (delta, mean centers at that delta).  Fixed-delta configs are returned unchanged."""
    if cfg.delta is not None:
        return float(cfg.delta), float("nan")
    assert cfg.target_centers
    n = cfg.prefix if prefix is None else prefix
    wl = Workload(cfg, device=device, streams=probe_streams)
    K, V = wl.tokens(0, n)
    cap = max(4 * cfg.target_centers, 1024)
    # bracket: the typical distance between two keys of one component is sigma*sqrt(2d)
    typical = cfg.sigma * (2.0 * cfg.d) ** 0.5
    lo = lo or 0.5 * typical
    hi = hi or 2.0 * typical
    best = (hi, mean_centers(cfg, hi, K, V, cap))
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        m = mean_centers(cfg, mid, K, V, cap)
        best = (mid, m)
        if abs(m - cfg.target_centers) <= rel_tol * cfg.target_centers:
            break
        if m > cfg.target_centers:      # too many centers: raise the threshold
            lo = mid
        else:
            hi = mid
    return float(best[0]), float(best[1])
