"""Empirical check of the paper's error guarantee (Section 1.3, Eq. (3); Theorem 1) on the HIP path.

For a stream that was compressed by the library, the output z of ``attend`` is compared with exact softmax
attention over the full cache:

    eps_hat = ||z - Attn(q, K, V)||_2 / ( ||softmax(K q)||_2 * ||V||_op )

Theorem 1 states eps_hat <= eps with probability >= 0.99 when s = Omega(d / eps^2),
t = Omega(eps^-2 e^{2 delta r} log n) and ||q|| <= r.  ``choose_parameters`` evaluates these two expressions
with explicit constants; ``measure`` runs the library (window 0, i.e. Algorithm 1 exactly as printed) and
returns the distribution of eps_hat over streams and queries.

Everything the method computes runs in the library (compression, estimator, and the exact attention it is
compared with); torch is used here only to evaluate the right-hand side of the bound (a softmax norm and a
spectral norm), which is not part of the method.

Command line:  python -m paper_2402_06082_amd.error_bound --eps 0.5 0.25 --delta-r 0.1 0.5
"""
from __future__ import annotations

import argparse
import json
import math
from typing import Dict, Optional, Tuple

import numpy as np
import torch

from . import binding
from .workloads import clusterable_streams

T_MAX = 64   # reservoir slots per cluster the library accepts


def choose_parameters(eps: float, d: int, n: int, delta: float, r: float, c_s: float = 1.0,
                      c_t: float = 1.0) -> Tuple[int, int]:
    """(s, t) of Theorem 1 with the constants of the Omega(.) made explicit:
    s = ceil(c_s d / eps^2),  t = ceil(c_t e^{2 delta r} ln(n) / eps^2)."""
    if not (eps > 0.0 and d > 0 and n > 0 and delta >= 0.0 and r >= 0.0 and c_s > 0.0 and c_t > 0.0):
        raise ValueError("eps, d, n, c_s, c_t must be positive; delta and r non-negative")
    s = math.ceil(c_s * d / eps ** 2)
    t = math.ceil(c_t * math.exp(2.0 * delta * r) * math.log(max(n, 2)) / eps ** 2)
    return int(s), int(t)


def bound_rhs(K: torch.Tensor, V: torch.Tensor, Q: torch.Tensor) -> torch.Tensor:
    """||softmax(K q)||_2 * ||V||_op for every (stream, query): [S, g] float64 (evaluation only)."""
    Kd, Qd = K.double(), Q.double()
    sc = torch.einsum("snd,sgd->sgn", Kd, Qd)
    sc = sc - sc.max(dim=-1, keepdim=True).values
    e = sc.exp()
    sm2 = e.pow(2).sum(-1).sqrt() / e.sum(-1)                       # ||softmax||_2
    Vd = V.double()
    gram = torch.einsum("snd,sne->sde", Vd, Vd).cpu().numpy()       # V^T V, [S, d, d]
    vop = np.sqrt(np.linalg.eigvalsh(gram)[:, -1].clip(min=0.0))    # spectral norm of V
    return sm2 * torch.from_numpy(vop).to(sm2.device).unsqueeze(-1)


def eps_hat(z: torch.Tensor, K: torch.Tensor, V: torch.Tensor, Q: torch.Tensor) -> torch.Tensor:
    """Left-hand side over right-hand side of Eq. (3) for every (stream, query): [S, g] float64."""
    exact = binding.exact_attend(K, V, Q).double()
    return (z.double() - exact).norm(dim=-1) / bound_rhs(K, V, Q)


def measure(streams: int, n: int, d: int, m: int, delta: float, r: float, s: int, t: int, g: int = 4,
            dtype=torch.float32, seed: int = 0, data_seed: int = 0, device="cuda:0",
            inputs: Optional[tuple] = None) -> Dict:
    """Compress ``streams`` (m, delta)-clusterable streams of n tokens with budgets (s, t) and return the
    distribution of eps_hat over streams x queries, with the number of clusters the library opened."""
    if not (0 <= t <= T_MAX):
        raise ValueError(f"t = {t} is outside the library's range 0..{T_MAX}")
    K, V, Q, _ = inputs if inputs is not None else clusterable_streams(streams, n, d, m, delta, r, g=g,
                                                                       seed=data_seed, device=device, dtype=dtype)
    sg = binding.SubGen(streams, d, delta, s, 0, dtype=dtype, q_per_stream=g, max_centers=max(2 * m, 16),
                        seed=seed, device=device, t_per_cluster=t)
    try:
        sg.ingest_prefix(K, V)
        z = sg.attend(Q)
        st = sg.stats()
        centers = sg.center_counts()
    finally:
        sg.close()
    e = eps_hat(z, K, V, Q).flatten().cpu().numpy()
    return {"eps_hat_median": float(np.median(e)), "eps_hat_p90": float(np.quantile(e, 0.90)),
            "eps_hat_p99": float(np.quantile(e, 0.99)), "eps_hat_max": float(e.max()), "pairs": int(e.size),
            "centers_max": int(centers.max()), "flags": int(st.flags_or), "s": int(s), "t": int(t),
            "delta_r": float(delta * r), "eps_hat": e}


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--eps", type=float, nargs="+", default=[0.5, 0.25])
    ap.add_argument("--delta-r", type=float, nargs="+", default=[0.1, 0.5, 1.0])
    ap.add_argument("--streams", type=int, default=256)
    ap.add_argument("--n", type=int, default=4096)
    ap.add_argument("--d", type=int, default=64)
    ap.add_argument("--m", type=int, default=32)
    ap.add_argument("--delta", type=float, default=0.5)
    ap.add_argument("--c-s", type=float, default=1.0)
    ap.add_argument("--c-t", type=float, default=1.0)
    ap.add_argument("--bf16", action="store_true")
    a = ap.parse_args(argv)
    dtype = torch.bfloat16 if a.bf16 else torch.float32
    for dr in a.delta_r:
        r = dr / a.delta
        inputs = clusterable_streams(a.streams, a.n, a.d, a.m, a.delta, r, g=4, seed=0, device="cuda:0", dtype=dtype)
        for eps in a.eps:
            s, t = choose_parameters(eps, a.d, a.n, a.delta, r, a.c_s, a.c_t)
            row = measure(a.streams, a.n, a.d, a.m, a.delta, r, s, min(t, T_MAX), inputs=inputs, dtype=dtype)
            e = row.pop("eps_hat")
            row.update(eps=eps, t_theorem=t, fraction_within_eps=float((e <= eps).mean()))
            print(json.dumps(row), flush=True)


if __name__ == "__main__":
    main()
