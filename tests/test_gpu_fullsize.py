"""Full-size parity: the n=16k, long-context and grouped-query workloads at their stated sizes, in the launch
configuration bench.py times (all streams in one launch, prefix ingested in 1024-token chunks, fused subgen_step),
checked against the oracle on 64 sampled streams (first / last index on every batch, layer and head axis plus
random picks) with the near-tie protocol of tests/parity_util.py, plus size-independent invariants on a larger
sample of streams."""
import os
import time

import numpy as np
import pytest
import torch

from paper_2402_06082_amd.workloads import BLOCK, CONFIGS, Workload
from tests.parity_util import REL_L2_TOL, OracleSet, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def progress(msg):
    """Long tests leave a trace of their steps (the oracle's share of a long-context stream takes a while)."""
    try:
        os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(ROOT, "gpurun_out", "fullsize_progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


def sampled_streams(cfg, total=64, seed=0):
    """First / last index on every (batch, layer, head) axis, all their combinations, plus random picks."""
    B, L, H = cfg.batch, cfg.layers, cfg.kv_heads
    lin = lambda b, l, h: (b * L + l) * H + h
    ids = {lin(b, l, h) for b in (0, B - 1) for l in (0, L - 1) for h in (0, H - 1)}
    r = np.random.default_rng(seed)
    while len(ids) < total:
        ids.add(int(r.integers(0, cfg.streams)))
    return sorted(ids)


def run_full_size(name, delta, steps, oracle_pieces=1):
    """Whole workload on the GPU, 64 streams in the oracle; returns what the caller prints."""
    from paper_2402_06082_amd import binding
    cfg = CONFIGS[name]
    wl = Workload(cfg, device=DEV)
    S = wl.S
    ids = sampled_streams(cfg)
    assert len(ids) >= 64 and ids[0] == 0 and ids[-1] == S - 1
    sg = binding.SubGen(S, cfg.d, delta, cfg.s, cfg.w, dtype=cfg.torch_dtype, q_per_stream=cfg.g, max_centers=4096,
                        assign_log_tokens=cfg.prefix + steps, seed=0, device=DEV)
    idx = torch.tensor(ids, device=DEV)
    hostK, hostV = [], []
    progress(f"{name}: ingesting {cfg.prefix} tokens x {S} streams")
    for t0 in range(0, cfg.prefix, 4 * BLOCK):
        K, V = wl.tokens(t0, t0 + 4 * BLOCK)
        sg.ingest_prefix(K, V)
        hostK.append(K[idx].cpu())
        hostV.append(V[idx].cpu())
        del K, V
    sg.sync()
    hostK, hostV = torch.cat(hostK, 1), torch.cat(hostV, 1)
    oset = OracleSet(ids, cfg.d, delta, cfg.s, cfg.w, seed=0, max_centers=4096)
    piece = (cfg.prefix + oracle_pieces - 1) // oracle_pieces
    for p0 in range(0, cfg.prefix, piece):
        oset.ingest(hostK[:, p0:p0 + piece], hostV[:, p0:p0 + piece])
        progress(f"{name}: oracle at token {min(p0 + piece, cfg.prefix)} of {cfg.prefix} ({len(ids)} streams, "
                 f"{oset.threads} threads)")
    del hostK, hostV
    forced_prefix = oset.reconcile(sg)                    # state after the prefix, bit for bit
    progress(f"{name}: state after the prefix equal, {forced_prefix} near-ties")

    K, V = wl.tokens(cfg.prefix, cfg.prefix + steps)
    Q = wl.queries(0, steps)
    outs = torch.empty(steps, S, cfg.g, cfg.d, dtype=torch.float32, device=DEV)
    for t in range(steps):
        sg.step(K[:, t].contiguous(), V[:, t].contiguous(), Q[:, t].contiguous(), outs[t])
    many = sg.attend_many(Q[:, steps - 1].contiguous()) if cfg.g > 1 else None    # the same queries as a block
    sg.sync()
    oset.decode(K[idx], V[idx], Q[idx])
    forced = oset.reconcile(sg)                           # state after the decode steps (replays if it must)
    ref = oset.reference()
    got = outs.cpu().numpy()
    assert np.isfinite(got).all()
    err = rel_l2(got[:, ids], ref)                        # per (step, stream, query)
    assert err.max() <= REL_L2_TOL, err.max()
    if many is not None:
        assert rel_l2(many.cpu().numpy()[ids], ref[steps - 1]).max() <= REL_L2_TOL

    # invariants that hold at any size, on 256 more streams: counts add up, every slot is filled, sampled tokens
    # are evicted ones, the decision log is consistent with the counts, no sticky flag
    st = sg.stats()
    assert st.flags_or == 0 and st.n_seen == cfg.prefix + steps
    r = np.random.default_rng(1)
    for sid in r.choice(S, size=256, replace=False):
        e = sg.export_state(int(sid), rows=False)
        assert e.counts.sum() + e.window_fill == e.n_seen and e.counts.min() >= 1
        assert e.sample_idx.min() >= 0 and e.sample_idx.max() < e.n_evicted
        assert len(e.assign) == e.n_evicted and e.assign.max() == e.m - 1
        assert np.array_equal(np.bincount(e.assign, minlength=e.m), e.counts)
    msg = (f"{name} full size: {S} streams x {cfg.g} queries, prefix {cfg.prefix}, {steps} fused steps, delta="
           f"{delta:.4f}, mean m={st.total_centers / S:.1f} (max {st.max_centers}), {len(ids)} oracle streams, "
           f"near-ties forced={forced} {oset.near_ties}, max rel-L2={err.max():.2e}")
    progress(msg)
    print(msg)
    return forced, st


def test_cfg3_full_size_sampled_streams():
    from paper_2402_06082_amd.tuning import tune_delta
    delta, _ = tune_delta(CONFIGS["cfg3"], DEV)
    forced, st = run_full_size("cfg3", delta, steps=24)
    assert forced <= 2 and 500 <= st.total_centers / st.streams <= 700


def test_cfg5_full_size_gqa_sampled_streams():
    """All 8192 KV streams x 4 queries with the whole 32768-token prefix (the LDS-tiled matrix-core kernels)."""
    forced, st = run_full_size("cfg5", 8.5234375, steps=16)
    assert forced <= 2 and 500 <= st.total_centers / st.streams <= 700


def test_cfg4_full_size_long_context_sampled_streams():
    """4096 streams, the whole 131072-token drifting prefix (token indices beyond 2^16, 128 coin passes per stream,
    center tables of about 2400 rows, 1024 sample slots, a 256-token window) on the four-wavefront kernels."""
    forced, st = run_full_size("cfg4", 8.5234375, steps=16, oracle_pieces=8)
    assert forced <= 4 and 2000 <= st.total_centers / st.streams <= 2900
