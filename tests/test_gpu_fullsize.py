"""Full-size parity: the n=16k workload in the launch configuration bench.py times (8192 streams,
prefix ingested in 1024-token chunks, fused subgen_step), checked against the oracle on sampled
streams, plus size-independent invariants on a larger sample."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from paper_2402_06082_amd.workloads import BLOCK, CONFIGS, Workload
from tests.parity_util import REL_L2_TOL, compare_state, make_oracles, rel_l2, to_f32_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sampled_streams(cfg, extra=3, seed=0):
    """First / last index on every (batch, layer, head) axis plus random picks."""
    B, L, H = cfg.batch, cfg.layers, cfg.kv_heads
    lin = lambda b, l, h: (b * L + l) * H + h
    ids = {lin(0, 0, 0), lin(B - 1, L - 1, H - 1), lin(0, 0, H - 1), lin(0, L - 1, 0), lin(B - 1, 0, 0)}
    r = np.random.default_rng(seed)
    while len(ids) < 5 + extra:
        ids.add(int(r.integers(0, cfg.streams)))
    return sorted(ids)


def test_cfg3_full_size_sampled_streams():
    from paper_2402_06082_amd import binding
    from paper_2402_06082_amd.tuning import tune_delta
    cfg = CONFIGS["cfg3"]
    steps = 24
    delta, _ = tune_delta(cfg, DEV)
    wl = Workload(cfg, device=DEV)
    S = wl.S
    ids = sampled_streams(cfg)
    sg = binding.SubGen(S, cfg.d, delta, cfg.s, cfg.w, dtype=cfg.torch_dtype, max_centers=2048,
                        assign_log_tokens=cfg.prefix + steps, seed=0, device=DEV)
    hostK, hostV = [], []
    for t0 in range(0, cfg.prefix, 4 * BLOCK):
        K, V = wl.tokens(t0, t0 + 4 * BLOCK)
        sg.ingest_prefix(K, V)
        hostK.append(to_f32_np(K[ids]))
        hostV.append(to_f32_np(V[ids]))
        del K, V
    hostK, hostV = np.concatenate(hostK, 1), np.concatenate(hostV, 1)
    oracles = make_oracles(S, cfg.d, delta, cfg.s, cfg.w, seed=0, stream_ids=ids)
    with ThreadPoolExecutor(8) as ex:
        list(ex.map(lambda a: a[0].ingest(a[1], a[2]), zip(oracles, hostK, hostV)))
    assert compare_state(sg, oracles, ids) == 0          # state after the prefix

    K, V = wl.tokens(cfg.prefix, cfg.prefix + steps)
    Q = wl.queries(0, steps)
    outs = torch.empty(steps, S, 1, cfg.d, dtype=torch.float32, device=DEV)
    for t in range(steps):
        sg.step(K[:, t].contiguous(), V[:, t].contiguous(), Q[:, t].contiguous(), outs[t])
    sg.sync()
    Kc, Vc, Qc = to_f32_np(K[ids]), to_f32_np(V[ids]), to_f32_np(Q[ids])
    ref = np.stack([o.decode(k, v, q) for o, k, v, q in zip(oracles, Kc, Vc, Qc)], axis=1)
    got = outs.cpu().numpy()[:, ids]
    err = rel_l2(got, ref)
    assert np.isfinite(outs.cpu().numpy()).all()
    assert err.max() <= REL_L2_TOL, err.max()
    assert compare_state(sg, oracles, ids) == 0          # state after the decode steps

    # invariants that hold at any size, on 256 more streams: counts add up, every slot is filled,
    # sampled tokens are evicted ones, no overflow flag
    st = sg.stats()
    assert st.flags_or == 0 and st.n_seen == cfg.prefix + steps
    r = np.random.default_rng(1)
    for sid in r.choice(S, size=256, replace=False):
        e = sg.export_state(int(sid), rows=False)
        assert e.counts.sum() + e.window_fill == e.n_seen and e.counts.min() >= 1
        assert e.sample_idx.min() >= 0 and e.sample_idx.max() < e.n_evicted
        assert len(e.assign) == e.n_evicted and e.assign.max() == e.m - 1
        assert np.array_equal(np.bincount(e.assign, minlength=e.m), e.counts)
    print(f"cfg3 full size: delta={delta:.4f} mean m={st.total_centers / S:.1f} sampled streams {ids} "
          f"max rel-L2={err.max():.2e}")


def test_cfg5_all_streams_sampled_against_the_oracle():
    """The GQA workload with all of its 8192 KV streams x 4 queries in one launch (the tile kernels in the launch
    configuration bench.py times); the prefix is cut to 8192 tokens so that the oracle finishes in seconds."""
    from paper_2402_06082_amd import binding
    cfg = CONFIGS["cfg5"]
    prefix, steps, delta = 8192, 12, 8.5234375
    wl = Workload(cfg, device=DEV)
    S = wl.S
    ids = sampled_streams(cfg)
    sg = binding.SubGen(S, cfg.d, delta, cfg.s, cfg.w, dtype=cfg.torch_dtype, q_per_stream=cfg.g, max_centers=2048,
                        assign_log_tokens=prefix + steps, seed=0, device=DEV)
    hostK, hostV = [], []
    for t0 in range(0, prefix, 4 * BLOCK):
        K, V = wl.tokens(t0, t0 + 4 * BLOCK)
        sg.ingest_prefix(K, V)
        hostK.append(to_f32_np(K[ids]))
        hostV.append(to_f32_np(V[ids]))
        del K, V
    hostK, hostV = np.concatenate(hostK, 1), np.concatenate(hostV, 1)
    oracles = make_oracles(S, cfg.d, delta, cfg.s, cfg.w, seed=0, stream_ids=ids)
    with ThreadPoolExecutor(8) as ex:
        list(ex.map(lambda a: a[0].ingest(a[1], a[2]), zip(oracles, hostK, hostV)))
    assert compare_state(sg, oracles, ids) == 0
    K, V = wl.tokens(prefix, prefix + steps)
    Q = wl.queries(0, steps)
    outs = torch.empty(steps, S, cfg.g, cfg.d, dtype=torch.float32, device=DEV)
    for t in range(steps):
        sg.step(K[:, t].contiguous(), V[:, t].contiguous(), Q[:, t].contiguous(), outs[t])
    many = sg.attend_many(Q[:, steps - 1].contiguous())          # the same queries once more, as a block
    sg.sync()
    Kc, Vc, Qc = to_f32_np(K[ids]), to_f32_np(V[ids]), to_f32_np(Q[ids])
    ref = np.stack([o.decode(k, v, q) for o, k, v, q in zip(oracles, Kc, Vc, Qc)], axis=1)
    got = outs.cpu().numpy()
    assert np.isfinite(got).all()
    err = rel_l2(got[:, ids], ref)
    assert err.max() <= REL_L2_TOL, err.max()
    assert rel_l2(many.cpu().numpy()[ids], ref[steps - 1]).max() <= REL_L2_TOL
    assert compare_state(sg, oracles, ids) == 0
    st = sg.stats()
    assert st.flags_or == 0 and st.n_seen == prefix + steps
    print(f"cfg5 all streams: mean m={st.total_centers / S:.1f} max rel-L2={err.max():.2e}")
