"""Shared helpers of the GPU parity tests: run the oracle on the same bytes and compare state."""
import numpy as np
import torch

from oracle.subgen_oracle import OracleStream

REL_L2_TOL = 2e-3      # attention outputs, fp32 accumulation (benchmark definition)
MARGIN_TOL = 1e-5      # decisions may differ from the oracle only below this relative margin


def to_f32_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


def rel_l2(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Relative L2 error of a against b over the last axis."""
    num = np.linalg.norm(a.astype(np.float64) - b, axis=-1)
    den = np.linalg.norm(b, axis=-1)
    return num / np.maximum(den, 1e-300)


def make_oracles(streams, d, delta, s, w, seed=0, max_centers=0, stream_ids=None, t=0):
    ids = list(stream_ids) if stream_ids is not None else list(range(streams))
    return [OracleStream(d, delta, s, w, seed=seed, stream=i, max_centers=max_centers, t=t) for i in ids]


def compare_state(sg, oracles, stream_ids=None, check_rows=True):
    """Bit-exact comparison of the library's state with the oracle's for the given streams.

    Returns the number of streams whose first differing decision sits below the near-tie
    margin (reported, not failed); anything else that differs raises AssertionError.
    """
    ids = list(stream_ids) if stream_ids is not None else list(range(len(oracles)))
    near_ties = 0
    for o, sid in zip(oracles, ids):
        st = sg.export_state(sid, rows=check_rows)
        assert st.n_seen == o.n_seen and st.n_evicted == o.n_evicted, (sid, st.n_seen, o.n_seen)
        same_assign = True
        if st.assign is not None:
            oa = o.assign[: len(st.assign)]
            if not np.array_equal(st.assign, oa):
                same_assign = False
                first = int(np.flatnonzero(st.assign != oa)[0])
                thr, gap = o.margins()
                margin = min(thr[first], gap[first])
                assert margin < MARGIN_TOL, (
                    f"stream {sid}: assignment of evicted token {first} differs (gpu {st.assign[first]}, oracle "
                    f"{oa[first]}) with decision margin {margin:.3e} >= {MARGIN_TOL}")
                near_ties += 1
                continue          # later state of this stream legitimately differs
        assert st.m == o.m, (sid, st.m, o.m)
        assert np.array_equal(st.counts.astype(np.int64), o.counts), f"stream {sid}: counts differ"
        assert st.counts.sum() + st.window_fill == st.n_seen - o.dropped
        assert bool(st.flags & 2) == (o.dropped > 0), (sid, st.flags, o.dropped)
        assert np.array_equal(st.sample_idx.astype(np.int64), o.sample_idx), f"stream {sid}: sampled indices differ"
        assert np.array_equal(st.sample_vn, o.sample_vn), f"stream {sid}: sample norms differ"
        assert st.mu == o.mu, (sid, st.mu, o.mu)
        assert st.window_fill == o.window_fill
        if check_rows:
            assert np.array_equal(st.centers, o.centers), f"stream {sid}: center rows differ"
            if o.n_evicted > 0:
                assert np.array_equal(st.sample_k, o.sample_k) and np.array_equal(st.sample_v, o.sample_v)
            assert np.array_equal(st.window_k, o.window_k) and np.array_equal(st.window_v, o.window_v)
        assert same_assign
    return near_ties
