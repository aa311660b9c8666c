"""Shared helpers of the GPU parity tests: run the oracle on the same bytes and compare state.

Near-tie protocol.  Both sides decide in double precision, so they can differ only where a distance sits within
rounding of the threshold or of the runner-up's distance.  When the library's assignment of a token differs from
the oracle's, the oracle's logged margin of that token (``OracleStream.margins``: relative distance to the
threshold, relative gap to the runner-up) must be below ``MARGIN_TOL``; the harness then forces the library's
decision for that token in a fresh oracle, replays the stream's whole input history and goes on comparing
everything, so nothing after a near-tie is left unchecked.  The number of forced decisions is reported.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from oracle.subgen_oracle import OracleStream

REL_L2_TOL = 2e-3      # attention outputs, fp32 accumulation (benchmark definition)
MARGIN_TOL = 1e-5      # decisions may differ from the oracle only below this relative margin
MAX_OVERRIDES_PER_STREAM = 8


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


def first_divergence(st, o):
    """None if the library's assignment log equals the oracle's, else (token, library's entry, oracle's entry,
    margin, kind) for the first token that differs; kind is "threshold" or "argmin"."""
    if st.assign is None:
        return None
    oa = o.assign[: len(st.assign)]
    if np.array_equal(st.assign, oa):
        return None
    first = int(np.flatnonzero(st.assign != oa)[0])
    thr, gap = o.margins()
    kind = "threshold" if thr[first] <= gap[first] else "argmin"
    return first, int(st.assign[first]), int(oa[first]), float(min(thr[first], gap[first])), kind


def assert_state_equal(st, o, sid, check_rows=True):
    """Everything the two sides hold for one stream, bit for bit."""
    assert st.n_seen == o.n_seen and st.n_evicted == o.n_evicted, (sid, st.n_seen, o.n_seen)
    if st.assign is not None:
        assert np.array_equal(st.assign, o.assign[: len(st.assign)]), f"stream {sid}: assignments differ"
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


def compare_state(sg, oracles, stream_ids=None, check_rows=True):
    """Bit-exact comparison of the library's state with the oracle's for the given streams.

    For callers that hold no input history to replay: a differing assignment inside the near-tie margin is
    counted and returned (the callers assert that the count is 0); the decisions before it, which both sides
    share by construction, and the part of the state that does not depend on the clustering (sampler, window)
    are still compared.  Anything else that differs raises AssertionError.
    """
    ids = list(stream_ids) if stream_ids is not None else list(range(len(oracles)))
    near_ties = 0
    for o, sid in zip(oracles, ids):
        st = sg.export_state(sid, rows=check_rows)
        div = first_divergence(st, o)
        if div is None:
            assert_state_equal(st, o, sid, check_rows)
            continue
        first, ga, oa, margin, kind = div
        assert margin < MARGIN_TOL, (
            f"stream {sid}: assignment of evicted token {first} differs (gpu {ga}, oracle {oa}) with decision "
            f"margin {margin:.3e} >= {MARGIN_TOL}")
        near_ties += 1
        # the sampler and the window do not depend on the clustering decision
        assert st.n_seen == o.n_seen and st.mu == o.mu
        assert np.array_equal(st.sample_idx.astype(np.int64), o.sample_idx)
        assert np.array_equal(st.sample_vn, o.sample_vn)
    return near_ties


class OracleSet:
    """Oracles of a subset of streams that remember their inputs, so that a stream can be replayed with a forced
    decision (near-tie protocol, see the module docstring).  Inputs are kept in the stream dtype on the host."""

    def __init__(self, ids, d, delta, s, w, seed=0, max_centers=0, t=0, threads=None):
        self.ids = [int(i) for i in ids]
        self.kw = dict(d=d, delta=delta, s=s, w=w, seed=seed, max_centers=max_centers, t=t)
        self.oracles = [self._fresh(i, {}) for i in self.ids]
        self.history = [[] for _ in self.ids]       # ("ingest", K, V) | ("decode", K, V, Q), torch CPU tensors
        self.refs = [[] for _ in self.ids]          # oracle outputs of the decode entries, [n, g, d] each
        self.overrides = [dict() for _ in self.ids]
        self.near_ties = {"threshold": 0, "argmin": 0}
        self.threads = threads or min(16, len(os.sched_getaffinity(0)))

    def _fresh(self, sid, overrides):
        o = OracleStream(self.kw["d"], self.kw["delta"], self.kw["s"], self.kw["w"], seed=self.kw["seed"], stream=sid,
                         max_centers=self.kw["max_centers"], t=self.kw["t"])
        if overrides:
            o.set_overrides(overrides)
        return o

    @staticmethod
    def _run(o, entry):
        if entry[0] == "ingest":
            o.ingest(entry[1].float().numpy(), entry[2].float().numpy())
            return None
        return o.decode(entry[1].float().numpy(), entry[2].float().numpy(), entry[3].float().numpy())

    def _map(self, fn, n):
        with ThreadPoolExecutor(self.threads) as ex:        # the C oracle releases the GIL
            return list(ex.map(fn, range(n)))

    def ingest(self, K, V):
        """K, V: [len(ids), n, d] tensors (any device) holding the subset's rows of a prefix chunk."""
        K, V = K.detach().cpu(), V.detach().cpu()
        assert K.shape[0] == len(self.ids)
        entries = [("ingest", K[i], V[i]) for i in range(len(self.ids))]
        for h, e in zip(self.history, entries):
            h.append(e)
        self._map(lambda i: self._run(self.oracles[i], entries[i]), len(self.ids))

    def decode(self, K, V, Q):
        """K, V: [len(ids), n, d], Q: [len(ids), n, g, d]; returns the oracle's outputs [n, len(ids), g, d]."""
        K, V, Q = K.detach().cpu(), V.detach().cpu(), Q.detach().cpu()
        entries = [("decode", K[i], V[i], Q[i]) for i in range(len(self.ids))]
        for h, e in zip(self.history, entries):
            h.append(e)
        outs = self._map(lambda i: self._run(self.oracles[i], entries[i]), len(self.ids))
        for r, o in zip(self.refs, outs):
            r.append(o)
        return np.stack(outs, axis=1)

    def reference(self):
        """Oracle outputs of all decode entries so far, [total steps, len(ids), g, d] (after any replay)."""
        return np.stack([np.concatenate(r, axis=0) for r in self.refs], axis=1)

    def _replay(self, i):
        o = self._fresh(self.ids[i], self.overrides[i])
        refs = []
        for e in self.history[i]:
            out = self._run(o, e)
            if out is not None:
                refs.append(out)
        self.oracles[i], self.refs[i] = o, refs

    def reconcile(self, sg, check_rows=True):
        """Compare every stream of the subset with the library; where the first differing assignment is a
        near-tie, force the library's decision in the oracle, replay the stream and compare again.  Returns the
        total number of forced decisions so far; anything that differs outside a near-tie raises."""
        pending = list(range(len(self.ids)))
        for _ in range(MAX_OVERRIDES_PER_STREAM + 1):
            again = []
            for i in pending:
                sid, o = self.ids[i], self.oracles[i]
                st = sg.export_state(sid, rows=check_rows)
                div = first_divergence(st, o)
                if div is None:
                    assert_state_equal(st, o, sid, check_rows)
                    continue
                first, ga, oa, margin, kind = div
                assert margin < MARGIN_TOL, (
                    f"stream {sid}: assignment of evicted token {first} differs (gpu {ga}, oracle {oa}) with "
                    f"decision margin {margin:.3e} >= {MARGIN_TOL}")
                assert len(self.overrides[i]) < MAX_OVERRIDES_PER_STREAM, f"stream {sid}: too many near-ties"
                opened_before = int(o.created[:first].sum())       # clusters that existed when the token arrived
                assert 0 <= ga <= opened_before, (sid, first, ga, opened_before)
                self.overrides[i][first] = OracleStream.FORCE_NEW if ga == opened_before else ga
                self.near_ties[kind] += 1
                again.append(i)
            if not again:
                break
            self._map(lambda j: self._replay(again[j]), len(again))
            pending = again
        assert not again
        return sum(len(ov) for ov in self.overrides)
