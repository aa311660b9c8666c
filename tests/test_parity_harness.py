"""The near-tie protocol of tests/parity_util.py, exercised on the CPU: the part of the "library" is played by a
second oracle whose decision at a planted token is forced the other way, so the harness's detection, override,
replay and strict comparison can be checked without a GPU."""
import types

import numpy as np
import pytest
import torch

from oracle.subgen_oracle import OracleStream
from tests.parity_util import OracleSet, compare_state


class FakeLibrary:
    """export_state() of streams that are themselves oracles (possibly with forced decisions)."""

    def __init__(self, oracles):
        self.oracles = oracles

    def export_state(self, sid, rows=True):
        o = self.oracles[sid]
        st = types.SimpleNamespace()
        st.m, st.n_seen, st.n_evicted, st.mu, st.window_fill = o.m, o.n_seen, o.n_evicted, o.mu, o.window_fill
        st.flags = 2 if o.dropped else 0
        st.counts, st.sample_idx, st.sample_vn = o.counts.astype(np.int32), o.sample_idx.astype(np.int32), o.sample_vn
        st.assign = o.assign
        st.centers, st.sample_k, st.sample_v = o.centers, o.sample_k, o.sample_v
        st.window_k, st.window_v = o.window_k, o.window_v
        return st


def planted_stream(eps, n=60, d=4, seed=0):
    """Keys around three far-apart points; token 20 sits at delta(1 + eps) from the first representative."""
    r = np.random.default_rng(seed)
    delta = 1.0
    base = np.array([[0, 0, 0, 0], [10, 0, 0, 0], [0, 10, 0, 0]], dtype=np.float64)
    K = base[r.integers(0, 3, size=n)] + 0.05 * r.normal(size=(n, d))
    K[0] = base[0]
    K[20] = base[0] + np.array([delta * (1.0 + eps), 0, 0, 0])
    V = r.normal(size=(n, d))
    Q = r.normal(size=(n, 1, d)) / 2
    f = lambda a: torch.tensor(a, dtype=torch.float32)
    return f(K), f(V), f(Q), delta


@pytest.mark.parametrize("w", [0, 3])
def test_near_tie_is_forced_replayed_and_everything_after_it_still_compared(w):
    K, V, Q, delta = planted_stream(eps=2e-6)
    n0 = 40
    plain = OracleStream(4, delta, 3, w, seed=1, stream=0)
    plain.ingest(K.numpy(), V.numpy())
    assert plain.assign[20] == 3 and plain.created[20]            # just outside delta: the oracle opens a cluster
    lib = OracleStream(4, delta, 3, w, seed=1, stream=0)
    lib.set_overrides({20: 0})                                    # the "library" rounds the other way and joins
    lib.ingest(K[:n0].numpy(), V[:n0].numpy())
    lib_out = lib.decode(K[n0:].numpy(), V[n0:].numpy(), Q[n0:].numpy())
    assert lib.m == plain.m - 1

    oset = OracleSet([0], 4, delta, 3, w, seed=1, threads=2)
    oset.ingest(K[None, :n0], V[None, :n0])
    before = oset.decode(K[None, n0:], V[None, n0:], Q[None, n0:])
    fake = FakeLibrary([lib])
    assert compare_state(fake, oset.oracles) == 1                 # without a history the tie can only be counted
    assert oset.reconcile(fake) == 1                              # with one it is forced and replayed
    assert oset.near_ties == {"threshold": 1, "argmin": 0} and oset.overrides[0] == {20: 0}
    assert compare_state(fake, oset.oracles) == 0
    after = oset.reference()
    assert np.array_equal(after[:, 0], lib_out)                   # outputs now follow the library's clustering
    assert not np.array_equal(after, before)                      # ... which changes the normaliser
    assert oset.reconcile(fake) == 1                              # idempotent


def test_a_difference_outside_the_margin_fails():
    K, V, Q, delta = planted_stream(eps=1e-3)
    lib = OracleStream(4, delta, 3, 0, seed=1, stream=0)
    lib.set_overrides({20: 0})
    lib.ingest(K.numpy(), V.numpy())
    oset = OracleSet([0], 4, delta, 3, 0, seed=1, threads=2)
    oset.ingest(K[None], V[None])
    with pytest.raises(AssertionError, match="decision margin"):
        oset.reconcile(FakeLibrary([lib]))
    with pytest.raises(AssertionError, match="decision margin"):
        compare_state(FakeLibrary([lib]), oset.oracles)


def test_a_wrong_sample_after_a_forced_tie_is_still_caught():
    """Before the protocol a stream with a near-tie was dropped from every later check; now a planted error in
    the sampler of such a stream fails."""
    K, V, Q, delta = planted_stream(eps=2e-6)
    lib = OracleStream(4, delta, 3, 0, seed=2, stream=0)          # another seed: other coins than the oracle set's
    lib.set_overrides({20: 0})
    lib.ingest(K.numpy(), V.numpy())
    oset = OracleSet([0], 4, delta, 3, 0, seed=1, threads=2)
    oset.ingest(K[None], V[None])
    with pytest.raises(AssertionError):
        oset.reconcile(FakeLibrary([lib]))


def test_argmin_near_tie_forces_the_runner_up():
    d, delta = 2, 2.0
    K = torch.tensor([[0.0, 0.0], [2.000004 * 1.0 + 0.0, 0.0], [1.0, 0.0], [0.5, 0.0]])   # token 2: 1 and 1.000004
    K[1, 0] = 2.000004
    V = torch.ones(4, d)
    plain = OracleStream(d, delta, 2, 0)
    plain.ingest(K.numpy(), V.numpy())
    assert plain.assign.tolist() == [0, 1, 0, 0]
    lib = OracleStream(d, delta, 2, 0)
    lib.set_overrides({2: 1})
    lib.ingest(K.numpy(), V.numpy())
    oset = OracleSet([0], d, delta, 2, 0, threads=1)
    oset.ingest(K[None], V[None])
    assert oset.reconcile(FakeLibrary([lib])) == 1 and oset.near_ties == {"threshold": 0, "argmin": 1}
    assert oset.oracles[0].counts.tolist() == [2, 2]
