"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU).

Each test states the passage it checks.  None of them re-types the oracle's
own formulas as the expected value: expectations are brute force on exact
integer data, textbook softmax attention, closed forms, published
known-answer vectors, or statistical laws the lemmas assert.
"""
import math
import os

import numpy as np
import pytest

from oracle.subgen_oracle import OracleStream, exact_attention, philox4x32_10, uniform24

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------
# random numbers (the coin flips of Algorithm 1)
# --------------------------------------------------------------------------
def test_philox_known_answer_vectors():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_uniform24_counter_layout_and_range():
    # slot j uses word j%4 of the block with counter (j//4, token lo, token hi, stream), key = seed
    seed, stream, token = 0x0123456789ABCDEF, 77, (5 << 32) + 9
    for slot in [0, 1, 2, 3, 4, 7, 1023]:
        words = philox4x32_10([slot // 4, token & 0xFFFFFFFF, token >> 32, stream],
                              [seed & 0xFFFFFFFF, seed >> 32])
        expect = (words[slot % 4] >> 8) / 2.0 ** 24
        got = uniform24(seed, stream, token, slot)
        assert got == expect and 0.0 <= got < 1.0


def test_uniform24_is_uniform_and_slots_are_independent():
    u = np.array([[uniform24(3, 1, t, j) for j in range(8)] for t in range(20000)])
    # chi-square on 16 bins per slot, 15 dof: 99.99% quantile is ~44
    for j in range(8):
        h, _ = np.histogram(u[:, j], bins=16, range=(0, 1))
        chi = ((h - 1250.0) ** 2 / 1250.0).sum()
        assert chi < 50.0
    # serial pairs (neighbouring slots, neighbouring tokens): correlation ~ N(0, 1/n)
    assert abs(np.corrcoef(u[:, 0], u[:, 1])[0, 1]) < 0.04
    assert abs(np.corrcoef(u[:-1, 2], u[1:, 2])[0, 1]) < 0.04
    # different streams / seeds give different sequences
    assert uniform24(3, 1, 5, 0) != uniform24(3, 2, 5, 0)
    assert uniform24(3, 1, 5, 0) != uniform24(4, 1, 5, 0)


# --------------------------------------------------------------------------
# clustering (UpdateSoftmaxNormalizer, Lemma 2, Definition 1)
# --------------------------------------------------------------------------
def brute_force_clusters(keys, delta):
    """Greedy threshold clustering in exact integer arithmetic (pure Python)."""
    centers, counts, assign = [], [], []
    for k in keys:
        best, arg = None, -1
        for i, x in enumerate(centers):
            dist2 = sum((int(a) - int(b)) ** 2 for a, b in zip(x, k))
            if best is None or dist2 < best:
                best, arg = dist2, i
        if arg >= 0 and best <= delta * delta:
            counts[arg] += 1
            assign.append(arg)
        else:
            centers.append(list(k))
            counts.append(1)
            assign.append(len(centers) - 1)
    return centers, counts, assign


@pytest.mark.parametrize("seed,d,delta", [(0, 1, 2), (1, 2, 3), (2, 3, 4), (3, 4, 5), (4, 4, 0)])
def test_clustering_matches_integer_brute_force(seed, d, delta):
    r = rng(seed)
    keys = r.integers(-8, 9, size=(64, d))
    o = OracleStream(d, delta, s=4, w=0)
    o.ingest(keys, r.normal(size=(64, d)))
    centers, counts, assign = brute_force_clusters(keys, delta)
    assert o.m == len(centers)
    assert o.centers.astype(int).tolist() == centers
    assert o.counts.tolist() == counts
    assert o.assign.tolist() == assign


def test_threshold_is_inclusive_and_ties_go_to_lowest_index():
    # 3-4-5 triangle: distance exactly 5 joins at delta = 5, not at delta just below
    for delta, m_expect in [(5.0, 1), (np.nextafter(np.float32(5.0), np.float32(0.0)), 2)]:
        o = OracleStream(2, delta, s=1, w=0)
        o.ingest([[0, 0], [3, 4]], [[1, 0], [1, 0]])
        assert o.m == m_expect
    # two representatives at equal distance from the third key: the older one wins
    o = OracleStream(1, 2.0, s=1, w=0)
    o.ingest([[0.0], [4.0], [2.0]], np.ones((3, 1)))
    assert o.m == 2 and o.counts.tolist() == [2, 1] and o.assign.tolist() == [0, 1, 0]
    o = OracleStream(1, 2.0, s=1, w=0)
    o.ingest([[4.0], [0.0], [2.0]], np.ones((3, 1)))
    assert o.centers[:, 0].tolist() == [4.0, 0.0] and o.counts.tolist() == [2, 1]


def test_nearest_not_first_within_threshold():
    # both representatives are within delta; the nearer (later) one must win
    o = OracleStream(1, 3.0, s=1, w=0)
    o.ingest([[0.0], [4.0], [2.5]], np.ones((3, 1)))
    assert o.assign.tolist() == [0, 1, 1]


@pytest.mark.parametrize("w", [0, 5])
def test_lemma2_invariants_on_random_stream(w):
    r = rng(10 + w)
    n, d, delta = 600, 8, 2.5
    comp = r.integers(0, 12, size=n)
    cent = r.normal(size=(12, d)) * 3
    K = (cent[comp] + 0.5 * r.normal(size=(n, d))).astype(np.float32)
    o = OracleStream(d, delta, s=8, w=w)
    o.ingest(K, r.normal(size=(n, d)))
    X, cnt, a = o.centers.astype(np.float64), o.counts, o.assign
    ev = K[: n - w].astype(np.float64)        # evicted tokens, in order
    assert o.n_evicted == n - w and len(a) == n - w
    # (2) counts are cluster sizes; they add up to the evicted tokens; window holds the rest
    assert np.array_equal(cnt, np.bincount(a, minlength=o.m))
    assert cnt.min() >= 1 and cnt.sum() + o.window_fill == o.n_seen == n
    # (1) the representative is the first key assigned to its cluster
    for j in range(o.m):
        assert np.array_equal(X[j], ev[np.flatnonzero(a == j)[0]])
    # (3) every key within delta of its representative
    assert (np.linalg.norm(ev - X[a], axis=1) <= delta).all()
    # (4) representatives pairwise more than delta apart
    D = np.linalg.norm(X[:, None] - X[None], axis=-1) + 1e9 * np.eye(o.m)
    assert (D > delta).all()
    # created flag marks exactly the first member of each cluster
    assert o.created.sum() == o.m


def test_separated_groups_give_exactly_m_centers_for_any_order():
    # Definition 1 + pigeonhole argument of Theorem 1: m groups of diameter <= delta whose
    # members are > delta away from every other group's members give exactly m clusters
    r = rng(5)
    m, d, delta = 7, 6, 1.0
    base = r.normal(size=(m, d))
    base *= 10.0 / np.linalg.norm(base, axis=1, keepdims=True) * np.arange(1, m + 1)[:, None]
    sizes = r.integers(3, 30, size=m)
    pts, lab = [], []
    for j in range(m):
        off = r.normal(size=(sizes[j], d))
        off *= (0.49 * delta * r.random((sizes[j], 1))) / np.linalg.norm(off, axis=1, keepdims=True)
        pts.append(base[j] + off)
        lab += [j] * sizes[j]
    pts, lab = np.concatenate(pts).astype(np.float32), np.array(lab)
    for trial in range(5):
        perm = r.permutation(len(pts))
        o = OracleStream(d, delta, s=2, w=0)
        o.ingest(pts[perm], np.ones((len(pts), d)))
        assert o.m == m
        # each cluster is one group: counts equal group sizes
        got = sorted(o.counts.tolist())
        assert got == sorted(sizes.tolist())
        first_lab = [lab[perm][np.flatnonzero(o.assign == j)[0]] for j in range(m)]
        assert sorted(first_lab) == list(range(m))


def test_capacity_overflow_joins_nearest():
    o = OracleStream(1, 0.5, s=1, w=0, max_centers=2)
    o.ingest([[0.0], [10.0], [20.0], [4.0]], np.ones((4, 1)))
    assert o.m == 2 and o.overflowed
    assert o.assign.tolist() == [0, 1, 1, 0] and o.counts.tolist() == [2, 2]


# --------------------------------------------------------------------------
# sampling (UpdateMatrixProduct, Lemma 1)
# --------------------------------------------------------------------------
def test_mu_and_first_token_fill():
    r = rng(1)
    V = r.normal(size=(40, 5)).astype(np.float32)
    o = OracleStream(5, 1.0, s=16, w=3)
    for t in range(40):
        o.update(r.normal(size=5), V[t])
        if t < 3:
            assert (o.sample_idx == -1).all() and o.mu == 0.0
        if t == 3:      # first eviction: all slots hold token 0 (Section 2.2)
            assert (o.sample_idx == 0).all()
            assert np.array_equal(o.sample_v, np.tile(V[0], (16, 1)))
    vn = (V[:37].astype(np.float64) ** 2).sum(1).astype(np.float32).astype(np.float64)
    assert o.mu == pytest.approx(vn.sum(), rel=1e-14)
    # stored per-slot squared norms and rows are those of the token the slot names
    idx = o.sample_idx
    assert np.array_equal(o.sample_vn, vn[idx].astype(np.float32))
    assert np.array_equal(o.sample_v, V[idx])


def test_second_token_probability_uses_mu_before_update():
    # two tokens with ||v1||^2 = 1, ||v2||^2 = 3: each slot must hold token 2 w.p. 3/4
    # (it would be 3/7 if mu were bumped before the coin flips)
    s = 40000
    o = OracleStream(1, 1.0, s=s, w=0, seed=9)
    o.update([0.0], [1.0])
    o.update([5.0], [math.sqrt(3.0)])
    frac = (o.sample_idx == 1).mean()
    assert abs(frac - 0.75) < 5 * math.sqrt(0.75 * 0.25 / s)


def test_lemma1_sampling_frequencies_and_slot_independence():
    r = rng(2)
    n, s, d = 12, 6, 3
    V = (r.normal(size=(n, d)) * r.uniform(0.3, 2.0, size=(n, 1))).astype(np.float32)
    K = r.normal(size=(n, d)).astype(np.float32)
    pr = (V.astype(np.float64) ** 2).sum(1)
    pr /= pr.sum()
    seeds = 6000
    hist = np.zeros((s, n))
    joint = np.zeros((n, n))
    for seed in range(seeds):
        o = OracleStream(d, 1.0, s=s, w=0, seed=seed)
        o.ingest(K, V)
        idx = o.sample_idx
        hist[np.arange(s), idx] += 1
        joint[idx[0], idx[1]] += 1
    # chi-square per slot, n-1 = 11 dof: 99.99% quantile ~ 39
    for j in range(s):
        chi = ((hist[j] - seeds * pr) ** 2 / (seeds * pr)).sum()
        assert chi < 45.0, (j, chi)
    # slots 0 and 1 independent: chi-square on the joint table, 120 dof + slack
    exp = seeds * np.outer(pr, pr)
    mask = exp > 5
    chi = ((joint - exp) ** 2 / exp)[mask].sum()
    assert chi < mask.sum() + 6 * math.sqrt(2 * mask.sum())


def test_zero_norm_values():
    o = OracleStream(2, 1.0, s=8, w=0)
    o.update([1.0, 0.0], [0.0, 0.0])          # first token, zero value: fills slots, mu stays 0
    assert (o.sample_idx == 0).all() and o.mu == 0.0
    q = np.array([0.3, 0.1], dtype=np.float32)
    assert np.array_equal(o.attend(q), np.zeros(2))
    o.update([1.0, 0.0], [2.0, 0.0])          # mu == 0 still: p = 1
    assert (o.sample_idx == 1).all() and o.mu == 4.0
    o.update([1.0, 0.0], [0.0, 0.0])          # zero value later: never sampled
    assert (o.sample_idx == 1).all() and o.mu == 4.0


# --------------------------------------------------------------------------
# query (QueryStreamAttn) — closed forms, exact special cases, statistics
# --------------------------------------------------------------------------
def test_single_token_returns_its_value():
    for w in [0, 1, 4]:
        o = OracleStream(3, 1.0, s=5, w=w)
        o.update([0.5, -1.0, 2.0], [1.5, -2.0, 0.25])
        out = o.attend([0.1, 0.2, 0.3])
        assert np.allclose(out, [1.5, -2.0, 0.25], rtol=1e-15)


def test_window_only_equals_textbook_attention():
    # n <= w: nothing is compressed, the answer is softmax(K q)^T V
    r = rng(3)
    n, d = 37, 16
    K, V = r.normal(size=(n, d)).astype(np.float32), r.normal(size=(n, d)).astype(np.float32)
    o = OracleStream(d, 0.7, s=4, w=64)
    for t in range(n):
        o.update(K[t], V[t])
        q = r.normal(size=d).astype(np.float32)
        assert np.allclose(o.attend(q), exact_attention(K[: t + 1], V[: t + 1], q), rtol=1e-12, atol=1e-14)
    assert o.m == 0 and o.n_evicted == 0


@pytest.mark.parametrize("w", [0, 7])
def test_delta_zero_denominator_is_exact_partition_function(w):
    r = rng(4)
    n, d = 200, 8
    K = r.normal(size=(40, d)).astype(np.float32)[r.integers(0, 40, size=n)]   # many exact duplicates
    V = r.normal(size=(n, d)).astype(np.float32)
    o = OracleStream(d, 0.0, s=8, w=w)
    o.ingest(K, V)
    assert o.m <= 40 and o.counts.sum() == n - w
    q = r.normal(size=d).astype(np.float32)
    _, den, mx = o.attend(q, return_den=True)
    Z = np.exp(K.astype(np.float64) @ q.astype(np.float64)).sum()
    assert den * math.exp(mx) == pytest.approx(Z, rel=1e-12)


def test_denominator_within_exp_delta_r_of_partition_function():
    # Lemma 2 (3) + Cauchy-Schwarz (as in the proof of Theorem 1): every key is within delta of
    # its representative, so tau / Z lies in [e^{-delta |q|}, e^{+delta |q|}]
    r = rng(6)
    n, d, delta = 500, 8, 1.5
    K = (r.normal(size=(10, d))[r.integers(0, 10, size=n)] * 3 + 0.4 * r.normal(size=(n, d))).astype(np.float32)
    o = OracleStream(d, delta, s=4, w=16)
    o.ingest(K, r.normal(size=(n, d)))
    assert o.m < n // 4
    for _ in range(10):
        q = (r.normal(size=d) / math.sqrt(d)).astype(np.float32)
        _, den, mx = o.attend(q, return_den=True)
        ratio = den * math.exp(mx) / np.exp(K.astype(np.float64) @ q.astype(np.float64)).sum()
        bound = math.exp(delta * np.linalg.norm(q.astype(np.float64)))
        assert 1.0 / bound <= ratio <= bound
        assert ratio != 1.0


def test_identical_keys_one_center():
    n, d = 50, 4
    k = np.array([0.5, -0.25, 1.0, 2.0], dtype=np.float32)
    r = rng(7)
    o = OracleStream(d, 0.3, s=8, w=0)
    o.ingest(np.tile(k, (n, 1)), r.normal(size=(n, d)))
    q = np.array([0.2, 0.1, -0.3, 0.05], dtype=np.float32)
    _, den, mx = o.attend(q, return_den=True)
    assert o.m == 1 and o.counts.tolist() == [n]
    assert den * math.exp(mx) == pytest.approx(n * math.exp(float(k.astype(np.float64) @ q.astype(np.float64))),
                                               rel=1e-13)


def test_identical_values_closed_form():
    # all v equal: weights are n_evicted/s, so out = v * (sum_W e^a + n_ev/s sum_M e^c) / den
    r = rng(8)
    n, d, s, w = 120, 6, 16, 10
    K = r.normal(size=(n, d)).astype(np.float32)
    v = r.normal(size=d).astype(np.float32)
    o = OracleStream(d, 0.0, s=s, w=w)       # delta = 0: den is exact
    o.ingest(K, np.tile(v, (n, 1)))
    q = (r.normal(size=d) * 0.3).astype(np.float32)
    out = o.attend(q)
    K64, q64 = K.astype(np.float64), q.astype(np.float64)
    sampled = K64[o.sample_idx]
    numer = np.exp(K64[n - w:] @ q64).sum() + (n - w) / s * np.exp(sampled @ q64).sum()
    Z = np.exp(K64 @ q64).sum()
    assert np.allclose(out, v.astype(np.float64) * numer / Z, rtol=1e-11)


def test_estimator_is_unbiased_with_delta_zero():
    # Lemma 1 + row-norm sampling: E[z] = exp(K q)^T V; with delta = 0 tau is exact, so the
    # mean of the output over seeds converges to exact attention at rate 1/sqrt(seeds)
    r = rng(9)
    n, d, s, w = 60, 4, 8, 4
    K = r.normal(size=(n, d)).astype(np.float32)
    V = (r.normal(size=(n, d)) * r.uniform(0.5, 1.5, size=(n, 1))).astype(np.float32)
    q = (r.normal(size=d) * 0.5).astype(np.float32)
    exact = exact_attention(K, V, q)
    seeds = 4000
    outs = np.empty((seeds, d))
    for seed in range(seeds):
        o = OracleStream(d, 0.0, s=s, w=w, seed=seed)
        o.ingest(K, V)
        outs[seed] = o.attend(q)
    mean, sem = outs.mean(0), outs.std(0) / math.sqrt(seeds)
    assert (np.abs(mean - exact) < 4.5 * sem).all()
    # the single-seed error is not small (this is an estimator, not the exact value) ...
    assert np.abs(outs[0] - exact).max() > 10 * sem.max()
    # ... and averaging m seeds shrinks it like 1/sqrt(m)
    e1 = np.linalg.norm(outs[:40].mean(0) - exact)
    e2 = np.linalg.norm(mean - exact)
    assert e2 < e1


def test_numerator_error_shrinks_with_sample_budget():
    # approximate matrix product: error ~ 1/sqrt(s) (Theorem 1 takes s = Omega(d / eps^2))
    r = rng(11)
    n, d = 400, 8
    K = (r.normal(size=(n, d)) * 0.7).astype(np.float32)
    V = r.normal(size=(n, d)).astype(np.float32)
    q = (r.normal(size=d) * 0.5).astype(np.float32)
    exact = exact_attention(K, V, q)
    err = {}
    for s in [16, 1024]:
        es = []
        for seed in range(24):
            o = OracleStream(d, 0.0, s=s, w=0, seed=seed)
            o.ingest(K, V)
            es.append(np.linalg.norm(o.attend(q) - exact))
        err[s] = np.mean(es)
    assert 4.0 < err[16] / err[1024] < 16.0      # sqrt(64) = 8 expected


def test_query_sees_the_token_of_its_own_step():
    # main loop of Algorithm 1: update first, then query
    r = rng(12)
    d = 4
    o = OracleStream(d, 0.0, s=4, w=2)
    K, V = r.normal(size=(2, d)).astype(np.float32), r.normal(size=(2, d)).astype(np.float32)
    o.update(K[0], V[0])
    o.update(K[1], V[1])
    q = r.normal(size=d).astype(np.float32)
    assert np.allclose(o.attend(q), exact_attention(K, V, q), rtol=1e-13)


def test_ingest_and_decode_are_loops_of_update_and_attend():
    r = rng(13)
    n, d = 90, 8
    K, V = r.normal(size=(n, d)).astype(np.float32), r.normal(size=(n, d)).astype(np.float32)
    Q = r.normal(size=(20, 2, d)).astype(np.float32)
    a = OracleStream(d, 2.0, s=8, w=6, seed=5, stream=3)
    b = OracleStream(d, 2.0, s=8, w=6, seed=5, stream=3)
    a.ingest(K[:50], V[:50])
    a.ingest(K[50:70], V[50:70])
    outs = a.decode(K[70:], V[70:], Q)
    ref = np.empty_like(outs)
    for t in range(n):
        b.update(K[t], V[t])
        if t >= 70:
            for h in range(2):
                ref[t - 70, h] = b.attend(Q[t - 70, h])
    assert np.array_equal(outs, ref)
    assert np.array_equal(a.sample_idx, b.sample_idx) and np.array_equal(a.counts, b.counts)
    # a different stream id draws different coins
    c = OracleStream(d, 2.0, s=8, w=6, seed=5, stream=4)
    c.ingest(K, V)
    assert not np.array_equal(c.sample_idx, b.sample_idx)


def test_exact_attention_against_library_softmax_and_uniform_case():
    import torch
    r = rng(14)
    K, V, q = r.normal(size=(33, 5)), r.normal(size=(33, 5)), r.normal(size=5)
    ref = torch.softmax(torch.from_numpy(K) @ torch.from_numpy(q), 0) @ torch.from_numpy(V)
    assert np.allclose(exact_attention(K, V, q), ref.numpy(), rtol=1e-12)
    assert np.allclose(exact_attention(np.zeros((7, 3)), V[:7, :3], q[:3]), V[:7, :3].mean(0), rtol=1e-13)


# --------------------------------------------------------------------------
# per-cluster reservoirs S_i (t >= 1): Algorithm 1 as printed (UpdateSoftmaxNormalizer, Lemma 2 (5),
# the tau line of QueryStreamAttn, Theorem 1's bound on tau)
# --------------------------------------------------------------------------
from oracle.subgen_oracle import uniform24_res  # noqa: E402


def test_reservoir_coin_counter_layout():
    seed, stream, token = 0x0123456789ABCDEF, 5, (3 << 32) + 77
    for slot in [0, 1, 5, 63]:
        words = philox4x32_10([slot // 4, token & 0xFFFFFFFF, (token >> 32) | 0x80000000, stream],
                              [seed & 0xFFFFFFFF, seed >> 32])
        assert uniform24_res(seed, stream, token, slot) == (words[slot % 4] >> 8) / 2.0 ** 24
        assert uniform24_res(seed, stream, token, slot) != uniform24(seed, stream, token, slot)


def test_reservoir_does_not_change_clustering_or_sampling():
    r = rng(20)
    n, d = 300, 6
    K = (r.normal(size=(8, d))[r.integers(0, 8, size=n)] * 3 + 0.3 * r.normal(size=(n, d))).astype(np.float32)
    V = r.normal(size=(n, d)).astype(np.float32)
    a = OracleStream(d, 1.2, s=8, w=4, seed=3)
    b = OracleStream(d, 1.2, s=8, w=4, seed=3, t=3)
    a.ingest(K, V)
    b.ingest(K, V)
    assert np.array_equal(a.assign, b.assign) and np.array_equal(a.counts, b.counts)
    assert np.array_equal(a.sample_idx, b.sample_idx) and a.mu == b.mu
    # every reservoir entry is a member of its own cluster (Lemma 2 (5): samples from C_i)
    ev = K[: n - 4]
    R = b.reservoirs
    for i in range(b.m):
        members = ev[b.assign == i]
        for j in range(3):
            assert (members == R[i, j]).all(axis=1).any()


def test_new_cluster_reservoir_is_t_copies_and_second_member_probability_half():
    o = OracleStream(1, 1.0, s=1, w=0, t=5)
    o.update([7.0], [1.0])
    assert np.array_equal(o.reservoirs, np.full((1, 5, 1), 7.0, dtype=np.float32))
    # second member of the cluster: each slot is replaced with probability 1/2
    t = 20000
    o = OracleStream(1, 1.0, s=1, w=0, t=t, seed=4)
    o.update([0.0], [1.0])
    o.update([0.5], [1.0])
    frac = (o.reservoirs[0, :, 0] == 0.5).mean()
    assert abs(frac - 0.5) < 5 * math.sqrt(0.25 / t)


def test_lemma2_reservoir_is_uniform_over_the_cluster_and_slots_independent():
    # one cluster of 9 distinguishable members (all within delta of the first)
    keys = np.array([[0.01 * i] for i in range(9)], dtype=np.float32)
    seeds = 5000
    hist = np.zeros((3, 9))
    joint = np.zeros((9, 9))
    for seed in range(seeds):
        o = OracleStream(1, 1.0, s=1, w=0, t=3, seed=seed)
        o.ingest(keys, np.ones((9, 1)))
        assert o.m == 1
        idx = np.rint(o.reservoirs[0, :, 0] / 0.01).astype(int)
        hist[np.arange(3), idx] += 1
        joint[idx[0], idx[1]] += 1
    for j in range(3):   # chi-square, 8 dof: 99.99% quantile ~ 31
        chi = ((hist[j] - seeds / 9.0) ** 2 / (seeds / 9.0)).sum()
        assert chi < 36.0, (j, chi)
    exp = seeds / 81.0
    chi = ((joint - exp) ** 2 / exp).sum()   # 80 dof
    assert chi < 80 + 6 * math.sqrt(160)


def test_tau_is_unbiased_and_tightens_with_t():
    # E[(n_i/t) sum_{k in S_i} e^{<q,k>}] = sum_{k in C_i} e^{<q,k>}: the mean of tau over seeds is the exact
    # partition function, and its spread shrinks like 1/sqrt(t) (the proof of Theorem 1 uses exactly this)
    r = rng(21)
    n, d, delta = 240, 6, 2.0
    K = (r.normal(size=(6, d))[r.integers(0, 6, size=n)] * 2.5 + 0.45 * r.normal(size=(n, d))).astype(np.float32)
    V = r.normal(size=(n, d)).astype(np.float32)
    q = (r.normal(size=d) * 0.8).astype(np.float32)
    Z = np.exp(K.astype(np.float64) @ q.astype(np.float64)).sum()
    spread = {}
    for t in (1, 16):
        taus = []
        for seed in range(1500 if t == 1 else 300):
            o = OracleStream(d, delta, s=2, w=5, seed=seed, t=t)
            o.ingest(K, V)
            assert o.m < n // 3
            _, den, mx = o.attend(q, return_den=True)
            taus.append(den * math.exp(mx))
        taus = np.array(taus)
        sem = taus.std() / math.sqrt(len(taus))
        assert abs(taus.mean() - Z) < 4.5 * sem, (t, taus.mean(), Z, sem)
        spread[t] = taus.std() / Z
    assert spread[1] > 0.01                       # a single sample per cluster is visibly noisy ...
    assert 2.5 < spread[1] / spread[16] < 6.5     # ... and 16 samples cut the noise about 4-fold
    # representative mode on the same data is deterministic but biased: it is not the exact Z
    o = OracleStream(d, delta, s=2, w=5)
    o.ingest(K, V)
    _, den, mx = o.attend(q, return_den=True)
    assert abs(den * math.exp(mx) / Z - 1.0) > 1e-3


def test_tau_within_one_plus_minus_eps_for_large_t():
    # Theorem 1 (tau bound): with t of the order eps^-2 e^{2 delta r} log n, tau is within (1 +- eps/3) Z
    r = rng(22)
    n, d, delta = 400, 8, 1.0
    K = (r.normal(size=(10, d))[r.integers(0, 10, size=n)] * 3 + 0.2 * r.normal(size=(n, d))).astype(np.float32)
    V = r.normal(size=(n, d)).astype(np.float32)
    q = (r.normal(size=d) / math.sqrt(d)).astype(np.float32)
    rq = float(np.linalg.norm(q))
    eps = 0.3
    t = int(math.ceil(eps ** -2 * math.exp(2 * delta * rq) * math.log(n)))
    Z = np.exp(K.astype(np.float64) @ q.astype(np.float64)).sum()
    bad = 0
    for seed in range(120):
        o = OracleStream(d, delta, s=2, w=0, seed=seed, t=t)
        o.ingest(K, V)
        _, den, mx = o.attend(q, return_den=True)
        bad += abs(den * math.exp(mx) / Z - 1.0) > eps / 3
    assert bad <= 1, (bad, t)


def test_delta_zero_reservoirs_give_exact_partition_function():
    r = rng(23)
    n, d = 150, 5
    K = r.normal(size=(25, d)).astype(np.float32)[r.integers(0, 25, size=n)]
    o = OracleStream(d, 0.0, s=4, w=3, t=2, seed=1)
    o.ingest(K, r.normal(size=(n, d)))
    q = r.normal(size=d).astype(np.float32)
    _, den, mx = o.attend(q, return_den=True)
    assert den * math.exp(mx) == pytest.approx(np.exp(K.astype(np.float64) @ q.astype(np.float64)).sum(), rel=1e-12)


# --------------------------------------------------------------------------
# one-shot greedy k-center compression (Section 3.2: applied once to the whole cache, r recent tokens kept)
# --------------------------------------------------------------------------
from itertools import combinations  # noqa: E402

from oracle.subgen_oracle import greedy_kcenter, kcenter_compress  # noqa: E402


def test_greedy_kcenter_matches_integer_brute_force_traversal():
    r = rng(30)
    pts = r.integers(-9, 10, size=(40, 3))
    sel, assign, mind = greedy_kcenter(pts, 7)
    # pure-Python farthest-point traversal in exact integer arithmetic
    chosen = [0]
    md = [sum((int(a) - int(b)) ** 2 for a, b in zip(p, pts[0])) for p in pts]
    for _ in range(6):
        j = max(range(len(pts)), key=lambda i: (md[i], -i))
        chosen.append(j)
        md = [min(m0, sum((int(a) - int(b)) ** 2 for a, b in zip(p, pts[j]))) for m0, p in zip(md, pts)]
    assert sel.tolist() == chosen and mind.astype(int).tolist() == md
    # assignment = nearest chosen center, lowest on ties
    D = ((pts[:, None, :] - pts[sel][None]) ** 2).sum(-1)
    assert np.array_equal(assign, D.argmin(1))


def test_greedy_kcenter_is_a_two_approximation():
    # Gonzalez / Dyer-Frieze guarantee: the greedy radius is at most twice the optimal k-center radius
    r = rng(31)
    pts = r.normal(size=(14, 2))
    k = 3
    _, _, mind = greedy_kcenter(pts, k)
    greedy_radius = math.sqrt(mind.max())
    D = np.linalg.norm(pts[:, None] - pts[None], axis=-1)
    opt = min(D[:, list(c)].min(1).max() for c in combinations(range(len(pts)), k))
    assert greedy_radius <= 2.0 * opt + 1e-12
    assert greedy_radius >= opt - 1e-12


def test_greedy_kcenter_separated_groups_and_radii():
    r = rng(32)
    base = np.array([[0.0, 0.0], [50.0, 0.0], [0.0, 50.0], [50.0, 50.0], [25.0, 90.0]])
    lab = r.integers(0, 5, size=200)
    lab[0] = 0
    pts = base[lab] + r.normal(size=(200, 2))
    sel, assign, mind = greedy_kcenter(pts, 5)
    assert sorted(lab[sel].tolist()) == [0, 1, 2, 3, 4]                 # one center per group
    assert all(len(set(lab[assign == i])) == 1 for i in range(5))       # clusters are the groups
    assert len(set(sel.tolist())) == 5 and sel[0] == 0
    # the selection radius never increases
    radii = [greedy_kcenter(pts, kk)[2].max() for kk in range(1, 9)]
    assert all(a >= b for a, b in zip(radii, radii[1:]))


def test_kcenter_compress_layout_and_edge_cases():
    r = rng(33)
    K, V = r.normal(size=(30, 4)), r.normal(size=(30, 4))
    idx, counts = kcenter_compress(K, V, k=6, r=5)
    assert idx[6:].tolist() == [25, 26, 27, 28, 29] and idx[0] == 0 and (idx[:6] < 25).all()
    assert counts.sum() == 25 and len(set(idx[:6].tolist())) == 6
    idx, counts = kcenter_compress(K[:8], V[:8], k=6, r=5)               # only 3 old tokens: 3 centers, rest unused
    assert idx.tolist() == [0, 2, 1, -1, -1, -1, 3, 4, 5, 6, 7] or sorted(idx[:3].tolist()) == [0, 1, 2]
    assert idx[3:6].tolist() == [-1, -1, -1] and counts.sum() == 3
    idx, counts = kcenter_compress(K[:3], V[:3], k=2, r=5)               # fewer tokens than the window
    assert idx.tolist() == [-1, -1, 0, 1, 2, -1, -1] and counts.sum() == 0


# --------------------------------------------------------------------------
# tokens with NaN / Inf (the paper is silent; reading: dropped when they leave the window)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("w", [0, 3])
def test_nonfinite_tokens_are_dropped_and_leave_the_rest_untouched(w):
    r = rng(31)
    n, d = 120, 8
    K = (r.normal(size=(5, d))[r.integers(0, 5, size=n)] * 3 + 0.2 * r.normal(size=(n, d))).astype(np.float32)
    V = r.normal(size=(n, d)).astype(np.float32)
    bad = {17: ("k", np.nan), 40: ("v", np.inf), 41: ("k", -np.inf), 90: ("v", np.nan)}
    Kb, Vb = K.copy(), V.copy()
    for i, (which, val) in bad.items():
        (Kb if which == "k" else Vb)[i, 3] = val
    keep = np.array([i for i in range(n) if i not in bad])
    a = OracleStream(d, 1.0, s=6, w=w, seed=9)
    a.ingest(Kb, Vb)
    # clustering and mu do not depend on token numbers: they must equal those of the stream with the bad
    # tokens removed beforehand (once every bad token has left the window, i.e. compare on evicted tokens)
    n_ev = n - w
    keep_ev = keep[keep < n_ev]
    c = OracleStream(d, 1.0, s=6, w=0, seed=9)
    c.ingest(K[keep_ev], V[keep_ev])
    assert a.dropped == sum(1 for i in bad if i < n_ev) and c.dropped == 0
    assert a.m == c.m and np.array_equal(a.counts, c.counts) and np.array_equal(a.centers, c.centers)
    assert a.mu == c.mu
    assert a.counts.sum() + a.window_fill == n - a.dropped
    full = a.assign
    assert np.array_equal(full[keep_ev], c.assign) and all(full[i] == -1 for i in bad if i < n_ev)
    # a dropped token is never a sample; the coins of the others keep their own token numbers
    assert not set(a.sample_idx.tolist()) & set(bad)
    for j, tok in enumerate(a.sample_idx):
        assert tok in keep_ev and np.array_equal(a.sample_k[j], K[tok]) and np.array_equal(a.sample_v[j], V[tok])
    # squared norms beyond fp32 count as non-finite
    b = OracleStream(d, 1.0, s=2, w=0, seed=1)
    big = np.full((1, d), 3e19, dtype=np.float32)
    b.ingest(big, V[:1])
    assert b.dropped == 1 and b.m == 0


# --------------------------------------------------------------------------
# decision log and near-tie margins (what the parity harness forgives by)
# --------------------------------------------------------------------------
def test_decision_log_distances_and_margins_on_hand_built_line():
    """1-D keys with distances known by hand (Algorithm 1, UpdateSoftmaxNormalizer: nearest representative,
    threshold delta).  delta = 1, representatives end up at 0 and 1.5."""
    o = OracleStream(1, 1.0, s=1, w=0, max_centers=2)
    keys = [0.0,      # opens cluster 0: no representative yet
            1.5,      # 1.5 > delta from 0: opens cluster 1, nearest is 0 at 1.5
            1.0,      # 1.0 from 0, 0.5 from 1.5: joins 1; runner-up 0 exactly at delta
            -1.0,     # exactly delta from 0 (threshold hit, margin 0); runner-up 1.5 at 2.5, outside delta
            0.7,      # 0.7 from 0, 0.8 from 1.5: both within delta, gap (0.8-0.7)/0.7
            0.25,     # 0.25 from 0, 1.25 from 1.5: runner-up outside delta
            9.5]      # 8 from 1.5, table full (capacity 2): forced join to cluster 1
    o.ingest(np.array(keys)[:, None], np.ones((len(keys), 1)))
    assert o.assign.tolist() == [0, 1, 1, 0, 0, 0, 1]
    assert o.created.tolist() == [1, 1, 0, 0, 0, 0, 0]
    assert o.counts.tolist() == [4, 3] and o.overflowed
    # squared distances in binary floating point of these decimal keys, computed the long way round
    f = lambda x: float(np.float32(x))
    d1 = [math.inf, 2.25, 0.25, 1.0, (f(0.7) - 0.0) ** 2, 0.0625, 64.0]
    d2 = [math.inf, math.inf, 1.0, 6.25, (1.5 - f(0.7)) ** 2, 1.5625, 90.25]
    assert o.dist1.tolist() == d1
    assert o.dist2.tolist() == d2
    thr, gap = o.margins()
    assert thr[0] == math.inf and gap[0] == math.inf             # nothing to compare with
    assert thr[1] == 0.5 and gap[1] == math.inf                  # |1.5 - 1| / 1, no runner-up
    assert thr[2] == 0.5 and gap[2] == 1.0                       # runner-up exactly at delta counts as inside: (1-.5)/.5
    assert thr[3] == 0.0 and gap[3] == math.inf                  # exact threshold hit; runner-up outside delta
    assert thr[4] == pytest.approx(0.3, rel=1e-6) and gap[4] == pytest.approx(0.1 / 0.7, rel=1e-6)
    assert thr[5] == 0.75 and gap[5] == math.inf                 # runner-up at 1.25 > delta
    assert thr[6] == 7.0 and gap[6] == math.inf                  # forced join: far outside the threshold


def test_margins_flag_exactly_the_planted_near_ties():
    """A key at delta(1 + eps) from its nearest representative has threshold margin eps; two representatives at
    distances r and r(1 + eps), both inside delta, have gap eps.  Anything the harness forgives must look like that."""
    for eps in (3e-6, 1e-3):
        o = OracleStream(1, 2.0, s=1, w=0)
        o.ingest(np.array([0.0, 2.0 * (1.0 + eps), -3.0, -3.0 + 1.0, -3.0 - (1.0 + eps) + 2.0 * (1.0 + eps)])[:, None],
                 np.ones((5, 1)))
        thr, gap = o.margins()
        assert thr[1] == pytest.approx(eps, rel=2e-2) and (thr[1] < 1e-5) == (eps < 1e-5)
        assert o.assign.tolist()[:4] == [0, 1, 2, 2] and thr[3] == 0.5
    o = OracleStream(1, 2.0, s=1, w=0)
    r = 1.0
    for eps in (4e-6, 1e-2):
        o = OracleStream(1, 2.0, s=1, w=0)
        o.ingest(np.array([0.0, 2.0 * r + r * eps, r])[:, None], np.ones((3, 1)))     # r from 0, r(1+eps) from the other
        thr, gap = o.margins()
        assert o.assign.tolist() == [0, 1, 0]
        assert gap[2] == pytest.approx(eps, rel=2e-2) and (gap[2] < 1e-5) == (eps < 1e-5)
        assert thr[2] == 0.5
    # on generic data no decision is anywhere near a tie
    g = rng(5)
    o = OracleStream(8, 2.5, s=2, w=3)
    o.ingest(g.normal(size=(400, 8)), g.normal(size=(400, 8)))
    thr, gap = o.margins()
    assert min(thr.min(), gap.min()) > 1e-5 and o.m > 5


def test_forced_decisions_replace_the_rule_only_at_their_token():
    """The override list of the near-tie protocol: the forced token takes the given decision, every other
    token follows Algorithm 1 on the state that results (integer keys on a line, expectations worked out by hand)."""
    keys = np.array([0, 10, 4, 5, 9, 14, 3, -2])[:, None].astype(float)
    vals = np.ones((8, 1))
    plain = OracleStream(1, 4.0, s=2, w=0)
    plain.ingest(keys, vals)
    assert plain.assign.tolist() == [0, 1, 0, 2, 1, 1, 2, 0]           # 4 joins 0 (distance 4 = delta), 5 opens 2
    forced = OracleStream(1, 4.0, s=2, w=0)
    forced.set_overrides({2: OracleStream.FORCE_NEW, 5: 0})
    forced.ingest(keys, vals)
    # token 2 (key 4) opens cluster 2 instead; then 5 joins it (distance 1), 9 joins 1, 14 is forced into 0,
    # 3 is nearest to 4 (cluster 2), -2 joins 0
    assert forced.assign.tolist() == [0, 1, 2, 2, 1, 0, 2, 0]
    assert forced.created.tolist() == [1, 1, 1, 0, 0, 0, 0, 0]
    assert forced.counts.tolist() == [3, 2, 3] and forced.overrides_used == 2
    assert forced.centers[:, 0].tolist() == [0.0, 10.0, 4.0]
    # sampling is untouched by the clustering decision
    assert forced.mu == plain.mu and forced.sample_idx.tolist() == plain.sample_idx.tolist()
    # an empty list changes nothing; a list may not be given to a stream that has started
    again = OracleStream(1, 4.0, s=2, w=0)
    again.set_overrides({})
    again.ingest(keys, vals)
    assert again.assign.tolist() == plain.assign.tolist()
    with pytest.raises(ValueError):
        again.set_overrides({1: 0})


def test_long_stream_samples_are_uniform_over_the_tokens_when_norms_are_equal():
    """Lemma 1 at the length of the long-context workload: with equal ||v|| every slot holds a token drawn
    uniformly from all tokens seen, also beyond token 2^16 and with coin probabilities down to 2^-17 (chi-square over
    16 equal ranges of the token index; slots of one stream are independent, three seeds)."""
    n, s, bins = 140000, 512, 16
    K = np.zeros((n, 2), dtype=np.float32)
    V = np.ones((n, 2), dtype=np.float32)
    counts = np.zeros(bins)
    for seed in (1, 2, 3):
        o = OracleStream(2, 1.0, s=s, w=0, seed=seed)
        o.ingest(K, V)
        idx = o.sample_idx
        assert idx.min() >= 0 and idx.max() < n and o.m == 1 and o.mu == 2.0 * n
        counts += np.bincount(idx * bins // n, minlength=bins)
    expected = 3 * s / bins
    chi2 = float(((counts - expected) ** 2 / expected).sum())
    assert chi2 < 37.7, (chi2, counts)          # chi-square, 15 degrees of freedom, p = 0.001
    assert counts[-1] > 0 and counts[0] > 0
