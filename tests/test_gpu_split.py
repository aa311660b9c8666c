"""Several workgroups per stream (opts.split_workgroups; automatic in contexts of at most 32 streams): every
workgroup scans a share of the rows, the last one to arrive combines the partial results and takes the decision.
State must equal the oracle's bit for bit for any number of workgroups, outputs within the usual tolerance."""
import numpy as np
import pytest
import torch

from tests.parity_util import REL_L2_TOL, compare_state, make_oracles, rel_l2, to_f32_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def clustered(S, n, d, g, seed, ncent=7, spread=0.2):
    gen = torch.Generator(device="cpu").manual_seed(seed)
    cent = torch.randn(S, ncent, d, generator=gen) * 2.0
    comp = torch.randint(0, ncent, (S, n), generator=gen)
    K = torch.gather(cent, 1, comp[..., None].expand(S, n, d)) + spread * torch.randn(S, n, d, generator=gen)
    V = torch.randn(S, n, d, generator=gen) * torch.exp(0.5 * torch.randn(S, n, 1, generator=gen))
    Q = torch.randn(S, n, g, d, generator=gen) / d ** 0.5
    return K, V, Q


@pytest.mark.parametrize("P", [2, 3, 8, 33, 64])
@pytest.mark.parametrize("dtype,d,g,s,w", [(torch.bfloat16, 128, 1, 37, 9), (torch.bfloat16, 128, 4, 130, 0),
                                           (torch.float32, 64, 1, 64, 32), (torch.bfloat16, 64, 2, 5, 70),
                                           (torch.bfloat16, 256, 1, 16, 3), (torch.float32, 32, 4, 1, 1)])
def test_split_step_update_attend_match_the_oracle(P, dtype, d, g, s, w):
    """Row counts below, at and above what P workgroups x 4 blocks cover; windows longer than the token count at
    first; s = 1; fused steps, then update and attend apart, on top of an ingested prefix."""
    from paper_2402_06082_amd import binding as b
    S, n0, n = 3, 90, 150
    K, V, Q = clustered(S, n, d, g, seed=P + d + s)
    K, V, Q = (x.to(dtype).to(DEV) for x in (K, V, Q))
    delta = 0.2 * (2 * d) ** 0.5 * 1.02
    sg = b.SubGen(S, d, delta, s, w, dtype=dtype, q_per_stream=g, assign_log_tokens=n, seed=5, device=DEV,
                  split_workgroups=P)
    one = b.SubGen(S, d, delta, s, w, dtype=dtype, q_per_stream=g, assign_log_tokens=n, seed=5, device=DEV,
                   split_workgroups=1)
    oracles = make_oracles(S, d, delta, s, w, seed=5)
    Kc, Vc, Qc = to_f32_np(K), to_f32_np(V), to_f32_np(Q)
    for t in range(n):
        kt, vt, qt = K[:, t].contiguous(), V[:, t].contiguous(), Q[:, t].contiguous()
        if t < n0 or t % 3:
            out = sg.step(kt, vt, qt)
            ref1 = one.step(kt, vt, qt)
        else:
            sg.update(kt, vt)
            out = sg.attend(qt)
            one.update(kt, vt)
            ref1 = one.attend(qt)
        ref = np.stack([o.decode(Kc[i, t:t + 1], Vc[i, t:t + 1], Qc[i, t:t + 1])[0] for i, o in enumerate(oracles)])
        assert np.isfinite(out.cpu().numpy()).all(), t
        assert rel_l2(out.cpu().numpy(), ref).max() <= REL_L2_TOL, t
        assert rel_l2(out.cpu().numpy(), ref1.cpu().numpy().astype(np.float64)).max() <= 1e-5, t
        if t in (0, w - 1, w, w + 1, n0, n - 1):
            assert compare_state(sg, oracles) == 0
    assert compare_state(sg, oracles) == 0 and compare_state(one, oracles) == 0
    assert sg.center_counts().max() >= 5


@pytest.mark.parametrize("P", [4, 32])
def test_split_exact_ties_duplicates_overflow_and_nonfinite_tokens(P):
    """Lattice keys (equal distances, distances exactly at the threshold), a full center table, NaN/Inf tokens."""
    from paper_2402_06082_amd import binding as b
    S, n, d, s, w = 4, 300, 128, 16, 5
    gen = torch.Generator(device="cpu").manual_seed(P)
    K = torch.randint(-1, 2, (S, n, d), generator=gen).float() * 0.5
    K[:, :, 8:] = 0.0
    V = torch.randn(S, n, d, generator=gen)
    Q = torch.randn(S, n, 1, d, generator=gen) / d ** 0.5
    K[0, 40, 3] = float("nan")
    V[1, 77, 0] = float("inf")
    K, V, Q = (t.to(torch.bfloat16).to(DEV) for t in (K, V, Q))
    for max_centers in (0, 9):
        sg = b.SubGen(S, d, 1.0, s, w, dtype=torch.bfloat16, assign_log_tokens=n, seed=2, device=DEV,
                      split_workgroups=P, max_centers=max_centers)
        oracles = make_oracles(S, d, 1.0, s, w, seed=2, max_centers=max_centers)
        outs = torch.stack([sg.step(K[:, t].contiguous(), V[:, t].contiguous(), Q[:, t].contiguous()) for t in range(n)])
        ref = np.stack([o.decode(to_f32_np(K[i]), to_f32_np(V[i]), to_f32_np(Q[i])) for i, o in enumerate(oracles)], 1)
        assert compare_state(sg, oracles) == 0
        ok = np.isfinite(ref).all(axis=(2, 3))
        assert rel_l2(outs.cpu().numpy()[ok], ref[ok]).max() <= REL_L2_TOL
        margins = [o.margins() for o in oracles]           # the data really is full of exact ties
        assert sum(int((thr == 0).sum()) for thr, _ in margins) > 20 and sum(int((gap == 0).sum()) for _, gap in margins) >= 1
        st = sg.stats()
        assert st.flags_or == (b.FLAG_NONFINITE | (b.FLAG_CENTER_OVERFLOW if max_centers else 0))
        assert [o.dropped for o in oracles] == [1, 1, 0, 0]


def test_split_is_chosen_for_small_contexts_and_survives_graph_replay():
    """The automatic choice (at most 32 streams) under HIP-graph replay: the arrival counters are left at zero by
    every launch, so a captured step can be replayed."""
    from paper_2402_06082_amd import binding as b
    S, d, g, s, w, n0, n = 2, 128, 1, 12, 5, 40, 70
    K, V, Q = clustered(S, n, d, g, seed=1)
    K, V, Q = (x.to(torch.bfloat16).to(DEV) for x in (K, V, Q))
    delta = 0.2 * (2 * d) ** 0.5 * 1.05
    oracles = make_oracles(S, d, delta, s, w, seed=8)
    Kc, Vc, Qc = to_f32_np(K), to_f32_np(V), to_f32_np(Q)
    for i, o in enumerate(oracles):
        o.ingest(Kc[i, :n0], Vc[i, :n0])
    side = torch.cuda.Stream(device=DEV)
    side.wait_stream(torch.cuda.current_stream(DEV))
    with torch.cuda.stream(side):
        sg = b.SubGen(S, d, delta, s, w, dtype=torch.bfloat16, assign_log_tokens=n, seed=8, device=DEV,
                      device_counter=True)
        sg.ingest_prefix(K[:, :n0].contiguous(), V[:, :n0].contiguous())
        kt, vt, qt = K[:, n0].clone(), V[:, n0].clone(), Q[:, n0].clone()
        out = torch.empty(S, g, d, dtype=torch.float32, device=DEV)
        sg.step(kt, vt, qt, out)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sg.step(kt, vt, qt, out)
    sg.sync()
    for i, o in enumerate(oracles):
        o.decode(Kc[i, n0:n0 + 1], Vc[i, n0:n0 + 1], Qc[i, n0:n0 + 1])
    for t in range(n0 + 1, n):
        with torch.cuda.stream(side):
            kt.copy_(K[:, t]); vt.copy_(V[:, t]); qt.copy_(Q[:, t])
            graph.replay()
        side.synchronize()
        ref = np.stack([o.decode(Kc[i, t:t + 1], Vc[i, t:t + 1], Qc[i, t:t + 1])[0] for i, o in enumerate(oracles)])
        assert rel_l2(out.cpu().numpy(), ref).max() <= REL_L2_TOL, t
    assert compare_state(sg, oracles) == 0
