"""Randomised parity: shapes, dtypes, kernel paths and options drawn from a seed, every trial checked against the
oracle (state bit for bit, outputs within tolerance) after a split prefix ingest, a few fused steps and one block of
queries.  The trial's parameters are printed before it runs."""
import numpy as np
import pytest
import torch

from tests.parity_util import REL_L2_TOL, compare_state, make_oracles, rel_l2, to_f32_np

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def one_trial(trial, big):
    from paper_2402_06082_amd import binding as b
    r = np.random.default_rng(trial)
    bf16 = r.random() < 0.7
    dtype = torch.bfloat16 if bf16 else torch.float32
    d = int(r.choice([64, 128, 128, 256] if bf16 else [32, 64, 128]))
    g = int(r.choice([1, 1, 2, 4]))
    if big:
        S = int(r.choice([1, 2, 3, 260]))
        s, w = int(r.integers(1, 700)), int(r.choice([0, 5, 64, 127, 128, 129, 300]))
        n, steps, C = int(r.integers(200, 2500)), int(r.integers(1, 6)), int(r.integers(20, 400))
    else:
        S = int(r.choice([1, 2, 3, 5, 130, 300]))
        s, w = int(r.integers(1, 200)), int(r.choice([0, 1, 3, 17, 64, 80]))
        n, steps, C = int(r.integers(1, 260)), int(r.integers(1, 12)), int(r.integers(2, 12))
    t = int(r.choice([0, 0, 0, 1, 3]))
    path = int(r.choice([0, 0, 1, 2]))
    scale = float(r.choice([0.0, 0.8, 1.0, 1.2]))
    maxc = int(r.choice([0, 0, 4, 64]))
    devcnt = bool(r.random() < 0.3)
    print(f"trial {trial}: bf16={bf16} d={d} g={g} S={S} s={s} w={w} n={n} steps={steps} t={t} path={path} C={C} "
          f"scale={scale} max_centers={maxc} device_counter={devcnt}", flush=True)
    gen = torch.Generator(device="cpu").manual_seed(trial)
    N = n + steps
    cent = torch.randn(S, C, d, generator=gen) * 2.0
    comp = torch.randint(0, C, (S, N), generator=gen)
    K = torch.gather(cent, 1, comp[..., None].expand(S, N, d)) + 0.2 * torch.randn(S, N, d, generator=gen)
    V = torch.randn(S, N, d, generator=gen) * torch.exp(0.5 * torch.randn(S, N, 1, generator=gen))
    Q = torch.randn(S, N, g, d, generator=gen) / d ** 0.5
    K, V, Q = (x.to(dtype).to(DEV) for x in (K, V, Q))
    delta = 0.2 * (2 * d) ** 0.5 * scale
    ids = sorted({0, S - 1, S // 2})
    sg = b.SubGen(S, d, delta, s, w, dtype=dtype, q_per_stream=g, max_centers=maxc, assign_log_tokens=N, seed=trial,
                  device=DEV, kernel_path=path, t_per_cluster=t, device_counter=devcnt)
    orc = make_oracles(S, d, delta, s, w, seed=trial, max_centers=maxc if maxc else 4096, stream_ids=ids, t=t)
    Kc, Vc, Qc = to_f32_np(K[ids]), to_f32_np(V[ids]), to_f32_np(Q[ids])
    cut = int(r.integers(0, n + 1))
    for lo, hi in [(0, cut), (cut, n)]:
        if hi > lo:
            sg.ingest_prefix(K[:, lo:hi].contiguous(), V[:, lo:hi].contiguous())
    for i, o in enumerate(orc):
        o.ingest(Kc[i, :n], Vc[i, :n])
    assert compare_state(sg, orc, stream_ids=ids) == 0
    for tt in range(n, N):
        out = sg.step(K[:, tt].contiguous(), V[:, tt].contiguous(), Q[:, tt].contiguous()).cpu().numpy()
        ref = np.stack([o.decode(Kc[i, tt:tt + 1], Vc[i, tt:tt + 1], Qc[i, tt:tt + 1])[0] for i, o in enumerate(orc)])
        assert rel_l2(out[ids], ref).max() <= REL_L2_TOL, ("step", tt)
    assert compare_state(sg, orc, stream_ids=ids) == 0
    nq = int(r.choice([1, 3, 16, 17, 40, 70]))
    Qm = (torch.randn(S, nq, d, generator=gen) / d ** 0.5).to(dtype).to(DEV)
    om = sg.attend_many(Qm).cpu().numpy()
    Qmc = to_f32_np(Qm[ids])
    refm = np.stack([[o.attend(Qmc[i, h]) for h in range(nq)] for i, o in enumerate(orc)])
    assert rel_l2(om[ids], refm).max() <= REL_L2_TOL, ("attend_many", nq)
    sg.close()


@pytest.mark.parametrize("first", [0, 20, 40, 60])
def test_random_small_states(first):
    for trial in range(first, first + 20):
        one_trial(trial, big=False)


@pytest.mark.parametrize("first", [5000, 5008])
def test_random_states_of_several_blocks(first):
    for trial in range(first, first + 8):
        one_trial(trial, big=True)
