"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr + r.stdout and "{" not in r.stdout      # no result line


def test_without_a_gpu_the_bench_fails_loudly():
    if torch.cuda.is_available():
        return                                   # covered by the GPU runs
    r = run("--steps", "1", "--warmup", "0", "--no-cpu-baseline")
    assert r.returncode != 0 and '"metric"' not in r.stdout             # no CPU fallback, no number


def test_cpu_leg_times_the_oracle_on_given_streams_and_compares_decisions(tmp_path):
    """The CPU-baseline child of bench.py: fed the rows of two streams and a decision log, it reports the oracle's
    rate and how the log compares with the oracle's own decisions (here the log is the oracle's, once as it is and
    once with one entry changed far from any tie)."""
    import json
    import numpy as np
    from oracle.subgen_oracle import OracleStream
    from paper_2402_06082_amd.workloads import CONFIGS, Workload
    cfg = CONFIGS["cfg2"]
    prefix, steps, ids, delta = 400, 40, [0, 3], 8.2
    wl = Workload(cfg, device="cpu", streams=4)
    K, V = wl.tokens(0, prefix + steps)
    Q = wl.queries(0, steps)
    logs = []
    for i in ids:
        o = OracleStream(cfg.d, delta, cfg.s, cfg.w, seed=0, stream=i)
        o.ingest(K[i].float().numpy(), V[i].float().numpy())
        logs.append(o.assign[: prefix + 10 - cfg.w].copy())
    raw = lambda t: t.view(torch.int16).numpy()
    for planted in (False, True):
        assign = np.stack(logs)
        if planted:
            assign[1, 200] += 1
        for name, arr in [("K", raw(K[ids])), ("V", raw(V[ids])), ("Q", raw(Q[ids])), ("ids", np.array(ids)),
                          ("assign", assign)]:
            np.save(tmp_path / f"{name}.npy", arr)
        r = run("--cpu-baseline-worker", str(tmp_path), "--config", "cfg2", "--delta", repr(delta), "--prefix",
                str(prefix))
        assert r.returncode == 0, r.stderr
        out = json.loads(r.stdout.strip().splitlines()[-1])
        assert out["streams"] == 2 and out["steps"] == steps and out["stream_steps_per_s"] > 0
        assert out["near_ties"] == 0 and out["mismatches"] == (1 if planted else 0)
        assert out["decisions_compared"] == (assign.shape[1] + 201 if planted else 2 * assign.shape[1])
