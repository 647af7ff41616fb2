"""Host-side pieces of the measurement tools (no GPU): the least-squares fit of Eq. 3
recovers known coefficients, the paper-shaped iterations it samples have the advertised
shape, and bench.py refuses more than one GPU."""
import subprocess
import sys

import numpy as np

from paper_2509_17357_amd import fit_eq3
from paper_2509_17357_amd import workloads as W


def test_fit_recovers_a_linear_model():
    rng = np.random.default_rng(3)
    k1, k2, b = 7.0e-6, 6.5e-7, 0.08
    rows = []
    for lp, nd, tot in fit_eq3.sample_grid(512):
        t = k1 * lp + k2 * tot + b
        rows.append({"l_ctxp": lp, "n_d": nd, "l_ctxd": tot, "ms": t * (1 + 1e-3 * rng.standard_normal())})
    res, pred = fit_eq3.fit(rows)
    assert abs(res["k_ctxp_ms_per_token"] / k1 - 1) < 0.02
    assert abs(res["k_ctxd_ms_per_token"] / k2 - 1) < 0.02
    assert abs(res["b_c_ms"] / b - 1) < 0.02
    assert res["r2"] > 0.999 and res["mape_percent"] < 0.5 and len(pred) == len(rows)


def test_sampled_iterations_have_the_paper_shape():
    for i, (lp, nd, tot) in enumerate(fit_eq3.sample_grid(512)):
        b = fit_eq3.make_batch(W, lp, nd, tot, 512, seed=9000 + i)
        assert b.total_q == 512 and b.n_seqs == nd + 1
        assert b.prefix_lens[0] == lp and b.chunk_lens[0] == 512 - nd
        assert int((b.prefix_lens[1:] + 1).sum()) == tot          # decode contexts include the current token
        assert (b.chunk_lens[1:] == 1).all() and (b.prefix_lens[1:] >= 1).all()


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, "bench.py", "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
