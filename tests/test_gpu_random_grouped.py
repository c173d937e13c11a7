"""Seeded random grouped steps against the oracle: shapes drawn so that they cross the choices the
library makes from the true number of distinct histories, which only the device knows (weight
streaming inside the staged, tiled and three-term kernels at <= 64 rows, the two shapes of the hidden
update, the work split of the output projection), in both number types and all three
log-sum-exp modes."""
import numpy as np
import pytest

import oracle
import paper_2007_11794_amd as rn
from workloads import CONFIGS, make_model, make_step_inputs

from harness import gpu_step_dedup, load_model

pytestmark = pytest.mark.gpu

HIDDEN = [64, 128, 192, 256, 320, 512, 576, 640, 768, 1024, 1216, 1280, 2048]
VOCAB = [300, 1000, 2049, 4096, 5000, 9001, 20000]
RAW = [1, 7, 40, 100, 257, 300, 513, 700, 1100, 2100, 4100, 5000]
DISTINCT = [1, 2, 31, 32, 33, 63, 64, 65, 100, 129, 200, 256, 300, 513, 600]


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_random_grouped_steps(seed):
    rng = np.random.default_rng(seed)
    for case in range(12):
        dtype = str(rng.choice(["bf16", "f32"]))
        H = int(rng.choice(HIDDEN))
        if dtype == "f32":
            H = min(H, 1024)
        V, N = int(rng.choice(VOCAB)), int(rng.choice(RAW))
        distinct = int(min(N, rng.choice(DISTINCT)))
        if V * H * distinct > 3e9:                       # keeps the oracle's share of the test short
            V = 2049
        K = int(rng.choice([1, 3, 8, 9, 17]))
        cfg = CONFIGS[3 if dtype == "bf16" else 2].scaled(V=V, H=H, B=N, K=K)
        model = make_model(cfg)
        x = make_step_inputs(cfg, rng)
        pick = rng.integers(0, distinct, N)
        pick[:distinct] = np.arange(distinct)
        pick = rng.permutation(pick)
        keys = (pick.astype(np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
        prev, h_in = x["prev"][pick], x["h_in"][pick]
        m = load_model(model, dtype, N)
        lse_mode = int(rng.choice([0, 1, 2]))
        m.set_option(rn.OPT_LSE_MODE, lse_mode)
        out = gpu_step_dedup(m, keys, prev, h_in, x["query"])
        what = "seed %d case %d: %s V=%d H=%d N=%d distinct=%d K=%d lse=%d" % (seed, case, dtype, V, H, N, distinct, K, lse_mode)
        U, rep, inv = oracle.dedup(keys)
        assert out["n_unique"] == U == distinct, what
        assert np.array_equal(out["rep"], rep) and np.array_equal(out["inverse"], inv), what
        ref = oracle.step(model, prev[rep], h_in[rep], x["query"], row_of_query=inv)
        tol_h, tol_lp = (1e-3, 2e-3) if dtype == "bf16" else (1e-5, 1e-5)
        assert np.max(np.abs(out["h_out"][:U] - ref["h_out"])) <= tol_h, what
        assert np.max(np.abs(out["logprob"] - ref["logprob"])) <= tol_lp, what
        assert m.last_error() == 0, what
        m.close()
