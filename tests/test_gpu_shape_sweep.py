"""A seeded sweep over small, awkward shapes (odd hidden sizes, vocabularies below one tile, one
row, many words per query, duplicates), every entry point, both element types, against the
oracle.  The shapes are drawn once from a fixed seed: the test is deterministic."""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_11794_amd as rn
from workloads import round_to_bf16

from harness import CachedStepper, gpu_step, gpu_step_dedup, load_model

pytestmark = pytest.mark.gpu

TOL = {"f32": (1e-5, 1e-5), "bf16": (2e-3, 1e-3)}


def shapes():
    rng = np.random.default_rng(20071179)
    out = []
    for i in range(36):
        dtype = "bf16" if i % 2 else "f32"
        V = int(rng.choice([2, 3, 31, 33, 255, 257, 1000, 4097, 6000]))
        H = int(rng.choice([1, 3, 4, 63, 64, 65, 100, 128, 130, 256, 300, 512, 516, 700]))
        B = int(rng.choice([1, 2, 31, 33, 63, 64, 65, 127, 129, 255, 257, 400]))
        K = int(rng.choice([1, 2, 7, 8, 9, 16, 17, 33, 70]))
        out.append((i, dtype, V, H, B, K))
    return out


@pytest.mark.parametrize("i,dtype,V,H,B,K", shapes())
def test_shape(i, dtype, V, H, B, K):
    rng = np.random.default_rng(1000 + i)
    sigma = 0.4 / np.sqrt(H)
    model = {"U": rng.normal(0, 0.3, (V, H)).astype(np.float32), "W": rng.normal(0, sigma, (H, H)).astype(np.float32),
             "O": rng.normal(0, sigma * 2, (H, V)).astype(np.float32), "bias": rng.normal(0, 0.5, V).astype(np.float32)}
    if dtype == "bf16":
        for k in ("U", "W", "O"):
            model[k] = round_to_bf16(model[k])
    N = B + int(rng.integers(0, 2 * B + 1))
    m = load_model(model, dtype, N)
    tol_lp, tol_h = TOL[dtype]
    # distinct rows + fan-out
    prev = rng.integers(0, V, B).astype(np.int32)
    h_in = rng.uniform(0, 1, (B, H)).astype(np.float32)
    if i % 3 == 0:
        h_in[0] = 0.0                                   # utterance start
    roq = np.concatenate([np.arange(B), rng.integers(0, B, N - B)]).astype(np.int32)
    query = rng.integers(0, V, (N, K)).astype(np.int32)
    ref = oracle.step(model, prev, h_in, query, row_of_query=roq)
    Hp = max(128, -(-H // 64) * 64)                      # the staged kernel exists for padded sizes 128, 256, 512
    # 5: weight streaming where the rows fit (at most 128), else as 0
    kernels = [0, 1, 3, 5] + ([2] if dtype == "bf16" and Hp in (128, 256, 512) else []) + ([4] if dtype == "f32" else []) + \
              ([6] if dtype == "bf16" else [])
    for kernel in kernels:
        m.set_option(rn.OPT_OUTPROJ_KERNEL, kernel)
        for lse_mode in (0, 1):
            m.set_option(rn.OPT_LSE_MODE, lse_mode)
            h, lp = gpu_step(m, prev, h_in, query, roq)
            dh, dlp = np.max(np.abs(h - ref["h_out"])), np.max(np.abs(lp - ref["logprob"]))
            assert dh <= tol_h and dlp <= tol_lp, (i, dtype, V, H, B, K, kernel, lse_mode, dh, dlp)
    m.set_option(rn.OPT_OUTPROJ_KERNEL, 0)
    m.set_option(rn.OPT_LSE_MODE, 0)
    # the same through ids: raw query n carries the history of row roq[n]
    ids = (roq.astype(np.uint64) * np.uint64(0x9E3779B97F4A7C15)) ^ np.uint64(i)
    out = gpu_step_dedup(m, ids, prev[roq], h_in[roq], query)
    U_, rep, inv = oracle.dedup(ids)
    assert out["n_unique"] == U_ == B and np.array_equal(out["rep"], rep) and np.array_equal(out["inverse"], inv)
    ref2 = oracle.step(model, prev[roq][rep], h_in[roq][rep], query, row_of_query=inv)
    assert np.max(np.abs(out["logprob"] - ref2["logprob"])) <= tol_lp
    assert np.max(np.abs(out["h_out"] - ref2["h_out"])) <= tol_h
    # and through a cache, twice: the second time everything is found
    cache = rn.rnnlm_cache_create(m, 2 * B)
    st = CachedStepper(m, cache, N, K)
    a = st.step(ids, prev[roq], h_in[roq], query)
    b = st.step(ids, prev[roq], h_in[roq], query)
    assert a["stats"] == (B, 0, B, B) and b["stats"] == (B, B, 0, B)
    assert np.max(np.abs(a["score"] - ref2["logprob"])) <= tol_lp and np.array_equal(a["score"], b["score"])
    assert m.last_error() == 0
    cache.close()
    m.close()
