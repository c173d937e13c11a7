"""Pins for the CPU oracle: closed forms, hand values, brute force, library routines.

None of these retypes the oracle's own code path: each expected value comes from a
closed form, a hand-computed fixture (tests/golden/onehot_tiny.txt), a pure-Python
brute-force evaluation of the definition, or a library routine (numpy matmul, scipy
logsumexp, torch log_softmax, numpy.unique).
"""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle
from workloads import CONFIGS, make_model, make_step_inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "onehot_tiny.txt")


def golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


def rand_model(rng, V, H, sigma=0.3, bias=True):
    return {"U": rng.normal(0, sigma, (V, H)).astype(np.float32),
            "W": rng.normal(0, sigma, (H, H)).astype(np.float32),
            "O": rng.normal(0, sigma, (H, V)).astype(np.float32),
            "bias": rng.normal(0, sigma, V).astype(np.float32) if bias else None}


# ------------------------------------------------------------------ hand values
def test_golden_case_A_onehot_embedding_and_output():
    g = golden()
    V, H = 4, 2
    m = {"U": np.zeros((V, H), np.float32), "W": np.zeros((H, H), np.float32),
         "O": np.zeros((H, V), np.float32), "bias": None}
    m["U"][1] = (math.log(3.0), 0.0)
    m["O"][0, 0] = 4.0 / 3.0 * math.log(2.0)
    out = oracle.step(m, prev=[1], h_in=[[0.3, 0.9]], query=[[0, 1, 2, 3]])
    # float32 storage of ln 3 and (4/3) ln 2 limits agreement to ~1e-7
    assert out["h_out"][0] == pytest.approx([g["A_h0"], g["A_h1"]], abs=1e-7)
    assert out["logprob"][0] == pytest.approx([g["A_logp0"]] + [g["A_logp1"]] * 3, abs=1e-7)


def test_golden_case_B_W_orientation():
    g = golden()
    V, H = 4, 2
    m = {"U": np.zeros((V, H), np.float32), "W": np.zeros((H, H), np.float32),
         "O": np.zeros((H, V), np.float32), "bias": None}
    m["W"][0, 1] = 2.0 * math.log(3.0)
    out = oracle.step(m, prev=[2], h_in=[[1.0, 0.5]], query=[[0]])
    assert out["h_out"][0] == pytest.approx([g["B_h0"], g["B_h1"]], abs=1e-7)


def test_golden_case_C_zero_weights_uniform():
    g = golden()
    for V, H in ((4, 2), (1000, 64)):
        m = {"U": np.zeros((V, H), np.float32), "W": np.zeros((H, H), np.float32),
             "O": np.zeros((H, V), np.float32), "bias": np.zeros(V, np.float32)}
        rng = np.random.default_rng(V)
        B, K = 3, 5
        out = oracle.step(m, prev=rng.integers(0, V, B), h_in=rng.random((B, H)),
                          query=rng.integers(0, V, (B, K)))
        assert np.all(out["h_out"] == 0.5)
        assert out["logprob"] == pytest.approx(-math.log(V), abs=1e-12)
        if V == 4:
            assert out["h_out"][0, 0] == g["C_h"]
            assert out["logprob"][0, 0] == pytest.approx(g["C_logp"], abs=1e-15)


# ------------------------------------------------------------------ closed forms
def test_zero_hidden_in_gives_sigmoid_of_embedding():
    rng = np.random.default_rng(7)
    V, H, B = 50, 12, 6
    m = rand_model(rng, V, H)
    prev = rng.integers(0, V, B)
    out = oracle.step(m, prev, np.zeros((B, H), np.float32), rng.integers(0, V, (B, 2)))
    expect = scipy.special.expit(m["U"][prev].astype(np.float64))
    assert np.max(np.abs(out["h_out"] - expect)) < 1e-15


def test_onehot_output_column_closed_form():
    rng = np.random.default_rng(11)
    V, H, B = 37, 9, 4
    t, c = 0.8, 5
    m = rand_model(rng, V, H, bias=False)
    m["O"][:] = 0
    m["O"][:, c] = np.float32(t)
    out = oracle.step(m, rng.integers(0, V, B), rng.random((B, H)), np.tile([c, 0], (B, 1)))
    s = out["h_out"].sum(axis=1) * float(np.float32(t))
    lse = np.log((V - 1) + np.exp(s))
    assert np.max(np.abs(out["lse"] - lse)) < 1e-12
    assert np.max(np.abs(out["logprob"][:, 0] - (s - lse))) < 1e-12
    assert np.max(np.abs(out["logprob"][:, 1] - (0 - lse))) < 1e-12


def test_probabilities_sum_to_one():
    cfg = CONFIGS[1]
    m = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed))
    out = oracle.step(m, x["prev"], x["h_in"], x["query"], want_full=True)
    total = np.exp(out["full_logp"]).sum(axis=1)
    assert np.max(np.abs(total - 1.0)) < 1e-9
    # the queried entries are entries of that same normalised distribution
    rows = np.arange(cfg.B)[:, None]
    assert np.array_equal(out["logprob"], out["full_logp"][rows, x["query"]])


def test_bias_shift_invariance_and_bias_is_used():
    rng = np.random.default_rng(3)
    V, H, B, K = 40, 8, 5, 6
    m = rand_model(rng, V, H)
    prev, h, q = rng.integers(0, V, B), rng.random((B, H)), rng.integers(0, V, (B, K))
    a = oracle.step(m, prev, h, q)
    m2 = dict(m, bias=(m["bias"] + np.float32(2.5)))
    b = oracle.step(m2, prev, h, q)
    # float32 bias + 2.5 is not exact; compare against the exactly shifted float32 values
    shift = m2["bias"].astype(np.float64) - m["bias"].astype(np.float64)
    assert np.max(np.abs(shift - 2.5)) < 1e-6
    assert np.max(np.abs(a["logprob"] - b["logprob"])) < 1e-6
    # zero O: the distribution is log_softmax(bias) whatever h is
    m3 = dict(m, O=np.zeros_like(m["O"]))
    c = oracle.step(m3, prev, h, q)
    ref = scipy.special.log_softmax(m["bias"].astype(np.float64))
    assert np.max(np.abs(c["logprob"] - ref[q])) < 1e-13


def test_large_logits_do_not_overflow():
    V, H = 2, 1
    m = {"U": np.full((V, H), 50.0, np.float32), "W": np.zeros((H, H), np.float32),
         "O": np.array([[1000.0, 0.0]], np.float32), "bias": None}
    out = oracle.step(m, [0], [[0.0]], [[0, 1]])
    hp = 1.0 / (1.0 + math.exp(-50.0))
    assert out["logprob"][0, 0] == pytest.approx(0.0, abs=1e-300)
    assert out["logprob"][0, 1] == pytest.approx(-1000.0 * hp, rel=1e-15)


# ------------------------------------------------------------------ brute force
def brute_force_step(m, prev, h_in, query):
    """The definition, term by term, in pure Python floats (doubles)."""
    V, H = m["U"].shape
    out_h, out_lp = [], []
    for b in range(len(prev)):
        hp = []
        for j in range(H):
            a = float(m["U"][prev[b]][j])
            for i in range(H):
                a += float(m["W"][j][i]) * float(h_in[b][i])
            hp.append(1.0 / (1.0 + math.exp(-a)))
        z = []
        for v in range(V):
            acc = float(m["bias"][v]) if m["bias"] is not None else 0.0
            for j in range(H):
                acc += float(m["O"][j][v]) * hp[j]
            z.append(acc)
        denom = sum(math.exp(zz) for zz in z)       # no max shift needed at these magnitudes
        out_h.append(hp)
        out_lp.append([math.log(math.exp(z[w]) / denom) for w in query[b]])
    return np.array(out_h), np.array(out_lp)


@pytest.mark.parametrize("V,H,B,K", [(2, 1, 1, 2), (7, 3, 4, 7), (16, 5, 6, 3), (16, 16, 3, 16)])
def test_brute_force_tiny(V, H, B, K):
    rng = np.random.default_rng(100 * V + H)
    m = rand_model(rng, V, H, sigma=0.7)
    prev = rng.integers(0, V, B).astype(np.int32)
    h_in = rng.random((B, H)).astype(np.float32)
    query = rng.integers(0, V, (B, K)).astype(np.int32)
    out = oracle.step(m, prev, h_in, query)
    bh, blp = brute_force_step(m, prev, h_in, query)
    assert np.max(np.abs(out["h_out"] - bh)) < 1e-14
    assert np.max(np.abs(out["logprob"] - blp)) < 1e-13


# ------------------------------------------------------------------ library routines
@pytest.mark.parametrize("V,H,B,K", [(300, 33, 17, 5), (1000, 64, 8, 4), (4099, 128, 9, 11)])
def test_against_numpy_scipy_torch(V, H, B, K):
    rng = np.random.default_rng(V)
    m = rand_model(rng, V, H, sigma=0.2)
    prev = rng.integers(0, V, B).astype(np.int32)
    h_in = rng.random((B, H)).astype(np.float32)
    query = rng.integers(0, V, (B, K)).astype(np.int32)
    out = oracle.step(m, prev, h_in, query)
    U, W, O, bias = (m[k].astype(np.float64) for k in ("U", "W", "O", "bias"))
    a = U[prev] + h_in.astype(np.float64) @ W.T          # W[j,i] multiplies h[i]
    hp = scipy.special.expit(a)
    z = hp @ O + bias
    lse = scipy.special.logsumexp(z, axis=1)
    assert np.max(np.abs(out["h_out"] - hp)) < 1e-13
    assert np.max(np.abs(out["lse"] - lse)) < 1e-11
    lp_torch = torch.log_softmax(torch.from_numpy(z), dim=1).numpy()
    rows = np.arange(B)[:, None]
    assert np.max(np.abs(out["logprob"] - lp_torch[rows, query])) < 1e-11


def test_row_of_query_fans_out():
    rng = np.random.default_rng(5)
    V, H, B, K, N = 60, 10, 4, 3, 11
    m = rand_model(rng, V, H)
    prev, h = rng.integers(0, V, B), rng.random((B, H))
    roq = rng.integers(0, B, N).astype(np.int32)
    q = rng.integers(0, V, (N, K)).astype(np.int32)
    out = oracle.step(m, prev, h, q, row_of_query=roq)
    # same thing asked row by row through the identity mapping
    full = oracle.step(m, prev, h, np.tile(np.arange(K), (B, 1)), want_full=True)["full_logp"]
    assert np.array_equal(out["logprob"], full[roq[:, None], q])


def test_bad_indices_are_rejected():
    rng = np.random.default_rng(5)
    m = rand_model(rng, 10, 4)
    with pytest.raises(ValueError):
        oracle.step(m, [10], rng.random((1, 4)), [[0]])
    with pytest.raises(ValueError):
        oracle.step(m, [0], rng.random((1, 4)), [[-1]])
    with pytest.raises(ValueError):
        oracle.step(m, [0], rng.random((1, 4)), [[0]], row_of_query=[1])


# ------------------------------------------------------------------ grouping of equal keys
def first_appearance_unique(keys):
    """numpy.unique re-ordered by first index (library routine)."""
    uniq, first, inv = np.unique(keys, return_index=True, return_inverse=True)
    order = np.argsort(first, kind="stable")
    rank = np.empty_like(order)
    rank[order] = np.arange(len(order))
    return len(uniq), first[order].astype(np.int32), rank[inv].astype(np.int32)


def brute_dedup(keys):
    rep, inverse = [], []
    for n, k in enumerate(keys):
        seen = [u for u, r in enumerate(rep) if keys[r] == k]
        if seen:
            inverse.append(seen[0])
        else:
            rep.append(n)
            inverse.append(len(rep) - 1)
    return len(rep), np.array(rep, np.int32), np.array(inverse, np.int32)


@pytest.mark.parametrize("N,distinct", [(0, 1), (1, 1), (2, 1), (64, 5), (64, 64), (1000, 37), (4096, 1229)])
def test_dedup_against_numpy_unique_and_brute_force(N, distinct):
    rng = np.random.default_rng(N + distinct)
    pool = rng.integers(0, 2 ** 64, size=distinct, dtype=np.uint64)
    pool[0] = np.uint64(0xFFFFFFFFFFFFFFFF)           # an all-ones key is an ordinary key
    if distinct > 1:
        pool[1] = np.uint64(0)
    keys = pool[rng.integers(0, distinct, size=N)]
    U, rep, inv = oracle.dedup(keys)
    U2, rep2, inv2 = first_appearance_unique(keys) if N else (0, np.zeros(0, np.int32), np.zeros(0, np.int32))
    assert U == U2 and np.array_equal(rep, rep2) and np.array_equal(inv, inv2)
    if N <= 64:
        U3, rep3, inv3 = brute_dedup(list(keys))
        assert U == U3 and np.array_equal(rep, rep3) and np.array_equal(inv, inv3)
    # invariants
    if N:
        assert np.array_equal(keys[rep[inv]], keys)
        assert np.all(np.diff(rep) > 0)
        assert np.array_equal(inv[rep], np.arange(U))
        assert U == len(set(keys.tolist()))


def test_dedup_keys_differing_in_one_half_are_distinct():
    hi = np.uint64(7) << np.uint64(32)
    keys = np.array([hi | np.uint64(1), hi | np.uint64(2), (np.uint64(8) << np.uint64(32)) | np.uint64(1),
                     hi | np.uint64(1)], dtype=np.uint64)
    U, rep, inv = oracle.dedup(keys)
    assert U == 3 and rep.tolist() == [0, 1, 2] and inv.tolist() == [0, 1, 2, 0]
