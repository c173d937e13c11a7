"""Pins for the oracle's cache that outlives a step (Table 1; Sections 3.2, 4.2, 5.3).

Expected values come from: the already pinned oracle.step / oracle.dedup on the special
case "nothing cached"; Python dict/set bookkeeping of which histories are stored; numpy /
scipy evaluations of the queried log-probabilities; closed forms (zero weights); literal
bit patterns for the packed index.
"""
import math

import numpy as np
import pytest
import scipy.special

import oracle


def rand_model(rng, V, H, sigma=0.3, bias=True):
    return {"U": rng.normal(0, sigma, (V, H)).astype(np.float32),
            "W": rng.normal(0, sigma, (H, H)).astype(np.float32),
            "O": rng.normal(0, sigma, (H, V)).astype(np.float32),
            "bias": rng.normal(0, sigma, V).astype(np.float32) if bias else None}


def rand_step(rng, V, H, N, K, id_pool):
    ids = rng.choice(id_pool, size=N).astype(np.uint64)
    # rows with equal ids carry equal histories (the id is the context index)
    by_id = {}
    prev = np.zeros(N, np.int32)
    h_in = np.zeros((N, H), np.float32)
    for n in range(N):
        if int(ids[n]) not in by_id:
            by_id[int(ids[n])] = (rng.integers(0, V), rng.uniform(0, 1, H).astype(np.float32))
        prev[n], h_in[n] = by_id[int(ids[n])]
    query = rng.integers(0, V, (N, K)).astype(np.int32)
    return ids, prev, h_in, query


def library_logprob(m, prev_row, h_row, words):
    """log-softmax at `words` for one history, from numpy + scipy in float64."""
    U, W, O = (m[k].astype(np.float64) for k in ("U", "W", "O"))
    h = scipy.special.expit(U[prev_row] + W @ h_row.astype(np.float64))
    z = h @ O + (0.0 if m["bias"] is None else m["bias"].astype(np.float64))
    return z[words] - scipy.special.logsumexp(z), h


# ------------------------------------------------------------------ nothing cached
@pytest.mark.parametrize("cache_kind", ["none", "capacity0", "empty"])
def test_without_stored_entries_equals_plain_step(cache_kind):
    rng = np.random.default_rng(11)
    V, H, N, K = 97, 12, 40, 5
    m = rand_model(rng, V, H)
    ids, prev, h_in, query = rand_step(rng, V, H, N, K, np.arange(1000, 1013, dtype=np.uint64))
    cache = {"none": None, "capacity0": oracle.Cache(H, 0), "empty": oracle.Cache(H, 64)}[cache_kind]
    got = oracle.step_cached(m, cache, ids, prev, h_in, query)
    U_, rep, inverse = oracle.dedup(ids)
    ref = oracle.step(m, prev[rep], h_in[rep], query, row_of_query=inverse)
    assert got["n_unique"] == U_
    assert np.array_equal(got["rep"], rep) and np.array_equal(got["inverse"], inverse)
    assert np.array_equal(got["h_out"], ref["h_out"])          # same arithmetic, same order
    assert np.array_equal(got["lse"], ref["lse"])
    assert np.array_equal(got["score"], ref["logprob"])
    assert got["stats"][:3] == (U_, 0, U_)
    assert got["stats"][3] == {"none": 0, "capacity0": 0, "empty": U_}[cache_kind]


# ------------------------------------------------------------------ stored values are returned
def test_hit_returns_stored_value_whatever_the_inputs_say():
    rng = np.random.default_rng(12)
    V, H, N, K = 64, 9, 24, 4
    m = rand_model(rng, V, H)
    cache = oracle.Cache(H, 100)
    ids, prev, h_in, query = rand_step(rng, V, H, N, K, np.arange(50, 58, dtype=np.uint64))
    first = oracle.step_cached(m, cache, ids, prev, h_in, query)
    # same ids and queries, but prev / h_in that would give other numbers if recomputed
    prev2 = (prev + 1) % V
    h2 = (1.0 - h_in).astype(np.float32)
    second = oracle.step_cached(m, cache, ids, prev2, h2, query)
    assert second["stats"] == (first["n_unique"], first["n_unique"], 0, first["n_unique"])
    assert np.array_equal(second["h_out"], first["h_out"])
    assert np.array_equal(second["score"], first["score"])
    # and recomputation really would differ
    fresh = oracle.step_cached(m, None, ids, prev2, h2, query)
    assert np.abs(fresh["score"] - first["score"]).max() > 1e-3


def test_values_against_numpy_scipy_over_three_steps():
    rng = np.random.default_rng(13)
    V, H, K = 211, 17, 6
    m = rand_model(rng, V, H)
    cache = oracle.Cache(H, 1000)
    stored = {}                     # id -> (prev, h_in) that were current when it was first computed
    pool = (np.arange(40, dtype=np.uint64) << np.uint64(32)) | np.uint64(7)
    for step in range(3):
        N = 30 + 5 * step
        ids = rng.choice(pool, size=N).astype(np.uint64)
        prev = rng.integers(0, V, N).astype(np.int32)
        h_in = rng.uniform(0, 1, (N, H)).astype(np.float32)
        # rows of one id agree within the step; across steps the inputs change on purpose
        first_of = {}
        for n in range(N):
            f = first_of.setdefault(int(ids[n]), n)
            prev[n], h_in[n] = prev[f], h_in[f]
        query = rng.integers(0, V, (N, K)).astype(np.int32)
        base = rng.normal(-5, 2, (N, K)).astype(np.float32)
        got = oracle.step_cached(m, cache, ids, prev, h_in, query, base_score=base)
        hits = len({int(i) for i in ids} & set(stored))
        for n in range(N):
            stored.setdefault(int(ids[n]), (prev[n], h_in[n].copy()))
        assert got["stats"] == (len(first_of), hits, len(first_of) - hits, len(stored))
        for n in range(N):
            p, h = stored[int(ids[n])]
            want, hvec = library_logprob(m, p, h, query[n])
            assert got["score"][n] == pytest.approx(want - base[n].astype(np.float64), abs=1e-11)
            assert got["h_out"][got["inverse"][n]] == pytest.approx(hvec, abs=1e-13)


# ------------------------------------------------------------------ bookkeeping
@pytest.mark.parametrize("capacity", [0, 1, 7, 25, 1000])
def test_bookkeeping_against_python_sets(capacity):
    rng = np.random.default_rng(100 + capacity)
    V, H, K = 16, 3, 2
    m = rand_model(rng, V, H)
    cache = oracle.Cache(H, capacity)
    stored = []                      # ids in the order they were stored
    totals = dict(lookups=0, hits=0, misses=0, unstored=0)
    pool = rng.integers(0, 2 ** 63, 60, dtype=np.uint64) | np.uint64(1 << 63)
    pool[0] = np.uint64(0xFFFFFFFFFFFFFFFF)                   # an ordinary key like any other
    pool[1] = np.uint64(0)
    for step in range(6):
        N = int(rng.integers(1, 40))
        ids, prev, h_in, query = rand_step(rng, V, H, N, K, pool)
        got = oracle.step_cached(m, cache, ids, prev, h_in, query)
        order = list(dict.fromkeys(int(i) for i in ids))      # first-appearance order
        hits = [i for i in order if i in stored]
        misses = [i for i in order if i not in stored]
        room = capacity - len(stored)
        stored += misses[:max(room, 0)]
        totals["lookups"] += len(order); totals["hits"] += len(hits); totals["misses"] += len(misses)
        totals["unstored"] += len(misses) - min(len(misses), max(room, 0))
        assert got["stats"] == (len(order), len(hits), len(misses), len(stored))
        assert [int(ids[r]) for r in got["rep"]] == order
    s = cache.stats()
    assert s == dict(entries=len(stored), **totals)
    assert s["entries"] <= capacity
    cache.reset()
    assert cache.stats() == dict(entries=0, lookups=0, hits=0, misses=0, unstored=0)
    ids, prev, h_in, query = rand_step(rng, V, H, 5, K, pool[:3])
    got = oracle.step_cached(m, cache, ids, prev, h_in, query)
    assert got["stats"][1] == 0                               # nothing survives a reset


def test_full_cache_keeps_the_first_histories_in_order_of_appearance():
    rng = np.random.default_rng(14)
    V, H, K = 32, 4, 3
    m = rand_model(rng, V, H)
    cache = oracle.Cache(H, 3)
    ids = np.array([9, 4, 9, 7, 2, 4, 8], dtype=np.uint64)    # appearance order 9 4 7 2 8
    _, prev, h_in, query = rand_step(rng, V, H, len(ids), K, ids)
    first_of = {}
    for n in range(len(ids)):
        f = first_of.setdefault(int(ids[n]), n)
        prev[n], h_in[n] = prev[f], h_in[f]
    a = oracle.step_cached(m, cache, ids, prev, h_in, query)
    assert a["stats"] == (5, 0, 5, 3)
    probe = np.array([2, 8, 7, 4, 9], dtype=np.uint64)
    _, p2, h2, q2 = rand_step(rng, V, H, len(probe), K, probe)
    b = oracle.step_cached(m, cache, probe, p2, h2, q2)
    assert b["stats"] == (5, 3, 2, 3)                         # 9, 4, 7 were kept; 2 and 8 were not
    # the kept ones answer from the first step's histories
    for n, key in enumerate(probe):
        if int(key) in (9, 4, 7):
            src = first_of[int(key)]
            want, _ = library_logprob(m, prev[src], h_in[src], q2[n])
        else:
            want, _ = library_logprob(m, p2[n], h2[n], q2[n])
        assert b["score"][n] == pytest.approx(want, abs=1e-11)


# ------------------------------------------------------------------ difference to the base score
def test_zero_weights_score_is_minus_log_V_minus_base():
    V, H, N, K = 50, 6, 4, 3
    m = {"U": np.zeros((V, H), np.float32), "W": np.zeros((H, H), np.float32),
         "O": np.zeros((H, V), np.float32), "bias": None}
    base = np.array([[-1.5, 0.0, 2.25]] * N, dtype=np.float32)
    got = oracle.step_cached(m, oracle.Cache(H, 8), np.arange(N, dtype=np.uint64), np.zeros(N, np.int32),
                             np.full((N, H), 0.3, np.float32), np.zeros((N, K), np.int32), base_score=base)
    assert got["score"] == pytest.approx(-math.log(V) - base.astype(np.float64), abs=1e-14)


def test_base_score_sign():
    rng = np.random.default_rng(15)
    V, H, N, K = 40, 5, 6, 4
    m = rand_model(rng, V, H)
    ids, prev, h_in, query = rand_step(rng, V, H, N, K, np.arange(6, dtype=np.uint64))
    base = rng.normal(-4, 1, (N, K)).astype(np.float32)
    plain = oracle.step_cached(m, None, ids, prev, h_in, query)
    diff = oracle.step_cached(m, None, ids, prev, h_in, query, base_score=base)
    assert diff["score"] == pytest.approx(plain["score"] - base.astype(np.float64), abs=1e-12)
    assert np.all((diff["score"] > plain["score"]) == (base < 0))


# ------------------------------------------------------------------ packed index
def test_pack_ids_bit_patterns():
    got = oracle.pack_ids([0, 1, 0xFFFFFFFF, 0x12345678, 0], [0, 2, 0xFFFFFFFF, 0x9ABCDEF0, 0xFFFFFFFF])
    assert [int(x) for x in got] == [0, 0x0000000100000002, 0xFFFFFFFFFFFFFFFF, 0x123456789ABCDEF0,
                                     0x00000000FFFFFFFF]
    # the two halves come back by shifting and masking
    assert [int(x) >> 32 for x in got] == [0, 1, 0xFFFFFFFF, 0x12345678, 0]
    assert [int(x) & 0xFFFFFFFF for x in got] == [0, 2, 0xFFFFFFFF, 0x9ABCDEF0, 0xFFFFFFFF]
