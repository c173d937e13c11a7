"""Pins for the oracle's hierarchical output layer (Section 2.1): Huffman tree and path
probabilities.  Expected values: hand-worked trees with and without ties
(tests/golden/huffman_ties.txt), a pure-Python restatement of the definition that finds the two
lightest live nodes by scanning, the cost of a construction on Python's heapq, exact Kraft
sums, the closed form for zero node vectors, a pure-Python evaluation of the path
probabilities, and the sum over all leaves."""
import heapq
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle


def lengths(off):
    return np.diff(off)


def heap_cost(freq):
    """Total weighted code length of an optimal prefix code = sum of all merged weights."""
    h = [float(f) for f in freq]
    heapq.heapify(h)
    cost = 0.0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def check_tree(V, off, entry):
    L = lengths(off)
    assert off[0] == 0 and off[-1] == len(entry) and np.all(L >= 1)
    # Kraft equality, exactly
    assert sum(Fraction(1, 2 ** int(l)) for l in L) == 1
    node = entry & 0x7FFFFFFF
    assert node.min() == 0 and node.max() == V - 2
    # every word starts at the root; paths are consistent: (node, bit) determines the next node
    nxt = {}
    leaf = {}
    for v in range(V):
        p = entry[off[v]:off[v + 1]]
        assert (p[0] & 0x7FFFFFFF) == V - 2
        for a, b in zip(p[:-1], p[1:]):
            key = (int(a) & 0x7FFFFFFF, (int(a) >> 31) & 1)
            assert nxt.setdefault(key, int(b) & 0x7FFFFFFF) == (int(b) & 0x7FFFFFFF)
        key = (int(p[-1]) & 0x7FFFFFFF, (int(p[-1]) >> 31) & 1)
        assert key not in leaf and key not in nxt
        leaf[key] = v
    # every inner node has exactly two children
    assert len(nxt) + len(leaf) == 2 * (V - 1)
    for n in range(V - 1):
        assert ((n, 0) in nxt or (n, 0) in leaf) and ((n, 1) in nxt or (n, 1) in leaf)


def golden_trees():
    """{case: (freq, [path of word 0, ...])}, a path being a list of node | bit << 31 entries."""
    raw = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "huffman_ties.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                key, *vals = line.split()
                raw[key] = vals
    cases = {}
    for key, vals in raw.items():
        case, what = key.split("_")
        if what == "freq":
            freq = [float(v) for v in vals]
            paths = []
            for w in range(len(freq)):
                steps = [s.split(".") for s in raw["%s_w%d" % (case, w)]]
                paths.append([int(n) | (int(b) << 31) for n, b in steps])
            cases[case] = (freq, paths)
    return cases


def paths_of(off, entry):
    return [[int(e) & 0xFFFFFFFF for e in entry[off[v]:off[v + 1]]] for v in range(len(off) - 1)]


def scan_huffman(freq):
    """The definition, by scanning: nodes 0 .. V-1 are the words, node V + n the n-th inner node
    made; take the two live nodes of least (weight, node number), the first gets code bit 0."""
    V = len(freq)
    weight = {v: float(freq[v]) for v in range(V)}
    parent = {}
    for n in range(V - 1):
        a = min(weight, key=lambda x: (weight[x], x))
        wa = weight.pop(a)
        b = min(weight, key=lambda x: (weight[x], x))
        wb = weight.pop(b)
        parent[a], parent[b] = (n, 0), (n, 1)
        weight[V + n] = wa + wb
    paths = []
    for v in range(V):
        p, x = [], v
        while x in parent:
            n, bit = parent[x]
            p.append(n | (bit << 31))
            x = V + n
        paths.append(p[::-1])
    return paths


@pytest.mark.parametrize("case", ["T1", "T2", "T3", "T4", "T5"])
def test_hand_worked_trees(case):
    freq, paths = golden_trees()[case]
    off, entry = oracle.huffman_build(freq)
    assert paths_of(off, entry) == paths
    assert scan_huffman(freq) == paths            # the restatement used below reads the same rule


@pytest.mark.parametrize("V,levels", [(2, 1), (3, 1), (9, 2), (40, 3), (200, 4), (500, 1000)])
def test_same_tree_as_the_scan_on_many_ties(V, levels):
    rng = np.random.default_rng(V * 31 + levels)
    for _ in range(4):
        freq = rng.integers(1, levels + 1, V).astype(np.float64)
        off, entry = oracle.huffman_build(freq)
        assert paths_of(off, entry) == scan_huffman(freq)
        check_tree(V, off, entry)


def test_textbook_example():
    off, entry = oracle.huffman_build([5, 9, 12, 13, 16, 45])
    assert lengths(off).tolist() == [4, 4, 3, 3, 3, 1]
    check_tree(6, off, entry)
    # the lighter of the first merge (5) is the child with code bit 0
    assert (entry[off[0 + 1] - 1] >> 31) & 1 == 0 and (entry[off[1 + 1] - 1] >> 31) & 1 == 1


@pytest.mark.parametrize("V,s", [(2, 0.0), (3, 1.0), (64, 0.0), (1000, 1.1), (5000, 1.0), (65536, 1.1)])
def test_tree_is_valid_and_optimal(V, s):
    freq = np.arange(1, V + 1, dtype=np.float64) ** -s * 1e6
    off, entry = oracle.huffman_build(freq)
    if V <= 5000:
        check_tree(V, off, entry)
    L = lengths(off)
    assert float(np.dot(freq, L)) == pytest.approx(heap_cost(freq), rel=1e-12)
    assert np.all(np.diff(L) >= 0) or s == 0.0             # rarer words never get shorter codes
    if s == 0.0 and V == 64:
        assert np.all(L == 6)


def rand_model(rng, V, H, sigma=0.5, freq=None):
    freq = rng.uniform(1, 100, V) if freq is None else freq
    off, entry = oracle.huffman_build(freq)
    return {"U": rng.normal(0, sigma, (V, H)).astype(np.float32), "W": rng.normal(0, sigma, (H, H)).astype(np.float32),
            "theta": rng.normal(0, sigma, (V - 1, H)).astype(np.float32), "path_off": off, "path_entry": entry}


@pytest.mark.parametrize("V,H", [(2, 1), (7, 3), (100, 8), (1000, 16)])
def test_leaves_sum_to_one(V, H):
    rng = np.random.default_rng(V)
    m = rand_model(rng, V, H)
    B = 3
    out = oracle.hs_step(m, rng.integers(0, V, B), rng.uniform(0, 1, (B, H)).astype(np.float32),
                         np.zeros((B, 1), np.int32), want_full=True)
    assert np.exp(out["full_logp"]).sum(axis=1) == pytest.approx(np.ones(B), abs=1e-12)
    assert np.all(out["full_logp"] < 0)


def test_zero_node_vectors_give_two_to_minus_length():
    rng = np.random.default_rng(2)
    V, H = 50, 4
    m = rand_model(rng, V, H)
    m["theta"][:] = 0
    out = oracle.hs_step(m, [0], rng.uniform(0, 1, (1, H)).astype(np.float32), np.arange(V, dtype=np.int32)[None, :])
    assert out["logprob"][0] == pytest.approx(-math.log(2.0) * lengths(m["path_off"]), abs=1e-13)


def test_two_words_is_one_sigmoid():
    m = {"U": np.zeros((2, 2), np.float32), "W": np.zeros((2, 2), np.float32),
         "theta": np.array([[1.5, -0.5]], np.float32)}
    m["path_off"], m["path_entry"] = oracle.huffman_build([1.0, 3.0])      # word 0 lighter: code bit 0
    out = oracle.hs_step(m, [0], [[0.2, 0.9]], [[0, 1]])
    x = 0.5 * 1.5 - 0.5 * 0.5                                              # h' = sigmoid(0) = 1/2 each
    assert out["logprob"][0] == pytest.approx([math.log(scipy.special.expit(x)), math.log(scipy.special.expit(-x))],
                                              abs=1e-15)


@pytest.mark.parametrize("V,H,B,K", [(5, 2, 2, 5), (33, 7, 4, 6)])
def test_against_pure_python(V, H, B, K):
    rng = np.random.default_rng(V + H)
    m = rand_model(rng, V, H)
    prev = rng.integers(0, V, B)
    h_in = rng.uniform(0, 1, (B, H)).astype(np.float32)
    N = B + 3
    roq = rng.integers(0, B, N).astype(np.int32)
    query = rng.integers(0, V, (N, K)).astype(np.int32)
    out = oracle.hs_step(m, prev, h_in, query, row_of_query=roq)
    for n in range(N):
        b = int(roq[n])
        hp = [1.0 / (1.0 + math.exp(-(float(m["U"][prev[b], j]) + sum(float(m["W"][j, i]) * float(h_in[b, i]) for i in range(H)))))
              for j in range(H)]
        for k in range(K):
            w = int(query[n, k])
            p = 1.0
            for e in m["path_entry"][m["path_off"][w]:m["path_off"][w + 1]]:
                node, bitv = int(e) & 0x7FFFFFFF, (int(e) >> 31) & 1
                x = sum(float(m["theta"][node, j]) * hp[j] for j in range(H))
                p *= 1.0 / (1.0 + math.exp(x if bitv else -x))
            assert out["logprob"][n, k] == pytest.approx(math.log(p), abs=1e-12)


def test_extreme_activations_stay_finite():
    rng = np.random.default_rng(4)
    m = rand_model(rng, 9, 3)
    m["theta"] *= 400.0
    out = oracle.hs_step(m, [1], [[0.3, 0.3, 0.3]], np.arange(9, dtype=np.int32)[None, :], want_full=True)
    assert np.all(np.isfinite(out["logprob"])) and np.exp(out["full_logp"]).sum() == pytest.approx(1.0, abs=1e-12)


# ------------------------------------------------------------------ through the cache (Table 1 around Section 2.1)
def numpy_path_logp(model, h, word):
    """log p(word | h) from numpy: the product of sigmoids along the word's path."""
    off, entry = model["path_off"], model["path_entry"].view(np.uint32)
    lp = 0.0
    for e in entry[off[word]:off[word + 1]]:
        x = float(model["theta"][int(e & 0x7FFFFFFF)].astype(np.float64) @ h)
        lp += -np.logaddexp(0.0, x if (e >> 31) else -x)
    return lp


def cached_case(rng, V, H, N, K, pool):
    freq = rng.zipf(1.3, V).astype(np.float64)
    off, entry = oracle.huffman_build(freq)
    model = {"U": rng.normal(0, 0.3, (V, H)).astype(np.float32), "W": rng.normal(0, 0.3, (H, H)).astype(np.float32),
             "theta": rng.normal(0, 0.6, (V - 1, H)).astype(np.float32), "path_off": off, "path_entry": entry}
    ids = rng.choice(pool, size=N).astype(np.uint64)
    by_id, prev, h_in = {}, np.zeros(N, np.int32), np.zeros((N, H), np.float32)
    for n in range(N):
        if int(ids[n]) not in by_id:
            by_id[int(ids[n])] = (rng.integers(0, V), rng.uniform(0, 1, H).astype(np.float32))
        prev[n], h_in[n] = by_id[int(ids[n])]
    return model, ids, prev, h_in, rng.integers(0, V, (N, K)).astype(np.int32)


@pytest.mark.parametrize("cache_kind", ["none", "capacity0", "empty"])
def test_cached_step_without_stored_entries_is_grouping_plus_plain_step(cache_kind):
    rng = np.random.default_rng(5)
    V, H, N, K = 61, 9, 30, 4
    model, ids, prev, h_in, query = cached_case(rng, V, H, N, K, np.arange(500, 511, dtype=np.uint64))
    cache = {"none": None, "capacity0": oracle.Cache(H, 0), "empty": oracle.Cache(H, 64)}[cache_kind]
    got = oracle.hs_step_cached(model, cache, ids, prev, h_in, query)
    U_, rep, inverse = oracle.dedup(ids)
    ref = oracle.hs_step(model, prev[rep], h_in[rep], query, row_of_query=inverse)
    assert got["n_unique"] == U_ and np.array_equal(got["rep"], rep) and np.array_equal(got["inverse"], inverse)
    assert np.array_equal(got["h_out"], ref["h_out"]) and np.array_equal(got["score"], ref["logprob"])
    stored = {"none": 0, "capacity0": 0, "empty": U_}[cache_kind]
    assert got["stats"] == (U_, 0, U_, stored)


def test_cached_step_answers_a_known_history_from_the_store_and_subtracts_the_base_score():
    """Second step: half of the ids are known and arrive with DIFFERENT prev / h_in (the stored context
    must win), the others are new; a bounded cache keeps what fits, in order of first appearance."""
    rng = np.random.default_rng(6)
    V, H, N, K = 47, 7, 24, 3
    model, ids1, prev1, h1, q1 = cached_case(rng, V, H, N, K, np.arange(100, 108, dtype=np.uint64))
    cache = oracle.Cache(H, 10)
    first = oracle.hs_step_cached(model, cache, ids1, prev1, h1, q1)
    known = {int(ids1[first["rep"][u]]): first["h_out"][u] for u in range(first["n_unique"])}
    assert first["stats"] == (len(known), 0, len(known), len(known))
    _, ids2, prev2, h2, q2 = cached_case(rng, V, H, N, K, np.arange(104, 116, dtype=np.uint64))
    base = rng.normal(0, 1, (N, K)).astype(np.float32)
    second = oracle.hs_step_cached(model, cache, ids2, prev2, h2, q2, base_score=base)
    hits = misses = 0
    entries = len(known)
    for u in range(second["n_unique"]):
        n = int(second["rep"][u])
        key = int(ids2[n])
        if key in known:
            hits += 1
            assert np.array_equal(second["h_out"][u], known[key])          # the stored bits, not a recomputation
        else:
            misses += 1
            expect = scipy.special.expit(model["U"][prev2[n]].astype(np.float64)
                                         + model["W"].astype(np.float64) @ h2[n].astype(np.float64))
            assert np.allclose(second["h_out"][u], expect, rtol=0, atol=1e-14)
            entries = min(entries + 1, 10)
    assert hits > 0 and misses > 0
    assert second["stats"] == (hits + misses, hits, misses, entries)
    for n in range(N):
        h = second["h_out"][second["inverse"][n]]
        for k in range(K):
            want = numpy_path_logp(model, h, int(q2[n, k])) - float(base[n, k])
            assert abs(second["score"][n, k] - want) <= 1e-12
    # every history the cache kept answers a third step without being computed
    third = oracle.hs_step_cached(model, cache, ids2, prev2, h2, q2)
    assert third["stats"][1] >= hits and third["stats"][3] == entries
    assert third["stats"][1] + third["stats"][2] == third["stats"][0]


def test_cached_step_still_gives_a_distribution_over_the_words():
    rng = np.random.default_rng(8)
    V, H = 23, 5
    model, ids, prev, h_in, _ = cached_case(rng, V, H, 6, 1, np.arange(3, dtype=np.uint64))
    query = np.tile(np.arange(V, dtype=np.int32), (6, 1))
    cache = oracle.Cache(H, 2)
    for _ in range(2):                                                       # computed, then (partly) from the store
        got = oracle.hs_step_cached(model, cache, ids, prev, h_in, query)
        assert np.allclose(np.exp(got["score"]).sum(axis=1), 1.0, rtol=0, atol=1e-12)
