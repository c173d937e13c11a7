"""Pins for the oracle's IndexTable / inverse IndexTable (Section 3.2; Table 1 steps 5, 7-12).

Expected values come from a Python dict keyed by (word, raw bytes of the hidden vector) that
numbers contexts in order of first appearance, from round trips, and from hand-made cases
that differ in exactly one bit."""
import numpy as np
import pytest

import oracle


def dict_intern(state, word, h, capacity):
    out = []
    for w, row in zip(word.tolist(), h):
        key = (w, row.tobytes())
        if key not in state and len(state) < capacity:
            state[key] = len(state)
        out.append(state.get(key, 0xFFFFFFFF))
    return np.array(out, dtype=np.uint32)


def draw(rng, N, H, pool_w, pool_h):
    word = pool_w[rng.integers(0, len(pool_w), N)].astype(np.int32)
    h = pool_h[rng.integers(0, len(pool_h), N)].astype(np.float32)
    return word, h


@pytest.mark.parametrize("capacity", [0, 1, 13, 10000])
def test_against_python_dict_over_several_calls(capacity):
    rng = np.random.default_rng(capacity + 3)
    H = 7
    pool_w = np.array([0, 1, 2, 65535, 7])
    pool_h = rng.uniform(0, 1, (9, H)).astype(np.float32)
    t = oracle.IndexTable(H, capacity)
    state = {}
    lookups = found = unstored = 0
    for call in range(6):
        N = int(rng.integers(0, 50))
        word, h = draw(rng, N, H, pool_w, pool_h)
        keys = list(dict.fromkeys((w, r.tobytes()) for w, r in zip(word.tolist(), h)))
        lookups += len(keys)
        found += sum(k in state for k in keys)
        unstored += max(0, sum(k not in state for k in keys) - (capacity - len(state)))
        want = dict_intern(state, word, h, capacity)
        got = t.intern(word, h)
        assert np.array_equal(got, want), call
    assert t.stats() == dict(entries=len(state), lookups=lookups, found=found, unstored=unstored)
    assert t.stats()["entries"] <= capacity


def test_round_trip_and_stability():
    rng = np.random.default_rng(5)
    H, N = 33, 200
    word = rng.integers(0, 50, N).astype(np.int32)
    h = rng.normal(0, 1, (N, H)).astype(np.float32)
    h[50:100] = h[0:50]                                    # repeated vectors, new or repeated words
    word[50:75] = word[0:25]
    t = oracle.IndexTable(H, 1000)
    a = t.intern(word, h)
    assert np.array_equal(a[50:75], a[0:25])
    assert np.array_equal(np.sort(np.unique(a)), np.arange(a.max() + 1))      # 0..count-1, no holes
    first = {}
    for n, i in enumerate(a.tolist()):
        first.setdefault(i, n)
    assert list(first.values()) == sorted(first.values())   # numbered in order of first appearance
    w2, h2 = t.fetch(a)
    assert np.array_equal(w2, word) and np.array_equal(h2.view(np.uint32), h.view(np.uint32))
    perm = rng.permutation(N)
    assert np.array_equal(t.intern(word[perm], h[perm]), a[perm])             # stable afterwards
    assert t.stats()["entries"] == len(first)
    t.reset()
    assert t.stats() == dict(entries=0, lookups=0, found=0, unstored=0)
    assert t.intern(word[perm][:1], h[perm][:1])[0] == 0


def test_every_bit_counts():
    H = 5
    base = np.array([0.25, 0.5, 0.0, 1.0, 0.75], dtype=np.float32)
    rows, words = [base.copy()], [3]
    for j in range(H):                                     # one ulp in each position
        r = base.copy()
        r[j] = np.nextafter(r[j], np.float32(2.0))
        rows.append(r); words.append(3)
    r = base.copy(); r[2] = -0.0                           # -0.0 is not +0.0
    rows.append(r); words.append(3)
    rows.append(base.copy()); words.append(4)              # same vector, other word
    rows.append(base.copy()); words.append(3)              # the very first context again
    t = oracle.IndexTable(H, 100)
    got = t.intern(np.array(words, np.int32), np.array(rows, np.float32))
    assert got.tolist() == list(range(H + 3)) + [0]
    with pytest.raises(ValueError):
        t.fetch(np.array([H + 3], np.uint32))
