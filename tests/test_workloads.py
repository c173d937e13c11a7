"""The input generators: distributions, bf16 exactness, decode-trace structure."""
import numpy as np

from workloads import (CONFIGS, DecodeTrace, bf16_bits, bounded_zipf_ids, make_model,
                       make_step_inputs, pack_history_id, round_to_bf16)


def test_round_to_bf16_is_nearest_even_and_idempotent():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -7, 1.0 + 3 * 2 ** -8, -0.03, 3.14159], np.float32)
    r = round_to_bf16(x)
    assert r[0] == 1.0
    assert r[1] == 1.0                      # tie -> even mantissa
    assert r[2] == np.float32(1.0 + 2 ** -7)
    assert r[3] == np.float32(1.0 + 2 ** -6)  # tie -> even
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(round_to_bf16(r), r)
    bits = bf16_bits(r)
    assert bits.dtype == np.uint16
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back, r)


def test_bounded_zipf_matches_pmf():
    rng = np.random.default_rng(0)
    V, s = 50, 1.0
    ids = bounded_zipf_ids(rng, V, s, 200000)
    assert ids.min() >= 0 and ids.max() < V
    pmf = np.arange(1, V + 1) ** (-s)
    pmf /= pmf.sum()
    freq = np.bincount(ids, minlength=V) / ids.size
    assert np.max(np.abs(freq - pmf)) < 5e-3


def test_configs_shapes_and_seeding():
    cfg = CONFIGS[3].scaled(V=512, H=64, B=16)
    m = make_model(cfg)
    assert m["U"].shape == (512, 64) and m["W"].shape == (64, 64) and m["O"].shape == (64, 512)
    bf16_bits(m["O"])                       # raises if not exact
    m2 = make_model(cfg)
    assert np.array_equal(m["U"], m2["U"])
    x = make_step_inputs(cfg, np.random.default_rng(1))
    assert x["prev"].shape == (16,) and x["h_in"].shape == (16, 64) and x["query"].shape == (16, 32)
    assert len(set(x["keys"].tolist())) == 16
    assert 0 < x["h_in"].min() and x["h_in"].max() < 1
    x1 = make_step_inputs(CONFIGS[1], np.random.default_rng(1))
    assert len(set(x1["prev"].tolist())) == CONFIGS[1].B


def test_pack_history_id_halves():
    k = pack_history_id(np.array([1, 2]), np.array([3, 0xFFFFFFFF]))
    assert k.dtype == np.uint64
    assert int(k[0]) == (1 << 32) | 3 and int(k[1]) == (2 << 32) | 0xFFFFFFFF


def test_decode_trace_structure():
    cfg = CONFIGS[4].scaled(V=300, H=8, N=200, K=2, steps=3)
    tr = DecodeTrace(cfg)
    x = tr.first()
    U0 = round(0.3 * 200)
    assert x["keys"].shape == (200,) and len(set(x["keys"].tolist())) == U0
    # rows with the same id hold the same history
    for n in range(200):
        same = np.flatnonzero(x["keys"] == x["keys"][n])
        assert np.all(x["prev"][same] == x["prev"][n])
        assert np.all(x["h_in"][same] == x["h_in"][n])
    # next step: stand-in "updated hidden" = a recognisable function of the row index
    uniq_keys, first = np.unique(x["keys"], return_index=True)
    order = np.argsort(first)
    inverse = np.empty(200, np.int64)
    for u, k in enumerate(uniq_keys[order]):
        inverse[x["keys"] == k] = u
    h_out = np.tile(np.arange(U0, dtype=np.float32)[:, None], (1, 8)) + 100
    y = tr.next(x, h_out, inverse)
    assert len(set(y["keys"].tolist())) == U0
    old = set(x["keys"].tolist())
    n_carried = sum(k in old for k in set(y["keys"].tolist()))
    assert n_carried == int(y["carried"].sum()) and 0 < n_carried < U0
    for n in range(200):
        if int(y["keys"][n]) in old:       # carried: identical history as before
            m = np.flatnonzero(x["keys"] == y["keys"][n])[0]
            assert y["prev"][n] == x["prev"][m] and np.array_equal(y["h_in"][n], x["h_in"][m])
        else:                              # grown from some row's updated hidden vector
            assert y["h_in"][n, 0] >= 100
