"""GPU tests of the hierarchical output layer (rnnlm_hs_load / rnnlm_hs_step) against the oracle,
through the C ABI.  Bars as for the full softmax: bf16 |dlogprob| <= 2e-3, |dh| <= 1e-3; fp32
1e-5."""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_11794_amd as rn
from workloads import CONFIGS, bf16_bits, bounded_zipf_ids, round_to_bf16

from harness import DEV

pytestmark = pytest.mark.gpu

TOL = {"f32": (1e-5, 1e-5), "bf16": (2e-3, 1e-3)}


def hs_model(rng, V, H, dtype, sigma, zipf_s=1.1):
    freq = np.arange(1, V + 1, dtype=np.float64) ** -zipf_s
    off, entry = oracle.huffman_build(freq)
    m = {"U": rng.normal(0, sigma, (V, H)).astype(np.float32), "W": rng.normal(0, sigma, (H, H)).astype(np.float32),
         "theta": rng.normal(0, 4 * sigma, (V - 1, H)).astype(np.float32), "path_off": off, "path_entry": entry}
    if dtype == "bf16":
        for k in ("U", "W", "theta"):
            m[k] = round_to_bf16(m[k])
    return m


def load(m, dtype, max_B):
    V, H = m["U"].shape
    if dtype == "bf16":
        return rn.rnnlm_hs_load(V, H, rn.RNNLM_BF16, bf16_bits(m["U"]), bf16_bits(m["W"]), bf16_bits(m["theta"]),
                                m["path_off"], m["path_entry"], max_B)
    return rn.rnnlm_hs_load(V, H, rn.RNNLM_F32, m["U"], m["W"], m["theta"], m["path_off"], m["path_entry"], max_B)


def gpu_hs_step(mod, prev, h_in, query, row_of_query=None, base=None):
    t = lambda a, d: None if a is None else torch.from_numpy(np.ascontiguousarray(a, d)).to(DEV)
    prev_t, h_t, q_t = t(prev, np.int32), t(h_in, np.float32), t(query, np.int32)
    B, (N, K) = prev_t.shape[0], q_t.shape
    h_out = torch.full((B, mod.H), float("nan"), device=DEV)
    lp = torch.full((N, K), float("nan"), device=DEV)
    rn.rnnlm_hs_step(mod, prev_t, h_t, q_t, h_out, lp, row_of_query=t(row_of_query, np.int32), base_score=t(base, np.float32))
    torch.cuda.synchronize()
    return h_out.cpu().numpy(), lp.cpu().numpy()


@pytest.mark.parametrize("dtype,V,H,B,K,N", [
    ("bf16", 5000, 512, 300, 8, 300),
    ("bf16", 4099, 160, 77, 5, 200),         # padded hidden size, fan-out through row_of_query
    ("bf16", 2, 64, 5, 2, 5),                # the smallest tree
    ("f32", 3001, 96, 64, 9, 64),
    ("f32", 20000, 256, 256, 16, 256),       # config 2's shape
    ("bf16", 3000, 250, 40, 12, 90),         # half a wave per node row (hidden size padded to 256)
    ("bf16", 3001, 128, 33, 32, 33),         # a quarter wave per node row, more than one batch of nodes
    ("f32", 2999, 128, 20, 40, 50),
])
def test_hs_step_matches_the_oracle(dtype, V, H, B, K, N):
    rng = np.random.default_rng(V + H)
    m = hs_model(rng, V, H, dtype, 0.05)
    mod = load(m, dtype, max(B, N))
    prev = rng.integers(0, V, B).astype(np.int32)
    h_in = rng.uniform(0, 1, (B, H)).astype(np.float32)
    query = bounded_zipf_ids(rng, V, 1.1, (N, K)).astype(np.int32) if V > 100 else rng.integers(0, V, (N, K)).astype(np.int32)
    query[0, 0] = V - 1                                         # a rare word: one of the longest paths
    roq = None if N == B else rng.integers(0, B, N).astype(np.int32)
    base = rng.normal(-5, 2, (N, K)).astype(np.float32)
    ref = oracle.hs_step(m, prev, h_in, query, row_of_query=roq)
    for use_base in (False, True):
        h, lp = gpu_hs_step(mod, prev, h_in, query, roq, base if use_base else None)
        want = ref["logprob"] - (base.astype(np.float64) if use_base else 0.0)
        dh, dlp = np.max(np.abs(h - ref["h_out"])), np.max(np.abs(lp - want))
        print("hs %s V=%d H=%d max|dh|=%.3g max|dlogprob|=%.3g longest path %d" %
              (dtype, V, H, dh, dlp, int(np.diff(m["path_off"]).max())), flush=True)
        assert dh <= TOL[dtype][1] and dlp <= TOL[dtype][0]
    assert mod.last_error() == 0
    mod.close()


def test_hs_bad_indices_and_wrong_entry_point():
    rng = np.random.default_rng(3)
    V, H, B, K = 300, 64, 6, 3
    m = hs_model(rng, V, H, "f32", 0.1)
    mod = load(m, "f32", 16)
    prev = rng.integers(0, V, B).astype(np.int32)
    h_in = rng.uniform(0, 1, (B, H)).astype(np.float32)
    query = rng.integers(0, V, (B, K)).astype(np.int32)
    query[1, 2] = V
    query[4, 0] = -1
    h, lp = gpu_hs_step(mod, prev, h_in, query)
    bad = np.zeros((B, K), bool); bad[1, 2] = bad[4, 0] = True
    assert np.all(np.isnan(lp[bad])) and np.all(np.isfinite(lp[~bad]))
    assert mod.last_error() == rn.FLAG_BAD_QUERY_WORD
    roq = np.array([0, 1, B, 2, -1, 3], np.int32)
    query = rng.integers(0, V, (B, K)).astype(np.int32)
    h, lp = gpu_hs_step(mod, prev, h_in, query, roq)
    assert np.all(np.isnan(lp[[2, 4]])) and np.all(np.isfinite(lp[[0, 1, 3, 5]]))
    assert mod.last_error() == rn.FLAG_BAD_ROW
    # a hierarchical model is refused by the full-softmax step
    with pytest.raises(rn.RnnlmError) as e:
        rn.rnnlm_step(mod, torch.zeros(B, dtype=torch.int32, device=DEV), torch.zeros((B, H), device=DEV),
                      torch.zeros((B, K), dtype=torch.int32, device=DEV), torch.zeros((B, H), device=DEV),
                      torch.zeros((B, K), device=DEV))
    assert e.value.status == -1
    # a tree that names a node beyond V-2 is refused at load
    bad_entry = m["path_entry"].copy(); bad_entry[5] = V - 1
    with pytest.raises(rn.RnnlmError):
        rn.rnnlm_hs_load(V, H, rn.RNNLM_F32, m["U"], m["W"], m["theta"], m["path_off"], bad_entry, 16)
    mod.close()


def test_hs_headline_shape_every_row():
    """V = 65536, H = 512, B = 1024, K = 32 (the headline workload's shape): every hidden row and
    every one of the 1024 x 32 log-probabilities against the oracle."""
    cfg = CONFIGS[3]
    rng = np.random.default_rng(cfg.seed)
    m = hs_model(rng, cfg.V, cfg.H, "bf16", cfg.sigma)
    mod = load(m, "bf16", cfg.B)
    prev = bounded_zipf_ids(rng, cfg.V, 1.1, cfg.B).astype(np.int32)
    h_in = (1.0 / (1.0 + np.exp(-rng.normal(0, 1, (cfg.B, cfg.H))))).astype(np.float32)
    query = bounded_zipf_ids(rng, cfg.V, 1.1, (cfg.B, cfg.K)).astype(np.int32)
    h, lp = gpu_hs_step(mod, prev, h_in, query)
    ref = oracle.hs_step(m, prev, h_in, query)
    dh, dlp = np.max(np.abs(h - ref["h_out"])), np.max(np.abs(lp - ref["logprob"]))
    print("hs headline shape: max|dh|=%.3g max|dlogprob|=%.3g mean path %.1f" %
          (dh, dlp, float(np.diff(m["path_off"])[query].mean())), flush=True)
    assert dh <= 1e-3 and dlp <= 2e-3 and np.all(np.isfinite(lp)) and np.all(lp < 0)
    assert mod.last_error() == 0
    mod.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_hs_million_words_few_rows(dtype):
    """The regime the paper runs the tree in (Section 5.1): about a million words, a hidden layer of
    100 units, and the few distinct histories a step of a well-cached search leaves.  V is odd on
    purpose; rare words sit 25 to 30 nodes deep, frequent ones a handful."""
    rng = np.random.default_rng(1234)
    V, H, K = 1000003, 100, 32
    m = hs_model(rng, V, H, dtype, 0.05)
    depth = np.diff(m["path_off"])
    assert depth.min() >= 1 and depth.max() >= 20
    mod = load(m, dtype, 64)
    for B in (1, 20, 64):
        prev = bounded_zipf_ids(rng, V, 1.1, B).astype(np.int32)
        h_in = rng.uniform(0, 1, (B, H)).astype(np.float32)
        query = bounded_zipf_ids(rng, V, 1.1, (B, K)).astype(np.int32)
        query[:, 0] = V - 1 - np.arange(B)                  # the rarest words: the longest paths
        query[:, 1] = np.arange(B)                          # the most frequent ones
        ref = oracle.hs_step(m, prev, h_in, query)
        h, lp = gpu_hs_step(mod, prev, h_in, query)
        dh, dlp = np.max(np.abs(h - ref["h_out"])), np.max(np.abs(lp - ref["logprob"]))
        print("hs V=%d H=%d %s B=%d: max|dh|=%.3g max|dlogprob|=%.3g deepest queried path %d" %
              (V, H, dtype, B, dh, dlp, int(depth[query].max())), flush=True)
        assert dh <= TOL[dtype][1] and dlp <= TOL[dtype][0]
    assert mod.last_error() == 0
    mod.close()


def hs_shapes():
    rng = np.random.default_rng(314)
    out = []
    for i in range(16):
        out.append((i, "bf16" if i % 2 else "f32", int(rng.choice([2, 3, 9, 33, 257, 1000, 4097])),
                    int(rng.choice([1, 3, 64, 65, 130, 256, 516, 700])), int(rng.choice([1, 2, 33, 64, 129, 300])),
                    int(rng.choice([1, 2, 7, 9, 17, 40]))))
    return out


@pytest.mark.parametrize("i,dtype,V,H,B,K", hs_shapes())
def test_hs_awkward_shapes(i, dtype, V, H, B, K):
    """Odd hidden sizes, trees of two or three words, single rows, many words per query, skewed and
    flat frequencies (deep and shallow trees)."""
    rng = np.random.default_rng(500 + i)
    m = hs_model(rng, V, H, dtype, 0.4 / np.sqrt(H), zipf_s=(0.0, 1.0, 2.0)[i % 3])
    N = B + int(rng.integers(0, B + 1))
    mod = load(m, dtype, N)
    prev = rng.integers(0, V, B).astype(np.int32)
    h_in = rng.uniform(0, 1, (B, H)).astype(np.float32)
    roq = np.concatenate([np.arange(B), rng.integers(0, B, N - B)]).astype(np.int32)
    query = rng.integers(0, V, (N, K)).astype(np.int32)
    query[0, 0] = V - 1
    ref = oracle.hs_step(m, prev, h_in, query, row_of_query=roq)
    h, lp = gpu_hs_step(mod, prev, h_in, query, roq)
    dh, dlp = np.max(np.abs(h - ref["h_out"])), np.max(np.abs(lp - ref["logprob"]))
    assert dh <= TOL[dtype][1] and dlp <= TOL[dtype][0], (i, dtype, V, H, B, K, dh, dlp, int(np.diff(m["path_off"]).max()))
    assert mod.last_error() == 0
    mod.close()


# ------------------------------------------------------------------------ the paper's whole RnnlmProb: cache + hierarchical layer
@pytest.mark.parametrize("dtype,V,H,K", [("bf16", 8200, 256, 5), ("bf16", 4099, 160, 2), ("f32", 3001, 96, 9),
                                         ("bf16", 5000, 100, 16)])
@pytest.mark.parametrize("capacity", [100000, 150, 0, None])
def test_hs_steps_through_the_cache_match_the_oracle(dtype, V, H, K, capacity):
    """Table 1 around the output layer of Section 2.1 (rnnlm_step_cached on a model loaded with
    rnnlm_hs_load; capacity None: rnnlm_step_dedup's case, nothing outlives the step).  Grouping and the
    hit / computed / stored counts bit-exact, values within the step's tolerances, and a history
    answered from the cache carries the hidden vector first computed, bit for bit."""
    from harness import CachedStepper
    rng = np.random.default_rng(V + H + (capacity or 7))
    m = hs_model(rng, V, H, dtype, 0.05)
    mod = load(m, dtype, 700)
    cache = rn.rnnlm_cache_create(mod, capacity) if capacity is not None else None
    ocache = oracle.Cache(H, capacity) if capacity is not None else None
    pool = (np.arange(400, dtype=np.uint64) << np.uint64(32)) | np.uint64(0x1234)
    pool[3] = np.uint64(0xFFFFFFFFFFFFFFFF)
    st = CachedStepper(mod, cache, 700, K)
    seen = {}
    for step, N in enumerate([300, 700, 64, 1, 513]):
        ids = rng.choice(pool, size=N).astype(np.uint64)
        prev = rng.integers(0, V, N).astype(np.int32)
        h_in = rng.uniform(0, 1, (N, H)).astype(np.float32)
        first = {}
        for n in range(N):                       # rows of one id agree within a step
            f = first.setdefault(int(ids[n]), n)
            prev[n], h_in[n] = prev[f], h_in[f]
        query = rng.integers(0, V, (N, K)).astype(np.int32)
        base = rng.normal(-6, 2, (N, K)).astype(np.float32) if step % 2 == 0 else None
        out = st.step(ids, prev, h_in, query, base)
        ref = oracle.hs_step_cached(m, ocache, ids, prev, h_in, query, base_score=base)
        what = "hs cached %s V=%d H=%d K=%d cap=%s step %d" % (dtype, V, H, K, capacity, step)
        assert out["n_unique"] == ref["n_unique"], what
        assert np.array_equal(out["rep"], ref["rep"]) and np.array_equal(out["inverse"], ref["inverse"]), what
        if capacity is not None:
            assert out["stats"] == ref["stats"], (what, out["stats"], ref["stats"])
        assert np.all(np.isnan(out["h_out_rest"])), what
        dh = np.max(np.abs(out["h_out"].astype(np.float64) - ref["h_out"]))
        ds = np.max(np.abs(out["score"].astype(np.float64) - ref["score"]))
        print("%s stats=%s max|dh|=%.3g max|dscore|=%.3g" % (what, out["stats"], dh, ds), flush=True)
        assert dh <= TOL[dtype][1] and ds <= TOL[dtype][0], (what, dh, ds)
        if capacity == 100000:                   # everything is kept: a known history returns the same bits
            for u in range(out["n_unique"]):
                key = int(ids[out["rep"][u]])
                if key in seen:
                    assert np.array_equal(out["h_out"][u], seen[key]), what
                else:
                    seen[key] = out["h_out"][u].copy()
    if cache is not None:
        assert cache.stats() == ocache.stats()
        cache.close()
    assert mod.last_error() == 0
    mod.close()


def test_hs_many_raw_queries_through_the_cache():
    """More raw queries than one workgroup groups (grid-wide grouping and lookup), a cache that fills up."""
    from harness import CachedStepper
    rng = np.random.default_rng(99)
    V, H, K = 2000, 64, 4
    m = hs_model(rng, V, H, "bf16", 0.1)
    mod = load(m, "bf16", 9000)
    pool = rng.integers(0, 2 ** 64, 7000, dtype=np.uint64)
    cache, ocache = rn.rnnlm_cache_create(mod, 3000), oracle.Cache(H, 3000)
    st = CachedStepper(mod, cache, 9000, K)
    for step, N in enumerate([6000, 9000, 4097]):
        ids = rng.choice(pool, size=N).astype(np.uint64)
        prev = rng.integers(0, V, N).astype(np.int32)
        h_in = rng.uniform(0, 1, (N, H)).astype(np.float32)
        first = {}
        for n in range(N):
            f = first.setdefault(int(ids[n]), n)
            prev[n], h_in[n] = prev[f], h_in[f]
        query = rng.integers(0, V, (N, K)).astype(np.int32)
        out = st.step(ids, prev, h_in, query, None)
        ref = oracle.hs_step_cached(m, ocache, ids, prev, h_in, query)
        assert out["n_unique"] == ref["n_unique"] and out["stats"] == ref["stats"], (step, out["stats"], ref["stats"])
        assert np.array_equal(out["rep"], ref["rep"]) and np.array_equal(out["inverse"], ref["inverse"])
        dh = np.max(np.abs(out["h_out"].astype(np.float64) - ref["h_out"]))
        ds = np.max(np.abs(out["score"].astype(np.float64) - ref["score"]))
        print("hs cached N=%d stats=%s max|dh|=%.3g max|dscore|=%.3g" % (N, out["stats"], dh, ds), flush=True)
        assert dh <= TOL["bf16"][1] and ds <= TOL["bf16"][0]
    assert cache.stats() == ocache.stats() and mod.last_error() == 0
    cache.close()
    mod.close()
