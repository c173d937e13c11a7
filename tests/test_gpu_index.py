"""GPU tests of the device-side IndexTable (rnnlm_index_*): contexts given by value get the
indices the oracle's table gives them, bit for bit, and come back unchanged."""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_11794_amd as rn
from workloads import round_to_bf16

from harness import DEV, CachedStepper, load_model

pytestmark = pytest.mark.gpu


def gpu_intern(t, word, h):
    N = len(word)
    w_t = torch.from_numpy(np.ascontiguousarray(word, np.int32)).to(DEV)
    h_t = torch.from_numpy(np.ascontiguousarray(h, np.float32)).to(DEV)
    idx = torch.full((N,), -7, dtype=torch.int32, device=DEV)
    rn.rnnlm_index_intern(t, w_t, h_t, idx)
    torch.cuda.synchronize()
    return idx.cpu().numpy().view(np.uint32)


def gpu_fetch(t, index):
    N = len(index)
    i_t = torch.from_numpy(np.ascontiguousarray(index, np.uint32).view(np.int32)).to(DEV)
    w_t = torch.full((N,), -9, dtype=torch.int32, device=DEV)
    h_t = torch.full((N, t.H), 7.0, device=DEV)
    rn.rnnlm_index_fetch(t, i_t, w_t, h_t)
    torch.cuda.synchronize()
    return w_t.cpu().numpy(), h_t.cpu().numpy()


@pytest.mark.parametrize("H", [5, 64, 512, 1000])
@pytest.mark.parametrize("capacity", [0, 37, 50000])
def test_indices_match_the_oracle(H, capacity):
    rng = np.random.default_rng(H * 7 + capacity)
    pool_h = rng.uniform(0, 1, (300, H)).astype(np.float32)
    pool_h[1] = pool_h[0]; pool_h[1, -1] = np.nextafter(pool_h[0, -1], np.float32(2))   # last element, one ulp
    pool_h[2] = pool_h[0]; pool_h[2, 0] = np.nextafter(pool_h[0, 0], np.float32(2))     # first element
    pool_h[3] = 0.0
    pool_h[4] = 0.0; pool_h[4, H // 2] = -0.0                                           # -0.0 is not +0.0
    pool_w = np.array([0, 1, 2, 3, 65535, 199999])
    t = rn.rnnlm_index_create(H, capacity, 6000)
    o = oracle.IndexTable(H, capacity)
    for call, N in enumerate([0, 1, 700, 4096, 5000, 333]):
        if H == 1000 and N > 1000:
            N = 900                                  # keeps the oracle's quadratic scan short
        word = pool_w[rng.integers(0, len(pool_w), N)].astype(np.int32)
        sel = rng.integers(0, 40 * (call + 1), N) % len(pool_h)
        h = pool_h[sel]
        got = gpu_intern(t, word, h)
        want = o.intern(word, h)
        assert np.array_equal(got, want), (H, capacity, call)
    s = t.stats()
    assert s["collisions"] == 0 and s["bad_fetch"] == 0
    assert {k: s[k] for k in ("entries", "lookups", "found", "unstored")} == o.stats()
    # forward direction
    held = s["entries"]
    if held:
        idx = rng.integers(0, held, 500).astype(np.uint32)
        w_g, h_g = gpu_fetch(t, idx)
        w_o, h_o = o.fetch(idx)
        assert np.array_equal(w_g, w_o) and np.array_equal(h_g.view(np.uint32), h_o.view(np.uint32))
    w_b, h_b = gpu_fetch(t, np.array([held, 0xFFFFFFFF, 0xFFFFFFFE], np.uint32))
    assert np.all(w_b == -1) and np.all(np.isnan(h_b))
    assert t.stats()["bad_fetch"] == 3
    t.reset()
    assert t.stats() == dict(entries=0, lookups=0, found=0, unstored=0, collisions=0, bad_fetch=0)
    t.close()


def test_search_by_indices_only():
    """Three steps of a search that keeps nothing but context indices: contexts are fetched from
    the table, scored through the cache with the packed (context, small-LM) ids, and the contexts
    that follow (queried word, updated hidden vector) are turned into indices again."""
    rng = np.random.default_rng(9)
    V, H, K, N = 4000, 128, 3, 256
    model = {k: round_to_bf16(rng.normal(0, 0.05, s).astype(np.float32))
             for k, s in (("U", (V, H)), ("W", (H, H)), ("O", (H, V)))}
    model["bias"] = None
    m = load_model(model, "bf16", N * K)
    table = rn.rnnlm_index_create(H, 100000, N * K)
    cache = rn.rnnlm_cache_create(m, 100000)
    o_table, o_cache = oracle.IndexTable(H, 100000), oracle.Cache(H, 100000)
    # utterance start: every hypothesis in the context (sentence-start word 0, zero vector)
    ctx_g = gpu_intern(table, np.zeros(1, np.int32), np.zeros((1, H), np.float32)).repeat(8)
    ctx_o = o_table.intern(np.zeros(1, np.int32), np.zeros((1, H), np.float32)).repeat(8)
    for step in range(3):
        n = len(ctx_g)
        assert np.array_equal(ctx_g, ctx_o), step
        small = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32)
        query = rng.integers(0, 40, (n, K)).astype(np.int32)        # few words: contexts meet again
        # device side
        prev_g, h_g = gpu_fetch(table, ctx_g)
        ids_t = torch.zeros(n, dtype=torch.int64, device=DEV)
        rn.rnnlm_pack_ids(torch.from_numpy(ctx_g.view(np.int32)).to(DEV), torch.from_numpy(small.view(np.int32)).to(DEV), ids_t)
        torch.cuda.synchronize()
        ids = ids_t.cpu().numpy().view(np.uint64)
        # the RNNLM result depends on the context index only: group on it (high half)
        out = CachedStepper(m, cache, n, K).step(ids >> np.uint64(32), prev_g, h_g, query)
        # oracle side
        prev_o, h_o = o_table.fetch(ctx_o)
        ref = oracle.step_cached(model, o_cache, oracle.pack_ids(ctx_o, small) >> np.uint64(32), prev_o, h_o, query)
        assert out["stats"] == ref["stats"], step
        assert np.max(np.abs(out["score"] - ref["score"])) <= 2e-3
        # the contexts that follow: (queried word, updated hidden vector of the history)
        next_w = query.reshape(-1)
        next_h_g = out["h_out"][out["inverse"]].repeat(K, axis=0)
        next_h_o = ref["h_out"][ref["inverse"]].astype(np.float32).repeat(K, axis=0)
        ctx_g = gpu_intern(table, next_w, next_h_g)[: 256]
        ctx_o = o_table.intern(next_w, next_h_o)[: 256]
    s = table.stats()
    assert s["collisions"] == 0
    assert {k: s[k] for k in ("entries", "lookups", "found", "unstored")} == o_table.stats()
    assert s["lookups"] < 1 + 8 * K + 2 * 256 * K          # equal contexts of one call were merged
    for x in (table, cache, m):
        x.close()
