"""The step entry points only launch kernels on the caller's stream, so a serving loop may
record them into a HIP graph.  Replays (with eager work and synchronisations in between)
must give exactly what the eager call gives on the same inputs."""
import numpy as np
import pytest
import torch

import paper_2007_11794_amd as rn
from workloads import round_to_bf16

from harness import DEV, keys_tensor, load_model

pytestmark = pytest.mark.gpu


def make_inputs(rng, V, H, N, K, pool):
    ids = rng.choice(pool, size=N).astype(np.uint64)
    prev = rng.integers(0, V, N).astype(np.int32)
    h_in = rng.uniform(0, 1, (N, H)).astype(np.float32)
    first = {}
    for n in range(N):
        f = first.setdefault(int(ids[n]), n)
        prev[n], h_in[n] = prev[f], h_in[f]
    return ids, prev, h_in, rng.integers(0, V, (N, K)).astype(np.int32)


@pytest.mark.parametrize("with_cache", [False, True])
def test_graph_replays_equal_eager(with_cache):
    rng = np.random.default_rng(21)
    V, H, N, K = 6000, 256, 500, 6
    model = {k: round_to_bf16(rng.normal(0, 0.05, s).astype(np.float32))
             for k, s in (("U", (V, H)), ("W", (H, H)), ("O", (H, V)))}
    model["bias"] = None
    m = load_model(model, "bf16", N)
    cache_g = rn.rnnlm_cache_create(m, 4000) if with_cache else None
    cache_e = rn.rnnlm_cache_create(m, 4000) if with_cache else None
    pool = np.arange(1, 300, dtype=np.uint64)

    def buffers():
        return dict(ids=torch.zeros(N, dtype=torch.int64, device=DEV), prev=torch.zeros(N, dtype=torch.int32, device=DEV),
                    h_in=torch.zeros((N, H), device=DEV), query=torch.zeros((N, K), dtype=torch.int32, device=DEV),
                    rep=torch.zeros(N, dtype=torch.int32, device=DEV), inv=torch.zeros(N, dtype=torch.int32, device=DEV),
                    nu=torch.zeros(1, dtype=torch.int32, device=DEV), h_out=torch.zeros((N, H), device=DEV),
                    score=torch.zeros((N, K), device=DEV),
                    ws=torch.empty(max(rn.rnnlm_dedup_workspace_bytes(N), 16), dtype=torch.uint8, device=DEV))

    def call(b, cache):
        rn.rnnlm_step_cached(m, cache, b["ids"], b["prev"], b["h_in"], b["query"], b["rep"], b["inv"], b["nu"],
                             b["h_out"], b["score"], b["ws"])

    def fill(b, x):
        ids, prev, h_in, query = x
        b["ids"].copy_(keys_tensor(ids)); b["prev"].copy_(torch.from_numpy(prev)); b["h_in"].copy_(torch.from_numpy(h_in))
        b["query"].copy_(torch.from_numpy(query))

    bg, be = buffers(), buffers()
    x0 = make_inputs(rng, V, H, N, K, pool)
    fill(bg, x0)
    call(bg, cache_g)                                   # warm-up outside the capture
    torch.cuda.synchronize()
    if with_cache:
        cache_g.reset()
        torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        call(bg, cache_g)                               # recorded, not run
    torch.cuda.synchronize()
    for it in range(4):
        x = make_inputs(rng, V, H, N, K, pool)
        fill(bg, x); fill(be, x)
        graph.replay()
        call(be, cache_e)                               # eager, its own cache with the same history
        torch.cuda.synchronize()
        for name in ("inv", "nu", "score"):
            assert torch.equal(bg[name], be[name]), (it, name)
        U = int(be["nu"].item())                        # rows beyond U are left untouched by contract
        assert torch.equal(bg["rep"][:U], be["rep"][:U]), it
        assert torch.equal(bg["h_out"][:U], be["h_out"][:U]), it
        assert torch.isfinite(bg["score"]).all()
    if with_cache:
        assert cache_g.stats() == cache_e.stats() and cache_g.stats()["hits"] > 0
        cache_g.close(); cache_e.close()
    assert m.last_error() == 0
    m.close()
