"""Parity of the HIP path with the CPU oracle, through the C ABI, on the seeded workloads.

Tolerances (written here, from the target statement): grouping indices bit-exact; fp32
models |dlogprob| <= 1e-5 and |dh| <= 1e-5; bf16 models (fp32-accumulated bf16 MFMA)
|dlogprob| <= 2e-3 and |dh| <= 1e-3.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_11794_amd as rn
from workloads import CONFIGS, DecodeTrace, make_model, make_step_inputs

from harness import gpu_dedup, gpu_step, gpu_step_dedup, load_model

pytestmark = pytest.mark.gpu

TOL = {"f32": (1e-5, 1e-5), "bf16": (2e-3, 1e-3)}      # (logprob, h)


def check(gpu_h, gpu_lp, ref, dtype, what=""):
    tol_lp, tol_h = TOL[dtype]
    dh = np.max(np.abs(gpu_h.astype(np.float64) - ref["h_out"])) if gpu_h.size else 0.0
    dlp = np.max(np.abs(gpu_lp.astype(np.float64) - ref["logprob"])) if gpu_lp.size else 0.0
    print("%s max|dh|=%.3g max|dlogprob|=%.3g" % (what, dh, dlp), flush=True)
    assert np.all(np.isfinite(gpu_h)) and np.all(np.isfinite(gpu_lp))
    assert dh <= tol_h, (what, dh)
    assert dlp <= tol_lp, (what, dlp)
    return dh, dlp


# ------------------------------------------------------------------------ config 1: tiny, fp32
def test_config1_tiny_full():
    cfg = CONFIGS[1]
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed))
    m = load_model(model, cfg.dtype, cfg.B)
    for lse_mode in (0, 1):
        m.set_option(rn.OPT_LSE_MODE, lse_mode)
        h, lp = gpu_step(m, x["prev"], x["h_in"], x["query"])
        check(h, lp, oracle.step(model, x["prev"], x["h_in"], x["query"]), "f32", "cfg1 lse_mode=%d" % lse_mode)
    assert m.last_error() == 0
    m.close()


# ------------------------------------------------------------------------ config 2: WSJ-sized, fp32, chained
def test_config2_chained_steps_full():
    cfg = CONFIGS[2]
    model = make_model(cfg)
    rng = np.random.default_rng(cfg.seed)
    m = load_model(model, cfg.dtype, cfg.B)
    x = make_step_inputs(cfg, rng)
    h_gpu = h_ref = x["h_in"]
    for step in range(cfg.steps):
        if step:
            x = make_step_inputs(cfg, rng)           # fresh prev/query draws every step
        ref = oracle.step(model, x["prev"], h_ref, x["query"])
        # (a) per-step error: both sides start from the oracle's state
        h1, lp1 = gpu_step(m, x["prev"], h_ref, x["query"])
        check(h1, lp1, ref, "f32", "cfg2 step %d (same state)" % step)
        # (b) accumulated error: the GPU keeps feeding on its own h_out
        h2, lp2 = gpu_step(m, x["prev"], h_gpu, x["query"])
        check(h2, lp2, ref, "f32", "cfg2 step %d (own state)" % step)
        h_gpu = h2
        h_ref = ref["h_out"].astype(np.float32)
    assert m.last_error() == 0
    m.close()


# ------------------------------------------------------------------------ bf16: reduced sizes, element by element
@pytest.mark.parametrize("V,H,B,K", [
    (5000, 512, 300, 8),      # several row groups and word tiles, ragged tails in both
    (777, 256, 130, 5),       # staged kernel at Hp = 256
    (1000, 100, 70, 3),       # the paper's hidden size: H not a multiple of anything useful
    (300, 64, 33, 2),
    (2000, 1024, 200, 4),     # hidden size beyond the staged kernel: tiled kernel (128-row tiles) by default
    (1500, 640, 300, 4),      # tiled kernel with 256-row tiles, hidden size not a power of two
    (2600, 640, 250, 3),      # tiled kernel, 128 words x 256 rows per workgroup with three stages
    (4000, 512, 29, 4),       # few rows: the weight-streaming kernel by default (one row block)
    (2100, 320, 64, 3),       # two row blocks in the streaming kernel, five groups per word block
    (900, 1024, 50, 2),       # the longest reduction the streaming kernel takes two row blocks of
    (3000, 256, 127, 2),      # four row blocks (on request only)
])
@pytest.mark.parametrize("kernel", [1, 2, 3, 5, 6])
@pytest.mark.parametrize("lse_mode", [1, 2])
def test_bf16_reduced_elementwise(V, H, B, K, kernel, lse_mode):
    cfg = CONFIGS[3].scaled(V=V, H=H, B=B, K=K)
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed + V))
    m = load_model(model, "bf16", B)
    m.set_option(rn.OPT_LSE_MODE, lse_mode)
    if kernel == 2 and max(128, -(-H // 64) * 64) not in (128, 256, 512):   # no staged kernel for this hidden size
        with pytest.raises(rn.RnnlmError):
            m.set_option(rn.OPT_OUTPROJ_KERNEL, kernel)
        kernel = 0                      # automatic choice instead (the tiled kernel at this size)
    # kernel 5 (weight streaming) serves up to 128 rows at these hidden sizes and hands larger
    # batches to the automatic choice
    m.set_option(rn.OPT_OUTPROJ_KERNEL, kernel)
    h, lp = gpu_step(m, x["prev"], x["h_in"], x["query"])
    check(h, lp, oracle.step(model, x["prev"], x["h_in"], x["query"]), "bf16",
          "bf16 V=%d H=%d B=%d kernel=%d lse=%d" % (V, H, B, kernel, lse_mode))
    assert m.last_error() == 0
    m.close()


@pytest.mark.parametrize("V,H,B,K", [(3000, 200, 150, 6), (1000, 64, 8, 4),
                                     (2500, 512, 61, 3),      # few rows: weight streaming, two launches of 32 rows
                                     (1200, 256, 64, 2),      # one launch, two row blocks
                                     (700, 768, 17, 2),       # the longest reduction whose three terms fit in LDS
                                     (900, 100, 97, 2)])      # on request only: four row blocks
def test_f32_reduced_elementwise_both_lse_modes(V, H, B, K):
    cfg = CONFIGS[2].scaled(V=V, H=H, B=B, K=K)
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed + V))
    m = load_model(model, "f32", B)
    ref = oracle.step(model, x["prev"], x["h_in"], x["query"])
    # plain FMA, LDS-tiled fp32-MFMA, bf16 three-term split, weight streaming (where it applies), automatic
    for kernel in (1, 3, 4, 5, 0):
        m.set_option(rn.OPT_OUTPROJ_KERNEL, kernel)
        for lse_mode in (1, 2):
            m.set_option(rn.OPT_LSE_MODE, lse_mode)
            h, lp = gpu_step(m, x["prev"], x["h_in"], x["query"])
            check(h, lp, ref, "f32", "f32 V=%d kernel=%d lse=%d" % (V, kernel, lse_mode))
    m.close()


# ------------------------------------------------------------------------ config 3: headline, full size, every row
def test_config3_headline_full_size_every_row():
    """All 1024 rows and all 1024 x 32 log-probabilities against the oracle, in the launch
    configuration bench.py times (automatic kernel choice) and with the plain kernel."""
    cfg = CONFIGS[3]
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed))
    m = load_model(model, cfg.dtype, cfg.B)
    ref = oracle.step(model, x["prev"], x["h_in"], x["query"])
    outs = {}
    for kernel in (0, 1):
        m.set_option(rn.OPT_OUTPROJ_KERNEL, kernel)
        h, lp = gpu_step(m, x["prev"], x["h_in"], x["query"])
        check(h, lp, ref, cfg.dtype, "cfg3 kernel=%d (all %d rows)" % (kernel, cfg.B))
        outs[kernel] = (h, lp)
    # extra, not the check: the two kernels share the hidden update, and their sums differ by rounding only
    assert np.array_equal(outs[0][0], outs[1][0])
    assert np.max(np.abs(outs[0][1] - outs[1][1])) <= 1e-4
    assert np.all(outs[0][1] < 0)
    assert m.last_error() == 0
    m.close()


def test_config3_model_few_rows_full_vocabulary():
    """The headline model with the few distinct histories a well-cached search leaves per step
    (Section 5.2): every row against the oracle, in the configuration the library picks by itself
    (the weight-streaming kernel), and against the plain kernel."""
    cfg = CONFIGS[3]
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed))
    m = load_model(model, cfg.dtype, 64)
    for B in (1, 7, 32, 33, 64):
        prev, h_in, query = x["prev"][:B], x["h_in"][:B], x["query"][:B]
        ref = oracle.step(model, prev, h_in, query)
        m.set_option(rn.OPT_OUTPROJ_KERNEL, 0)
        h, lp = gpu_step(m, prev, h_in, query)
        check(h, lp, ref, "bf16", "cfg3 model, %d rows" % B)
        m.set_option(rn.OPT_OUTPROJ_KERNEL, 1)
        h1, lp1 = gpu_step(m, prev, h_in, query)
        assert np.array_equal(h1, h) and np.max(np.abs(lp1 - lp)) <= 1e-4
    assert m.last_error() == 0
    m.close()


@pytest.mark.parametrize("V,H,N,distinct", [(5000, 512, 400, 20), (3000, 256, 300, 50), (2000, 128, 200, 64),
                                            (2000, 512, 260, 65), (40000, 512, 1024, 7),
                                            (66000, 640, 300, 20),      # tiled kernel (256 x 256 tiles): one row group, 256 splits
                                            (9000, 640, 300, 20),       # tiled kernel, fewer word tiles than workgroups
                                            (12000, 1216, 300, 30),     # tiled kernel streams one row block (all its LDS holds)
                                            (12000, 1216, 300, 40),     # ... and does not: one row group of tiles
                                            (2000, 640, 500, 10),       # 128 x 256 tiles; more workgroups than 32-word blocks
                                            (2000, 640, 500, 50),       # ... two row blocks streamed
                                            (3000, 1024, 700, 25),      # hidden update: both shapes launched, the small one works
                                            (3000, 1024, 700, 600),     # ... the large one works
                                            (3000, 512, 1500, 40),      # hidden update: large launch, 32 rows per workgroup after all
                                            (3000, 512, 1500, 700),     # ... up to the row blocks the grid has workgroups for (768)
                                            (3000, 512, 1500, 800),     # ... beyond: 64 rows per workgroup
                                            (3000, 768, 900, 500),
                                            (3000, 768, 900, 600)])
def test_many_raw_queries_few_distinct_histories(V, H, N, distinct):
    """The search repeats itself (Section 5.2): N raw queries, a handful of distinct histories.  The
    host sizes the launch for N rows; the kernel learns the true count on the device and streams
    the weights when it is small."""
    cfg = CONFIGS[3].scaled(V=V, H=H, B=N, K=5)
    model = make_model(cfg)
    rng = np.random.default_rng(V + N)
    x = make_step_inputs(cfg, rng)
    pick = rng.integers(0, distinct, N)
    pick[:distinct] = np.arange(distinct)
    keys = (pick.astype(np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
    prev, h_in = x["prev"][pick], x["h_in"][pick]
    m = load_model(model, "bf16", N)
    for lse_mode in (1, 2):
        m.set_option(rn.OPT_LSE_MODE, lse_mode)
        out = gpu_step_dedup(m, keys, prev, h_in, x["query"])
        U_, rep, inv = oracle.dedup(keys)
        assert out["n_unique"] == U_ == distinct and np.array_equal(out["rep"], rep) and np.array_equal(out["inverse"], inv)
        ref = oracle.step(model, prev[rep], h_in[rep], x["query"], row_of_query=inv)
        check(out["h_out"], out["logprob"], ref, "bf16", "N=%d distinct=%d lse=%d" % (N, distinct, lse_mode))
    assert m.last_error() == 0
    m.close()


@pytest.mark.parametrize("V,H,N,distinct", [(20000, 256, 300, 20),     # fewer splits than workgroups
                                            (40000, 256, 400, 50),     # two row blocks
                                            (5000, 512, 260, 30),      # one row block is all that fits
                                            (5000, 512, 260, 40),      # does not fit: three-term kernel, one row group
                                            (3000, 256, 500, 150)])
def test_many_raw_queries_few_distinct_histories_fp32(V, H, N, distinct):
    """The same for fp32 models (the paper's precision): the three-term kernel derives its work split
    from the true count and streams the fp32 weights when at most 64 rows are left."""
    cfg = CONFIGS[2].scaled(V=V, H=H, B=N, K=5)
    model = make_model(cfg)
    rng = np.random.default_rng(V + N)
    x = make_step_inputs(cfg, rng)
    pick = rng.integers(0, distinct, N)
    pick[:distinct] = np.arange(distinct)
    keys = (pick.astype(np.uint64) + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
    prev, h_in = x["prev"][pick], x["h_in"][pick]
    m = load_model(model, "f32", N)
    for lse_mode in (1, 2):
        m.set_option(rn.OPT_LSE_MODE, lse_mode)
        out = gpu_step_dedup(m, keys, prev, h_in, x["query"])
        U_, rep, inv = oracle.dedup(keys)
        assert out["n_unique"] == U_ == distinct and np.array_equal(out["rep"], rep) and np.array_equal(out["inverse"], inv)
        ref = oracle.step(model, prev[rep], h_in[rep], x["query"], row_of_query=inv)
        check(out["h_out"], out["logprob"], ref, "f32", "fp32 N=%d distinct=%d lse=%d" % (N, distinct, lse_mode))
    assert m.last_error() == 0
    m.close()


@pytest.mark.parametrize("dtype,V,H,B,K", [("bf16", 1500, 640, 5000, 2),     # tiled kernel: more row groups than workgroups per XCD
                                           ("bf16", 3000, 256, 9000, 2),     # staged kernel, 36 row groups
                                           ("f32", 1200, 128, 6000, 2)])     # three-term kernel, 24 row groups
def test_more_row_groups_than_workgroups(dtype, V, H, B, K):
    """Large batches on a small vocabulary: a workgroup takes several (row group, split) items in turn."""
    cfg = CONFIGS[3 if dtype == "bf16" else 2].scaled(V=V, H=H, B=B, K=K)
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed + B))
    m = load_model(model, dtype, B)
    h, lp = gpu_step(m, x["prev"], x["h_in"], x["query"])
    check(h, lp, oracle.step(model, x["prev"], x["h_in"], x["query"]), dtype, "%s V=%d H=%d B=%d" % (dtype, V, H, B))
    assert m.last_error() == 0
    m.close()


# ------------------------------------------------------------------------ config 5: stress, full size, every row
def test_config5_stress_full_size_every_row():
    """All 2048 rows and all 2048 x 64 log-probabilities against the oracle (V = 200000 is not a
    multiple of any tile: the ragged last tile is part of every row's sum)."""
    cfg = CONFIGS[5]
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed))
    m = load_model(model, cfg.dtype, cfg.B)
    h, lp = gpu_step(m, x["prev"], x["h_in"], x["query"])
    ref = oracle.step(model, x["prev"], x["h_in"], x["query"])
    check(h, lp, ref, cfg.dtype, "cfg5 (all %d rows)" % cfg.B)
    assert np.all(lp < 0)
    m.set_option(rn.OPT_OUTPROJ_KERNEL, 1)        # extra: the plain kernel, against the oracle as well
    h1, lp1 = gpu_step(m, x["prev"], x["h_in"], x["query"])
    check(h1, lp1, ref, cfg.dtype, "cfg5 plain kernel (all %d rows)" % cfg.B)
    assert np.array_equal(h1, h)
    assert m.last_error() == 0
    m.close()


# ------------------------------------------------------------------------ config 4: decode trace
def test_config4_reduced_trace_elementwise():
    """A small trace, every step compared in full, the GPU feeding on its own h_out and the
    oracle on its own; grouping indices bit-exact every step."""
    cfg = CONFIGS[4].scaled(V=3000, H=128, N=600, K=4, steps=6)
    model = make_model(cfg)
    m = load_model(model, "bf16", cfg.N)
    tr_g, tr_o = DecodeTrace(cfg), DecodeTrace(cfg)
    xg, xo = tr_g.first(), tr_o.first()
    for step in range(cfg.steps):
        assert np.array_equal(xg["keys"], xo["keys"]) and np.array_equal(xg["query"], xo["query"])
        out = gpu_step_dedup(m, xg["keys"], xg["prev"], xg["h_in"], xg["query"])
        U, rep, inv = oracle.dedup(xo["keys"])
        assert out["n_unique"] == U == tr_o.U0
        assert np.array_equal(out["rep"], rep) and np.array_equal(out["inverse"], inv)
        assert np.all(np.isnan(out["h_out_rest"]))          # rows beyond n_unique stay untouched
        ref = oracle.step(model, xo["prev"][rep], xo["h_in"][rep], xo["query"], row_of_query=inv)
        # own-state drift grows slowly; the per-step bar still has to hold along the trace
        check(out["h_out"], out["logprob"], ref, "bf16", "cfg4-reduced step %d" % step)
        # duplicates of one history get bit-identical answers when they ask the same word
        xg = tr_g.next(xg, out["h_out"], out["inverse"])
        xo = tr_o.next(xo, ref["h_out"], inv)
    assert m.last_error() == 0
    m.close()


def test_config4_full_size_trace():
    """N = 4096 raw queries, about 30 % distinct, 50 chained steps at V = 65536, H = 512; the GPU
    feeds on its own h_out and the oracle on its own.  Every step: grouping bit-exact, every distinct
    history's hidden vector and every raw query's log-probabilities against the oracle, and
    carried-over histories score bit-identically to the step before."""
    cfg = CONFIGS[4]
    model = make_model(cfg)
    m = load_model(model, cfg.dtype, cfg.N)
    tr_g, tr_o = DecodeTrace(cfg), DecodeTrace(cfg)
    xg, xo = tr_g.first(), tr_o.first()
    prev_by_key = {}
    worst_h = worst_lp = 0.0
    for step in range(cfg.steps):
        assert np.array_equal(xg["keys"], xo["keys"]) and np.array_equal(xg["query"], xo["query"])
        assert np.array_equal(xg["prev"], xo["prev"])
        out = gpu_step_dedup(m, xg["keys"], xg["prev"], xg["h_in"], xg["query"])
        U, rep, inv = oracle.dedup(xo["keys"])
        assert out["n_unique"] == U == tr_o.U0, step
        assert np.array_equal(out["rep"], rep) and np.array_equal(out["inverse"], inv), step
        ref = oracle.step(model, xo["prev"][rep], xo["h_in"][rep], xo["query"], row_of_query=inv)
        dh, dlp = check(out["h_out"], out["logprob"], ref, "bf16", "cfg4 step %d (all %d histories)" % (step, U))
        worst_h, worst_lp = max(worst_h, dh), max(worst_lp, dlp)
        assert np.all(out["logprob"] < 0), step
        # cache reuse: the same history id seen in the previous step gives the same h_out bits
        keys_u = xg["keys"][rep]
        hits = 0
        for u, k in enumerate(keys_u.tolist()):
            if k in prev_by_key:
                assert np.array_equal(out["h_out"][u], prev_by_key[k]), (step, u)
                hits += 1
        if step:
            assert hits == int(xg["carried"].sum()) > 0
        prev_by_key = {k: out["h_out"][u].copy() for u, k in enumerate(keys_u.tolist())}
        xg = tr_g.next(xg, out["h_out"], out["inverse"])
        xo = tr_o.next(xo, ref["h_out"], inv)
    print("cfg4 trace: worst max|dh|=%.3g max|dlogprob|=%.3g over %d steps" % (worst_h, worst_lp, cfg.steps), flush=True)
    assert m.last_error() == 0
    m.close()


# ------------------------------------------------------------------------ grouping of equal ids
@pytest.mark.parametrize("N,distinct", [(0, 1), (1, 1), (2, 1), (63, 7), (1024, 1024), (4096, 1229), (4096, 1),
                                        (4097, 1300), (6000, 2500), (7168, 7168), (7168, 1), (7169, 3000),   # up to 7168: one workgroup
                                        (100000, 30000), (100000, 100000), (50000, 3),
                                        (1100000, 300000)])                                                # more than 1024 counting workgroups
def test_dedup_bit_exact(N, distinct):
    rng = np.random.default_rng(N * 7 + distinct)
    pool = rng.integers(0, 2 ** 64, size=distinct, dtype=np.uint64)
    pool[0] = np.uint64(0xFFFFFFFFFFFFFFFF)              # the all-ones id is an ordinary id
    if distinct > 2:
        pool[1], pool[2] = np.uint64(0), np.uint64(1) << np.uint64(63)
    keys = pool[rng.integers(0, distinct, size=N)] if N else np.zeros(0, np.uint64)
    if N == distinct:
        keys = pool[rng.permutation(N)]
    U, rep, inv = gpu_dedup(keys)
    Uo, repo, invo = oracle.dedup(keys) if N <= 5000 else None_or_numpy(keys)
    assert U == Uo
    assert np.array_equal(rep, repo) and np.array_equal(inv, invo)
    for _ in range(100 if N <= 100000 else 20):           # run-to-run identical (the order never comes from a race)
        U2, rep2, inv2 = gpu_dedup(keys)
        assert U2 == U and np.array_equal(rep2, rep) and np.array_equal(inv2, inv)


def None_or_numpy(keys):
    """For sizes where the quadratic oracle is slow: the first-appearance reordering of
    numpy.unique, which tests/test_oracle_pins.py shows equal to the oracle."""
    uniq, first, inv = np.unique(keys, return_index=True, return_inverse=True)
    order = np.argsort(first, kind="stable")
    rank = np.empty_like(order)
    rank[order] = np.arange(len(order))
    return len(uniq), first[order].astype(np.int32), rank[inv].astype(np.int32)


# ------------------------------------------------------------------------ edge cases
def small_model(dtype="bf16", V=500, H=64, seed=3):
    cfg = CONFIGS[3].scaled(V=V, H=H, B=16, K=4, dtype=dtype)
    return cfg, make_model(cfg, seed=seed)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_zero_initial_hidden_and_single_row(dtype):
    cfg, model = small_model(dtype)
    m = load_model(model, dtype, 16)
    prev = np.array([7], np.int32)
    h0 = np.zeros((1, cfg.H), np.float32)                 # utterance start: zero hidden vector
    q = np.array([[0, 499, 7, 7]], np.int32)              # repeated query words are allowed
    h, lp = gpu_step(m, prev, h0, q)
    check(h, lp, oracle.step(model, prev, h0, q), dtype, "zero h_in, B=1")
    assert lp[0, 2] == lp[0, 3]
    m.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_empty_batches_are_no_ops(dtype):
    cfg, model = small_model(dtype)
    m = load_model(model, dtype, 16)
    e_i = torch.zeros(0, dtype=torch.int32, device="cuda:0")
    rn.rnnlm_step(m, e_i, torch.zeros((0, cfg.H), device="cuda:0"), torch.zeros((0, 4), dtype=torch.int32, device="cuda:0"),
                  torch.zeros((0, cfg.H), device="cuda:0"), torch.zeros((0, 4), device="cuda:0"))
    # K = 0: hidden update still happens
    x = make_step_inputs(cfg, np.random.default_rng(0))
    h, lp = gpu_step(m, x["prev"], x["h_in"], np.zeros((16, 0), np.int32))
    ref = oracle.step(model, x["prev"], x["h_in"], np.zeros((16, 0), np.int32))
    assert lp.shape == (16, 0)
    assert np.max(np.abs(h - ref["h_out"])) <= TOL[dtype][1]
    torch.cuda.synchronize()
    assert m.last_error() == 0
    m.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_row_of_query_fan_out_and_duplicates(dtype):
    cfg, model = small_model(dtype)
    m = load_model(model, dtype, 64)
    rng = np.random.default_rng(5)
    x = make_step_inputs(cfg, rng)
    N = 50
    roq = rng.integers(0, cfg.B, N).astype(np.int32)
    q = rng.integers(0, cfg.V, (N, 4)).astype(np.int32)
    q[10], roq[10] = q[3], roq[3]                        # a repeated lookup
    h, lp = gpu_step(m, x["prev"], x["h_in"], q, row_of_query=roq)
    check(h, lp, oracle.step(model, x["prev"], x["h_in"], q, row_of_query=roq), dtype, "fan-out")
    assert np.array_equal(lp[10], lp[3])
    m.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bad_indices_raise_flags_and_nan_only_where_they_apply(dtype):
    cfg, model = small_model(dtype)
    m = load_model(model, dtype, 64)
    x = make_step_inputs(cfg, np.random.default_rng(1))
    good_h, good_lp = gpu_step(m, x["prev"], x["h_in"], x["query"])
    assert m.last_error() == 0
    prev = x["prev"].copy(); prev[3] = cfg.V             # one past the end
    q = x["query"].copy(); q[5, 1] = -1
    h, lp = gpu_step(m, prev, x["h_in"], q)
    assert m.last_error() == rn.FLAG_BAD_PREV_WORD | rn.FLAG_BAD_QUERY_WORD
    assert m.last_error() == 0                            # reading clears the flag
    assert np.all(np.isnan(h[3])) and np.all(np.isnan(lp[3]))
    assert np.isnan(lp[5, 1])
    ok_rows = [r for r in range(cfg.B) if r != 3]
    assert np.array_equal(h[ok_rows], good_h[ok_rows])
    mask = np.ones_like(lp, bool); mask[3] = False; mask[5, 1] = False
    assert np.array_equal(lp[mask], good_lp[mask])
    roq = np.arange(cfg.B, dtype=np.int32); roq[2] = cfg.B
    h, lp = gpu_step(m, x["prev"], x["h_in"], x["query"], row_of_query=roq)
    assert m.last_error() == rn.FLAG_BAD_ROW
    assert np.all(np.isnan(lp[2])) and np.array_equal(lp[[0, 1, 3]], good_lp[[0, 1, 3]])
    m.close()


def test_range_and_argument_errors_with_a_real_model():
    cfg, model = small_model("bf16")
    m = load_model(model, "bf16", 8)
    x = make_step_inputs(cfg, np.random.default_rng(1))    # 16 rows > max_B = 8
    with pytest.raises(rn.RnnlmError) as e:
        gpu_step(m, x["prev"], x["h_in"], x["query"])
    assert e.value.status == -4
    h = torch.zeros((4, cfg.H), device="cuda:0")
    with pytest.raises(rn.RnnlmError) as e:               # h_out aliasing h_in
        rn.rnnlm_step(m, torch.zeros(4, dtype=torch.int32, device="cuda:0"), h,
                      torch.zeros((4, 2), dtype=torch.int32, device="cuda:0"), h, torch.zeros((4, 2), device="cuda:0"))
    assert e.value.status == -1
    with pytest.raises(rn.RnnlmError):
        m.set_option(99, 0)
    m.close()
    with pytest.raises(ValueError):
        m.handle


def test_running_maximum_fallback_when_logits_are_huge():
    """Weights so large that no fixed offset fits fp32: the library must fall back to the
    running maximum by itself, and the forced fixed offset must be refused."""
    rng = np.random.default_rng(2)
    V, H, B, K = 400, 64, 40, 4
    model = {"U": rng.normal(0, 0.5, (V, H)).astype(np.float32), "W": rng.normal(0, 0.1, (H, H)).astype(np.float32),
             "O": rng.normal(0, 4.0, (H, V)).astype(np.float32), "bias": rng.normal(0, 1, V).astype(np.float32)}
    m = load_model(model, "f32", B)
    with pytest.raises(rn.RnnlmError):
        m.set_option(rn.OPT_LSE_MODE, 2)
    prev, h_in, q = rng.integers(0, V, B), rng.random((B, H)), rng.integers(0, V, (B, K))
    h, lp = gpu_step(m, prev, h_in, q)
    ref = oracle.step(model, prev, h_in, q)
    assert np.max(np.abs(h - ref["h_out"])) <= 1e-5
    # logits are O(100): fp32 cannot hold them to 1e-5 absolute; 1e-6 relative to |z| can be asked
    scale = np.max(np.abs(ref["logprob"]))
    assert np.max(np.abs(lp - ref["logprob"])) <= 5e-6 * scale + 1e-5
    m.close()


# ------------------------------------------------------------------------ a vocabulary of the paper's largest size
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_million_word_vocabulary(dtype):
    """V = 1,000,003 (Section 5.1's in-house vocabulary is about a million words; odd on purpose:
    ragged last tile), H = 128, full softmax: 130 rows (bf16: staged kernel; fp32: three-term
    kernel) and the first 20 of them alone (weight-streaming kernels)."""
    rng = np.random.default_rng(99)
    V, H, B, K = 1000003, 128, 130, 6
    from workloads import bounded_zipf_ids, round_to_bf16
    model = {k: rng.normal(0, 0.05, s).astype(np.float32) for k, s in (("U", (V, H)), ("W", (H, H)), ("O", (H, V)))}
    model["bias"] = None
    if dtype == "bf16":
        for k in ("U", "W", "O"):
            model[k] = round_to_bf16(model[k])
    m = load_model(model, dtype, B)
    prev = bounded_zipf_ids(rng, V, 1.1, B)
    prev[0] = V - 1
    h_in = rng.uniform(0, 1, (B, H)).astype(np.float32)
    query = bounded_zipf_ids(rng, V, 1.1, (B, K))
    query[:, 0] = V - 1 - np.arange(B)                  # words of the last, ragged tile
    ref = oracle.step(model, prev, h_in, query)
    h, lp = gpu_step(m, prev, h_in, query)
    check(h, lp, ref, dtype, "V=1000003 %s, %d rows" % (dtype, B))
    h, lp = gpu_step(m, prev[:20], h_in[:20], query[:20])
    check(h, lp, {"h_out": ref["h_out"][:20], "logprob": ref["logprob"][:20]}, dtype, "V=1000003 %s, 20 rows" % dtype)
    assert m.last_error() == 0
    m.close()


# ------------------------------------------------------------------------ measurement aid
def test_matrix_rate_probe_reports_a_rate_between_nothing_and_the_data_sheet_peak():
    """rnnlm_probe_mfma_rate: the figures bench.py prints beside the roofline.  All-zero operands may
    not be slower than random ones (same instruction stream; only the clock under load differs)."""
    rates = {}
    for feed in (0, 1):
        for data in (0, 1):
            tf, ghz = rn.rnnlm_probe_mfma_rate(feed, data, 5)
            assert 100.0 < tf < 2600.0 and 0.3 < ghz < 3.0, (feed, data, tf, ghz)
            rates[(feed, data)] = tf
    assert rates[(0, 0)] >= 0.95 * rates[(0, 1)] and rates[(1, 0)] >= 0.95 * rates[(1, 1)]
