#!/usr/bin/env python3
"""Benchmark of the batched RNNLM step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = one pass of the whole hot path over one batch of the headline workload
(V = 65536, H = 512, B = N = 1024 hypotheses, K = 32 query words each, bf16 weights):
grouping of the history ids, hidden update, fused output projection + log-sum-exp, query
gather -- a single rnnlm_step_dedup call, inputs already resident in HBM.  Prints ONE JSON
line: whole-job hypothesis-steps/s, the roofline of the dominant kernel (output projection
+ log-sum-exp, MFMA-bound) timed with HIP events on its stream, and the CPU oracle timed on
a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0        # MI355X dense bf16 MFMA, published
PEAK_FP32_TFLOPS = 157.3         # MI355X fp32 vector (and fp32 matrix), published
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E, published
# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) scaled
# by a plain copy of known size; they cannot be measured live, so every figure names the kernel it was
# measured on and the summary under profiles/ that holds the command, and is only reported when the
# launch that was timed is that kernel on that workload (otherwise "traffic" is null).
TRAFFIC = {
    ("outproj_staged_kernel<512, true>", 3): (78.0e6, "profiles/step_kernels_cfg3_large_vocab_hbm_traffic.md"),
    ("outproj_rowstream_kernel", 5): (1238.0e6, "profiles/outproj_rowstream_cfg5_stress_hbm_fetch.md"),
    ("outproj_stream_kernel", 6): (260.3e6, "profiles/step_kernels_cfg6_paper_regime_kernel_trace.md"),
    ("outproj_stream_kernel", 2): (21.2e6, "profiles/outproj_stream_few_rows_kernel_trace_and_fetch.md"),
    ("outproj_stream_kernel", 3): (67.8e6, "profiles/outproj_stream_few_rows_kernel_trace_and_fetch.md"),
    ("outproj_stream_kernel", 5): (411.5e6, "profiles/outproj_stream_few_rows_kernel_trace_and_fetch.md"),
}
# The path kernel of the hierarchical output layer, by workload number: HBM bytes per launch
# (FETCH_SIZE + WRITE_SIZE, copy-calibrated).
HS_TRAFFIC = {
    3: (53.8e6, "profiles/hs_step_cfg3_shape_kernel_trace_and_traffic.md"),
    6: (2.83e6, "profiles/hs_step_cfg6_paper_regime_kernel_trace_and_traffic.md"),
}
MIN_TIMED_REGION_S = 0.1         # the event-timed repetitions together last at least this long
MIN_REPETITIONS = 20


def timed_repetitions(step, steps, first_pass_s, torch):
    """`steps` calls of step() between two events on the launch stream, repeated at least
    MIN_REPETITIONS times and for at least MIN_TIMED_REGION_S in all (whatever --steps says);
    the repetitions queue back to back.  Returns the per-repetition times in ms, sorted."""
    reps = max(MIN_REPETITIONS, int(MIN_TIMED_REGION_S / max(first_pass_s, 1e-6)) + 1)
    reps = min(reps, 2000)
    pairs = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        pairs.append((e0, e1))
    torch.cuda.synchronize()
    return sorted(a.elapsed_time(b) for a, b in pairs)


def median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def bench_hs(args, cfg, rn, torch, np) -> int:
    """One step = hidden update + path evaluation of the N x K queried words (rnnlm_hs_step) on
    the chosen workload's shape.  The tree is Huffman's over the workload's Zipf word frequencies,
    node vectors N(0, (4 sigma)^2); inputs as the full-softmax bench."""
    from workloads import bf16_bits, make_model, make_step_inputs
    dev = "cuda:0"
    bf16 = cfg.dtype == "bf16"
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(cfg.seed)) if cfg.unique_frac is None else None
    V, H, N, K = cfg.V, cfg.H, cfg.N, cfg.K
    freq = np.arange(1, V + 1, dtype=np.float64) ** -(cfg.zipf_s or 0.0)
    off, entry = rn.rnnlm_huffman_build(freq)
    theta = np.random.default_rng(cfg.seed + 7).normal(0, 4 * cfg.sigma, (V - 1, H)).astype(np.float32)
    if bf16:
        theta = bf16_round(theta, np)
        m = rn.rnnlm_hs_load(V, H, rn.RNNLM_BF16, bf16_bits(model["U"]), bf16_bits(model["W"]), bf16_bits(theta), off,
                             entry, N)
    else:
        m = rn.rnnlm_hs_load(V, H, rn.RNNLM_F32, model["U"], model["W"], theta, off, entry, N)
    if args.cache is not None:
        return bench_hs_cached(args, cfg, m, rn, torch, np)
    prev = torch.from_numpy(x["prev"]).to(dev)
    h_in = torch.from_numpy(x["h_in"]).to(dev)
    query = torch.from_numpy(x["query"]).to(dev)
    h_out = torch.zeros((N, H), device=dev)
    lp = torch.zeros((N, K), device=dev)

    def step():
        rn.rnnlm_hs_step(m, prev, h_in, query, h_out, lp)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_first = time.perf_counter() - t0
    rep_ms = timed_repetitions(step, args.steps, dt_first, torch)
    dt = median(rep_ms) * 1e-3
    assert m.last_error() == 0
    k_ms = median([rn.rnnlm_hs_time_query(m, query, h_out, lp, 20) for _ in range(7)])
    nodes = int(np.diff(off)[x["query"]].sum())              # path nodes of all queried words
    # the kernel computes one dot product per DISTINCT node of a raw query's K paths
    node_of = entry & 0x7FFFFFFF
    distinct = sum(len(set(np.concatenate([node_of[off[w]:off[w + 1]] for w in row]).tolist())) for row in x["query"])
    es = 2 if bf16 else 4
    alg_bytes = distinct * H * es + N * H * 4 + N * K * 8.0
    # HBM bytes per launch of the path kernel as rocprofv3 counted them (FETCH_SIZE + WRITE_SIZE, scaled by a
    # plain copy of known size): the upper tree levels repeat across queries and come out of L2, so this is
    # less than the algorithmic figure; the roofline fraction is taken on what HBM really moved
    traffic, traffic_source = HS_TRAFFIC.get(args.config, (None, None))
    moved = traffic if traffic is not None else alg_bytes
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        om = {"U": model["U"], "W": model["W"], "theta": theta,
              "path_off": off, "path_entry": entry}
        rows = N                                   # the whole step: the tree makes the oracle cheap too
        t = time.perf_counter()
        ref = oracle.hs_step(om, x["prev"][:rows], x["h_in"][:rows], x["query"][:rows])
        cdt = time.perf_counter() - t
        cpu = {"value": round(rows / cdt, 2), "unit": "hypothesis-steps/s", "cores": oracle.max_threads(), "kind": "oracle",
               "sample": "all %d rows of the same step (hidden update + paths of their %d queried words), %.3f s wall"
                         % (rows, rows * K, cdt),
               "max_abs_dlogprob_vs_gpu": float(np.max(np.abs(lp.cpu().numpy()[:rows] - ref["logprob"])))}
    out = {"metric": "RNNLM hypothesis-steps/sec, hierarchical output layer (V=%d,H=%d,B=%d)" % (V, H, N),
           "value": round(N * args.steps / dt, 1), "unit": "hypothesis-steps/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
           "config": {"workload": "%s with the hierarchical output layer: V=%d H=%d B=N=%d K=%d, Huffman tree over "
                                  "Zipf(%g) frequencies, mean path of a queried word %.1f nodes, %.0f distinct nodes "
                                  "among the %d words of a query"
                                  % (cfg.name, V, H, N, K, cfg.zipf_s or 0, nodes / float(N * K), distinct / float(N), K)},
           "timing": {"method": "median of %d repetitions of %d steps, each bracketed by HIP events on the launch stream"
                                % (len(rep_ms), args.steps)},
           "roofline": {"kernel": "hs_query_shared_kernel" if K >= 4 else "hs_query_kernel", "bound": "hbm",
                        "achieved": round(moved / (k_ms * 1e-3) / 1e9, 1),
                        "peak": 8000.0, "unit": "GB/s", "frac": round(moved / (k_ms * 1e-3) / 8e12, 4),
                        "traffic": traffic, "traffic_source": traffic_source,
                        "us_per_launch": round(k_ms * 1e3, 2), "algorithmic_bytes_per_launch": alg_bytes,
                        "algorithmic_gbs_incl_l2_hits": round(alg_bytes / (k_ms * 1e-3) / 1e9, 1),
                        "note": ("achieved = HBM bytes per launch from the profile / launch time" if traffic is not None else
                                 "no HBM counter figure for this workload: achieved uses the algorithmic bytes, an "
                                 "upper bound of what HBM moved") +
                                "; algorithmic bytes = one node vector per distinct path node of every raw query + "
                                "hidden rows + ids and outputs (the upper tree levels repeat across queries and are "
                                "served by L2)"},
           "cpu_baseline": cpu}
    print(json.dumps(out))
    m.close()
    return 0


def bench_hs_cached(args, cfg, m, rn, torch, np) -> int:
    """The paper's whole RnnlmProb (Table 1): a decode trace of raw queries through the cache kept between
    steps, scored with the hierarchical output layer (rnnlm_step_cached on a model loaded with
    rnnlm_hs_load).  A "step" of the timed loop is a pass over the whole trace (one utterance: the cache is
    reset at its start); reported per step of the trace, beside the same trace without the cache."""
    from workloads import DecodeTrace
    if cfg.unique_frac is None:
        print("bench.py: --cache needs the decode-trace workload (--config 4)", file=sys.stderr)
        return 2
    dev = "cuda:0"
    N, K, H = cfg.N, cfg.K, cfg.H
    rep = torch.empty(N, dtype=torch.int32, device=dev)
    inv = torch.empty(N, dtype=torch.int32, device=dev)
    nu = torch.zeros(1, dtype=torch.int32, device=dev)
    h_out = torch.zeros((N, H), device=dev)
    lp = torch.zeros((N, K), device=dev)
    ws = torch.empty(rn.rnnlm_dedup_workspace_bytes(N), dtype=torch.uint8, device=dev)
    tr = DecodeTrace(cfg, carry_frac=args.carry_frac)
    xt, trace = tr.first(), []
    for _ in range(args.trace_steps):               # built once, untimed: step t+1 grows from what step t returned
        dev_in = tuple(torch.from_numpy(a).to(dev) for a in (xt["keys"].view(np.int64), xt["prev"], xt["h_in"], xt["query"]))
        rn.rnnlm_step_dedup(m, *dev_in, rep, inv, nu, h_out, lp, ws)
        torch.cuda.synchronize()
        trace.append(dev_in)
        xt = tr.next(xt, h_out.cpu().numpy(), inv.cpu().numpy())
    cache = rn.rnnlm_cache_create(m, args.cache)
    stats = torch.zeros(4, dtype=torch.int32, device=dev)

    def cached_pass():
        cache.reset()
        for dev_in in trace:
            rn.rnnlm_step_cached(m, cache, *dev_in, rep, inv, nu, h_out, lp, ws, step_stats=stats)

    def uncached_pass():
        for dev_in in trace:
            rn.rnnlm_step_dedup(m, *dev_in, rep, inv, nu, h_out, lp, ws)

    results = {}
    for name, fn in (("uncached", uncached_pass), ("cached", cached_pass)):
        for _ in range(max(args.warmup, 1)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        rep_ms = timed_repetitions(fn, args.steps, time.perf_counter() - t0, torch)
        results[name] = median(rep_ms) * 1e-3 / (args.steps * args.trace_steps)
    st = cache.stats()
    assert m.last_error() == 0
    out = {"metric": "RNNLM hypothesis-steps/sec, hierarchical output layer through the cache (V=%d,H=%d,N=%d)" % (cfg.V, H, N),
           "value": round(N / results["cached"], 1), "unit": "hypothesis-steps/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(results["cached"] * 1e3, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
           "config": {"workload": "%s with the hierarchical output layer through the cache: V=%d H=%d N=%d raw queries "
                                  "(%d distinct histories per step, %.0f %% of them kept from step to step) K=%d, trace of "
                                  "%d steps, cache reset at its start"
                                  % (cfg.name, cfg.V, H, N, tr.U0, 100 * args.carry_frac, K, args.trace_steps)},
           "timing": {"method": "median of event-bracketed repetitions of %d passes over the trace" % args.steps},
           "roofline": None, "cpu_baseline": None,
           "cache": {"capacity": args.cache, "trace_steps": args.trace_steps, "carry_frac": args.carry_frac,
                     "uncached_value": round(N / results["uncached"], 1),
                     "uncached_ms_per_step": round(results["uncached"] * 1e3, 4),
                     "hit_ratio": round(st["hits"] / max(st["lookups"], 1), 4), "entries": st["entries"],
                     "note": "value = raw queries / s over the trace through the cache; hit_ratio over distinct "
                             "histories per step; uncached_value = same trace without the cache"}}
    print(json.dumps(out))
    cache.close()
    m.close()
    return 0


def bf16_round(a, np):
    from workloads import round_to_bf16
    return round_to_bf16(a)


def bench_index_table(args, cfg, rn, torch, np) -> int:
    """One "step" = the N*K contexts that follow a step (queried word, updated hidden vector of its
    history) turned into indices; reported for new contexts and for contexts the table already
    holds, plus the fetch of N contexts.  Prints one JSON line; HBM-bound (every call walks the
    hidden vectors once)."""
    dev = "cuda:0"
    M, H = cfg.N * cfg.K, cfg.H
    reps = max(4, min(args.steps, 40))
    table = rn.rnnlm_index_create(H, M * (reps + 2), M)
    g = torch.Generator(device=dev).manual_seed(cfg.seed)
    word = torch.randint(0, cfg.V, (M,), generator=g, device=dev, dtype=torch.int32)
    batches = [torch.rand((M, H), generator=g, device=dev) for _ in range(reps + 1)]
    index = torch.zeros(M, dtype=torch.int32, device=dev)
    rn.rnnlm_index_intern(table, word, batches[0], index)            # warm-up
    torch.cuda.synchronize()

    def timed(fn, n):
        t0 = time.perf_counter()
        for i in range(n):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    t_new = timed(lambda i: rn.rnnlm_index_intern(table, word, batches[1 + i], index), reps)
    t_known = timed(lambda i: rn.rnnlm_index_intern(table, word, batches[1 + i], index), reps)
    w2 = torch.zeros(cfg.N, dtype=torch.int32, device=dev)
    h2 = torch.zeros((cfg.N, H), device=dev)
    t_fetch = timed(lambda i: rn.rnnlm_index_fetch(table, index[: cfg.N], w2, h2), reps)
    st = table.stats()
    assert st["collisions"] == 0 and st["bad_fetch"] == 0 and st["unstored"] == 0
    row_bytes = 4.0 * H
    out = {"metric": "IndexTable contexts/sec (H=%d, %d contexts per call)" % (H, M),
           "value": round(M / t_new, 1), "unit": "contexts/s", "n_gpus": 1, "steps": reps, "warmup": 1,
           "ms_per_step": round(t_new * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "u32", "data": "synthetic",
           "config": {"workload": "%s: contexts of the step's shape, N*K = %d x H = %d floats, all new" % (cfg.name, M, H)},
           "roofline": {"kernel": "context_hash + index_commit", "bound": "hbm",
                        "achieved": round(3 * M * row_bytes / t_new / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                        "frac": round(3 * M * row_bytes / t_new / 8e12, 4), "traffic": None,
                        "note": "algorithmic bytes of a call with new contexts: rows read by the hash, read and "
                                "written by the commit = 3 x %d x %d B" % (M, int(row_bytes))},
           "cpu_baseline": None,
           "index_table": {"intern_new_us": round(t_new * 1e6, 1), "intern_known_us": round(t_known * 1e6, 1),
                           "fetch_%d_us" % cfg.N: round(t_fetch * 1e6, 1), "entries": st["entries"]}}
    print(json.dumps(out))
    table.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--outproj-kernel", type=int, default=0,
                    help="0 auto, 1 plain, 2 staged, 3 tiled, 4 bf16 three-term split (fp32 models), "
                         "5 weight streaming (bf16 models, few rows)")
    ap.add_argument("--rows", type=int, default=None, metavar="B",
                    help="the chosen workload with only B rows per step (full-softmax workloads 1, 2, 3, 5): "
                         "the few distinct histories a well-cached search leaves; up to 64 rows of a bf16 "
                         "model the output projection is then bound by reading the weights once, and the "
                         "roofline is reported against HBM bandwidth")
    ap.add_argument("--lse-mode", type=int, default=0, help="0 auto, 1 running max, 2 fixed offset")
    ap.add_argument("--config", type=int, default=3,
                    help="workload number (default 3 = the headline one the metric is quoted on; "
                         "4 and 5 are the decode-trace and stress workloads)")
    ap.add_argument("--cache", type=int, default=None, metavar="CAPACITY",
                    help="config 4 only: time a decode trace of --trace-steps steps through a cache of "
                         "CAPACITY histories kept between the steps (reset at the start of every pass)")
    ap.add_argument("--trace-steps", type=int, default=8)
    ap.add_argument("--unique-frac", type=float, default=None,
                    help="config 4 only: share of distinct histories among the N raw queries of a step "
                         "(0.3 in the workload as specified; the paper reports about 0.1)")
    ap.add_argument("--carry-frac", type=float, default=0.5,
                    help="config 4 with --cache: share of the distinct histories kept from one step of the "
                         "trace to the next, i.e. found in the cache (0.5 as specified; the paper reports "
                         "a hit ratio of almost 0.89)")
    ap.add_argument("--gemm-reference", action="store_true",
                    help="also time the platform's GEMM (torch.matmul, bf16) on the output projection's "
                         "contraction alone, logits written to HBM, no log-sum-exp: context for the roofline")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the matrix-core rate probe that is run after the timed region when the "
                         "roofline is the MFMA one (rnnlm_probe_mfma_rate: what the device sustains on the "
                         "output projection's loop shape, reported beside the data-sheet peak); "
                         "--no-cpu-baseline skips it too (runs under a profiler)")
    ap.add_argument("--graph-steps", type=int, default=0, metavar="G",
                    help="also record G steps into one HIP graph and time its replays (reported under "
                         "\"graph\"; the headline value stays the eager one)")
    ap.add_argument("--hs", action="store_true",
                    help="the chosen workload with the hierarchical output layer (Huffman tree over the "
                         "Zipf word frequencies) in place of the full softmax")
    ap.add_argument("--index-table", action="store_true",
                    help="time the device-side IndexTable instead of the step: contexts of the chosen "
                         "workload's shape (N x K contexts of H floats) turned into indices and fetched back")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy kernel, as the known-size "
                         "reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (rows are independent, so the step would shard "
              "by replicating the weights and splitting the rows); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2007_11794_amd as rn
    from workloads import CONFIGS, DecodeTrace, bf16_bits, make_model, make_step_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    rn.lib()                                   # raises if librnnlm.so is not built
    dev = "cuda:0"
    cfg = CONFIGS[args.config]
    if args.rows is not None:
        if cfg.unique_frac is not None or args.rows < 1 or args.rows > cfg.B:
            print("bench.py: --rows needs a workload without a decode trace and 1 <= B <= its row count",
                  file=sys.stderr)
            return 2
        cfg = cfg.scaled(B=args.rows)
    if args.unique_frac is not None:
        if cfg.unique_frac is None or not 0.0 < args.unique_frac <= 1.0:
            print("bench.py: --unique-frac needs the decode-trace workload (--config 4) and a share in (0, 1]",
                  file=sys.stderr)
            return 2
        cfg = cfg.scaled(unique_frac=args.unique_frac, B=int(round(args.unique_frac * cfg.N)))
    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)      # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.index_table:
        return bench_index_table(args, cfg, rn, torch, np)
    if args.hs:
        if (cfg.unique_frac is not None) != (args.cache is not None):
            print("bench.py: --hs times one row per raw query (workloads 1, 2, 3, 5, 6), or with --cache the "
                  "decode-trace workload (--config 4) through the cache", file=sys.stderr)
            return 2
        return bench_hs(args, cfg, rn, torch, np)
    bf16 = cfg.dtype == "bf16"
    model = make_model(cfg)
    if cfg.unique_frac is not None:
        x = DecodeTrace(cfg).first()               # N raw queries, about 30 % distinct histories
    else:
        x = make_step_inputs(cfg, np.random.default_rng(cfg.seed))
    if bf16:
        m = rn.rnnlm_load(cfg.V, cfg.H, rn.RNNLM_BF16, bf16_bits(model["U"]), bf16_bits(model["W"]),
                          bf16_bits(model["O"]), None, cfg.N)
    else:
        m = rn.rnnlm_load(cfg.V, cfg.H, rn.RNNLM_F32, model["U"], model["W"], model["O"], None, cfg.N)
    m.set_option(rn.OPT_OUTPROJ_KERNEL, args.outproj_kernel)
    m.set_option(rn.OPT_LSE_MODE, args.lse_mode)

    N, K, H = cfg.N, cfg.K, cfg.H
    keys = torch.from_numpy(x["keys"].view(np.int64)).to(dev)
    prev = torch.from_numpy(x["prev"]).to(dev)
    h_in = torch.from_numpy(x["h_in"]).to(dev)
    query = torch.from_numpy(x["query"]).to(dev)
    rep = torch.empty(N, dtype=torch.int32, device=dev)
    inv = torch.empty(N, dtype=torch.int32, device=dev)
    nu = torch.zeros(1, dtype=torch.int32, device=dev)
    h_out = torch.zeros((N, H), device=dev)
    lp = torch.zeros((N, K), device=dev)
    ws = torch.empty(rn.rnnlm_dedup_workspace_bytes(N), dtype=torch.uint8, device=dev)

    def step():
        rn.rnnlm_step_dedup(m, keys, prev, h_in, query, rep, inv, nu, h_out, lp, ws)

    cache_info = None
    if args.cache is not None:
        if cfg.unique_frac is None:
            print("bench.py: --cache needs the decode-trace workload (--config 4)", file=sys.stderr)
            return 2
        # The trace is built once, untimed: step t+1 grows from the hidden vectors step t returned.
        tr = DecodeTrace(cfg, carry_frac=args.carry_frac)
        xt, trace = tr.first(), []
        for _ in range(args.trace_steps):
            dev_in = tuple(torch.from_numpy(a).to(dev) for a in
                           (xt["keys"].view(np.int64), xt["prev"], xt["h_in"], xt["query"]))
            rn.rnnlm_step_dedup(m, *dev_in, rep, inv, nu, h_out, lp, ws)
            torch.cuda.synchronize()
            trace.append(dev_in)
            xt = tr.next(xt, h_out.cpu().numpy(), inv.cpu().numpy())
        cache = rn.rnnlm_cache_create(m, args.cache)
        stats = torch.zeros(4, dtype=torch.int32, device=dev)

        def step():                                 # one pass over the whole trace = one utterance
            cache.reset()
            for dev_in in trace:
                rn.rnnlm_step_cached(m, cache, *dev_in, rep, inv, nu, h_out, lp, ws, step_stats=stats)

        def uncached_pass():
            for dev_in in trace:
                rn.rnnlm_step_dedup(m, *dev_in, rep, inv, nu, h_out, lp, ws)

        for _ in range(3):
            uncached_pass()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            uncached_pass()
        torch.cuda.synchronize()
        cache_info = {"capacity": args.cache, "trace_steps": args.trace_steps, "carry_frac": args.carry_frac,
                      "uncached_value": round(N * args.trace_steps * 20 / (time.perf_counter() - t0), 1)}

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # exactly --steps steps between two synchronisations (host clock) ...
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_first = time.perf_counter() - t0
    # ... and the same --steps steps again and again between HIP events on the launch stream: the
    # reported figure is the median repetition
    rep_ms = timed_repetitions(step, args.steps, dt_first, torch)
    dt = median(rep_ms) * 1e-3
    B = int(nu.item())                              # distinct histories actually scored
    assert (B == cfg.B or cfg.unique_frac is not None) and m.last_error() == 0
    ms_per_step = dt / args.steps * 1e3
    value = N * args.steps / dt
    timing = {"method": "median of %d repetitions of %d steps, each bracketed by HIP events on the launch stream"
                        % (len(rep_ms), args.steps),
              "ms_per_step_min": round(rep_ms[0] / args.steps, 4), "ms_per_step_max": round(rep_ms[-1] / args.steps, 4),
              "ms_per_step_first_pass_host_clock": round(dt_first / args.steps * 1e3, 4)}
    if cache_info is not None:                      # a "step" was a pass over the whole trace
        ms_per_step /= args.trace_steps
        value *= args.trace_steps
        for k in ("ms_per_step_min", "ms_per_step_max", "ms_per_step_first_pass_host_clock"):
            timing[k] = round(timing[k] / args.trace_steps, 4)
        st = cache.stats()
        cache_info.update(hit_ratio=round(st["hits"] / max(st["lookups"], 1), 4), entries=st["entries"],
                          note="value = raw queries / s over the trace through the cache; hit_ratio over "
                               "distinct histories per step; uncached_value = same trace without the cache")

    graph_info = None
    if args.graph_steps > 0 and cache_info is None:
        # the same steps recorded once and replayed: what a serving loop that batches several steps
        # (of different utterances) into one graph launch sees
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(g, stream=side):
            for _ in range(args.graph_steps):
                step()
        torch.cuda.synchronize()
        replays = max(1, args.steps // args.graph_steps)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            g.replay()
        torch.cuda.synchronize()
        g_dt = time.perf_counter() - t0
        graph_info = {"steps_per_graph": args.graph_steps, "replays": replays,
                      "ms_per_step": round(g_dt / (replays * args.graph_steps) * 1e3, 4),
                      "value": round(N * replays * args.graph_steps / g_dt, 1)}

    # dominant kernel: output projection + log-sum-exp, timed alone with HIP events on its stream, launched
    # as the timed step launches it (the kernel reads the number of distinct rows from the device)
    reps = 50 if cfg.V * cfg.H <= 65536 * 512 else 10
    k3_groups = sorted(m.time_outproj(cfg.N, reps, n_rows_dev=nu) for _ in range(7))
    k3_ms = median(k3_groups)
    flops = 2.0 * B * cfg.H * cfg.V                 # the contraction on the distinct rows, each product once
    # fp32 models run the contraction on the bf16 matrix cores (from 64 rows on the tiled kernel,
    # below that the weight-streaming one when H <= 768): six bf16 products per fp32 product
    # (three-term split of both operands); `achieved` counts every fp32 product once, the rate at
    # which bf16 products are issued is reported beside it
    split3 = (not bf16) and args.outproj_kernel in (0, 4, 5) and (B >= 64 or cfg.H <= 768 or args.outproj_kernel == 4)
    on_mfma = bf16 or split3
    achieved = flops / (k3_ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if on_mfma else PEAK_FP32_TFLOPS
    # few rows (one launch of the weight-streaming kernel: up to 64 rows of a bf16 model with
    # H <= 1216, up to 32 rows of an fp32 model with H <= 768): the launch reads the (padded) output
    # weights once, nothing else of size
    streamed = args.outproj_kernel in (0, 5) and ((bf16 and B <= 64 and cfg.H <= 1216) or
                                                  (not bf16 and B <= 32 and cfg.H <= 768))
    Hp = max(128 if bf16 else 64, -(-cfg.H // 64) * 64)
    kernel_name = m.outproj_kernel_name(cfg.N)      # the library names the kernel it launches
    if kernel_name == "outproj_staged_kernel":
        kernel_name += "<%d, %s>" % (Hp, "true" if args.lse_mode in (0, 2) else "false")
    assert streamed == (kernel_name == "outproj_stream_kernel"), (streamed, kernel_name)
    traffic, traffic_source = TRAFFIC.get((kernel_name, args.config if args.unique_frac is None else -1), (None, None))
    if args.rows is not None and not streamed:
        traffic, traffic_source = None, None
    k3_timing = {"us_per_launch": round(k3_ms * 1e3, 2), "us_per_launch_min": round(k3_groups[0] * 1e3, 2),
                 "us_per_launch_max": round(k3_groups[-1] * 1e3, 2),
                 "timing": "median of 7 groups of %d back-to-back launches between HIP events on the launch stream, "
                           "row count read on the device as in the step" % reps}
    if streamed:
        Vp = -(-cfg.V // 256) * 256
        wbytes = float(Hp) * Vp * (2 if bf16 else 4)
        gbs = wbytes / (k3_ms * 1e-3) / 1e9
        roofline = {"kernel": "%s (weight streaming, %d rows)" % (kernel_name, B), "bound": "hbm",
                    "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": traffic, "traffic_source": traffic_source,
                    "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE, copy-calibrated)",
                    "bytes_per_launch": wbytes, "flop_per_launch": flops}
    else:
        roofline = {"kernel": kernel_name + (" (fp32 as 6 bf16 products)" if split3 else ""),
                    "bound": "mfma" if on_mfma else "alu", "achieved": round(achieved, 2), "peak": peak,
                    "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                    "traffic": traffic, "traffic_source": traffic_source,
                    "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE+WRITE_SIZE, copy-calibrated)",
                    "flop_per_launch": flops}
        if split3:
            roofline["bf16_products_issued_tflops"] = round(6.0 * achieved, 2)
    roofline.update(k3_timing)

    if roofline["bound"] == "mfma" and not args.no_mfma_probe and not args.no_cpu_baseline:
        # context for `frac`: the rate this device sustains on the same loop shape with nothing else
        # to do (one probe launch = 68.7 GFLOP, the size of the headline launch), after the timed region
        probe = {}
        for name, feed, data in (("registers_zeros", 0, 0), ("registers_random", 0, 1),
                                 ("lds_feed_exp_zeros", 1, 0), ("lds_feed_exp_random", 1, 1)):
            tf, ghz = rn.rnnlm_probe_mfma_rate(feed, data, 20)
            probe[name] = {"tflops": round(tf, 1), "core_ghz": round(ghz, 3)}
        roofline["sustained_probe"] = probe
        roofline["frac_of_sustained"] = round(achieved / probe["lds_feed_exp_random"]["tflops"], 4)

    # what a kernel launch costs on this machine whatever the kernel does (empty kernel, back to back between
    # two events): the floor under every small kernel of the step
    launch_floor_us = round(median([rn.rnnlm_time_empty_launch(1000) for _ in range(5)]), 2)

    gemm_ref = None
    if args.gemm_reference and bf16:
        a = (torch.rand((B, H), device=dev) - 0.5).to(torch.bfloat16)
        w = torch.from_numpy(model["O"].T.copy()).to(dev).to(torch.bfloat16)       # [V][H], as the library keeps it
        logits = torch.empty((B, cfg.V), device=dev, dtype=torch.bfloat16)
        for _ in range(5):
            torch.matmul(a, w.t(), out=logits)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            torch.matmul(a, w.t(), out=logits)
        e1.record()
        torch.cuda.synchronize()
        g_ms = e0.elapsed_time(e1) / 20
        gemm_ref = {"what": "torch.matmul bf16 [B,H] x [H,V] -> bf16 logits in HBM (no log-sum-exp)",
                    "us_per_launch": round(g_ms * 1e3, 2), "tflops": round(flops / (g_ms * 1e-3) / 1e12, 1),
                    "logit_bytes_written": B * cfg.V * 2}
        del a, w, logits

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        if cache_info is not None:
            # the buffers hold the last step of the trace: score the first step (the one whose host
            # inputs are at hand) once more, untimed, so that the oracle is compared like with like
            rn.rnnlm_step_dedup(m, keys, prev, h_in, query, rep, inv, nu, h_out, lp, ws)
            torch.cuda.synchronize()
            B = int(nu.item())
        # calibrate on one row per thread, then size the sample to roughly 12 s of wall time
        threads = oracle.max_threads()
        t = time.perf_counter()
        rep_h = rep.cpu().numpy()[:B]
        inv_h = inv.cpu().numpy()
        def oracle_rows(n):                        # the first n distinct histories and their queries
            raw = np.flatnonzero(inv_h < n)
            return raw, oracle.step(model, x["prev"][rep_h[:n]], x["h_in"][rep_h[:n]], x["query"][raw],
                                    row_of_query=inv_h[raw])
        oracle_rows(threads)
        t_round = time.perf_counter() - t
        rows = min(B, threads * max(1, int(round(12.0 / max(t_round, 1e-3)))))
        t = time.perf_counter()
        raw, ref = oracle_rows(rows)
        cdt = time.perf_counter() - t
        err = float(np.max(np.abs(lp.cpu().numpy()[raw] - ref["logprob"])))
        # the same oracle on ONE core: a few rows, sized to about 3 s
        one_rows = min(B, 4)
        t = time.perf_counter()
        raw1 = np.flatnonzero(inv_h < one_rows)
        oracle.step(model, x["prev"][rep_h[:one_rows]], x["h_in"][rep_h[:one_rows]], x["query"][raw1],
                    row_of_query=inv_h[raw1], num_threads=1)
        t_one = time.perf_counter() - t
        more = min(B, max(one_rows, int(one_rows * 3.0 / max(t_one, 1e-3))))
        if more > one_rows:
            one_rows = more
            t = time.perf_counter()
            raw1 = np.flatnonzero(inv_h < one_rows)
            oracle.step(model, x["prev"][rep_h[:one_rows]], x["h_in"][rep_h[:one_rows]], x["query"][raw1],
                        row_of_query=inv_h[raw1], num_threads=1)
            t_one = time.perf_counter() - t
        cpu = {"value": round(rows / cdt, 2), "unit": "hypothesis-steps/s", "cores": threads, "kind": "oracle",
               "sample": "first %d of %d distinct rows of the same step (hidden update + full-vocabulary "
                         "log-sum-exp + their queries), %.1f s wall" % (rows, B, cdt),
               "max_abs_dlogprob_vs_gpu": err,
               "one_core": {"value": round(one_rows / t_one, 2), "unit": "hypothesis-steps/s", "cores": 1,
                            "sample": "first %d distinct rows of the same step, %.1f s wall" % (one_rows, t_one)}}

    out = {
        "metric": "RNNLM hypothesis-steps/sec (V=%d,H=%d,B=%d)" % (cfg.V, cfg.H, cfg.N),
        "value": round(value, 1),
        "unit": "hypothesis-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": "%s%s: V=%d H=%d N=%d raw queries (%d distinct histories) K=%d, %s weights "
                               "N(0,%g), Zipf(%g) word ids (0 = uniform), one step incl. history-id grouping"
                               % (cfg.name, (" (headline)" if args.config == 3 else "") if args.rows is None
                                  else " cut to %d rows" % args.rows, cfg.V, cfg.H, cfg.N, B, cfg.K,
                                  cfg.dtype, cfg.sigma, cfg.zipf_s or 0),
                   "V": cfg.V, "H": cfg.H, "B": B, "N": cfg.N, "K": cfg.K},
        "timing": timing,
        "launch_floor_us": launch_floor_us,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if B != N and cache_info is None:
        # raw queries are the hypothesis-steps (grouping is the method's gain); the rate over the
        # distinct histories that were actually computed, for comparison with the other workloads
        out["distinct_rows_per_s"] = round(B * args.steps / dt, 1)
    if cache_info is not None:
        out["cache"] = cache_info
    if gemm_ref is not None:
        out["gemm_reference"] = gemm_ref
    if graph_info is not None:
        out["graph"] = graph_info
    print(json.dumps(out))
    m.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
