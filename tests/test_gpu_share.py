"""One loaded model, several handles (rnnlm_model_share): every handle has scratch of its own, so
steps may run on different streams at the same time; the weights live until the last handle is
released.  Also the overlap check on h_in / h_out."""
import numpy as np
import pytest
import torch

import oracle
import paper_2007_11794_amd as rn
from workloads import CONFIGS, make_model, make_step_inputs

from harness import DEV, gpu_step, load_model

pytestmark = pytest.mark.gpu


def device_inputs(x):
    return (torch.from_numpy(x["prev"]).to(DEV), torch.from_numpy(x["h_in"]).to(DEV), torch.from_numpy(x["query"]).to(DEV))


@pytest.mark.parametrize("dtype,V,H,B,K", [("bf16", 6000, 512, 300, 6), ("f32", 3000, 128, 100, 4), ("bf16", 2500, 640, 40, 3)])
def test_shared_handles_on_two_streams_match_the_oracle(dtype, V, H, B, K):
    cfg = CONFIGS[3 if dtype == "bf16" else 2].scaled(V=V, H=H, B=B, K=K)
    model = make_model(cfg)
    base = load_model(model, dtype, B)
    other = base.share(B)
    xs = [make_step_inputs(cfg, np.random.default_rng(cfg.seed + i)) for i in range(2)]
    refs = [oracle.step(model, x["prev"], x["h_in"], x["query"]) for x in xs]
    ins = [device_inputs(x) for x in xs]
    outs = [(torch.full((B, H), float("nan"), device=DEV), torch.full((B, K), float("nan"), device=DEV)) for _ in xs]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(20):                     # interleaved launches: the two handles' kernels overlap in time
        for handle, stream, i, o in zip((base, other), streams, ins, outs):
            rn.rnnlm_step(handle, i[0], i[1], i[2], o[0], o[1], stream=stream.cuda_stream)
    torch.cuda.synchronize()
    tol_lp, tol_h = (2e-3, 1e-3) if dtype == "bf16" else (1e-5, 1e-5)
    for o, ref in zip(outs, refs):
        assert np.max(np.abs(o[0].cpu().numpy() - ref["h_out"])) <= tol_h
        assert np.max(np.abs(o[1].cpu().numpy() - ref["logprob"])) <= tol_lp
    assert base.last_error() == 0 and other.last_error() == 0
    # the weights outlive the handle that loaded them
    base.close()
    h, lp = gpu_step(other, xs[0]["prev"], xs[0]["h_in"], xs[0]["query"])
    assert np.array_equal(h, outs[0][0].cpu().numpy()) and np.array_equal(lp, outs[0][1].cpu().numpy())
    third = other.share(7)                    # a share of a share, smaller batches
    h3, lp3 = gpu_step(third, xs[1]["prev"][:7], xs[1]["h_in"][:7], xs[1]["query"][:7])
    assert np.max(np.abs(h3 - refs[1]["h_out"][:7])) <= tol_h and np.max(np.abs(lp3 - refs[1]["logprob"][:7])) <= tol_lp
    with pytest.raises(rn.RnnlmError) as e:   # its own max_B
        gpu_step(third, xs[1]["prev"][:8], xs[1]["h_in"][:8], xs[1]["query"][:8])
    assert e.value.status == -4
    other.close()
    third.close()


def test_options_and_flags_belong_to_the_handle():
    cfg = CONFIGS[3].scaled(V=900, H=64, B=16, K=3)
    model = make_model(cfg)
    x = make_step_inputs(cfg, np.random.default_rng(5))
    base = load_model(model, "bf16", 16)
    base.set_option(rn.OPT_LSE_MODE, 1)
    other = base.share(16)                    # starts as a copy of the options
    other.set_option(rn.OPT_OUTPROJ_KERNEL, 1)
    prev = x["prev"].copy(); prev[2] = cfg.V
    gpu_step(other, prev, x["h_in"], x["query"])
    assert base.last_error() == 0 and other.last_error() == rn.FLAG_BAD_PREV_WORD
    ref = oracle.step(model, x["prev"], x["h_in"], x["query"])
    for handle in (base, other):
        h, lp = gpu_step(handle, x["prev"], x["h_in"], x["query"])
        assert np.max(np.abs(lp - ref["logprob"])) <= 2e-3 and np.max(np.abs(h - ref["h_out"])) <= 1e-3
    other.close()
    base.close()


def test_overlapping_hidden_blocks_are_refused():
    cfg = CONFIGS[3].scaled(V=500, H=64, B=8, K=2)
    m = load_model(make_model(cfg), "bf16", 8)
    buf = torch.zeros(3 * 8 * 64, device=DEV)
    prev = torch.zeros(8, dtype=torch.int32, device=DEV)
    q = torch.zeros((8, 2), dtype=torch.int32, device=DEV)
    lp = torch.zeros((8, 2), device=DEV)
    h_in = buf[: 8 * 64].view(8, 64)
    for shift in (0, 64, 7 * 64 + 60):        # same block, one row apart, the last four floats shared
        h_out = buf[shift: shift + 8 * 64].view(8, 64)
        with pytest.raises(rn.RnnlmError) as e:
            rn.rnnlm_step(m, prev, h_in, q, h_out, lp)
        assert e.value.status == -1
    rn.rnnlm_step(m, prev, h_in, q, buf[8 * 64: 16 * 64].view(8, 64), lp)      # back to back is fine
    torch.cuda.synchronize()
    m.close()
