"""Shared helpers for the GPU tests: upload a workload, call the library through its
binding, bring results back as numpy.  No arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2007_11794_amd as rn
from workloads import bf16_bits

DEV = "cuda:0"


def load_model(model: dict, dtype: str, max_B: int) -> rn.RnnlmModel:
    V, H = model["U"].shape
    if dtype == "bf16":
        U, W, O = (bf16_bits(model[k]) for k in ("U", "W", "O"))
        code = rn.RNNLM_BF16
    else:
        U, W, O = (np.ascontiguousarray(model[k], np.float32) for k in ("U", "W", "O"))
        code = rn.RNNLM_F32
    return rn.rnnlm_load(V, H, code, U, W, O, model.get("bias"), max_B)


def keys_tensor(keys: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(keys, np.uint64).view(np.int64)).to(DEV)


def gpu_step(m: rn.RnnlmModel, prev, h_in, query, row_of_query=None):
    prev_t = torch.from_numpy(np.ascontiguousarray(prev, np.int32)).to(DEV)
    h_t = torch.from_numpy(np.ascontiguousarray(h_in, np.float32)).to(DEV)
    q_t = torch.from_numpy(np.ascontiguousarray(query, np.int32)).to(DEV)
    B, (N, K) = prev_t.shape[0], q_t.shape
    roq_t = None if row_of_query is None else torch.from_numpy(np.ascontiguousarray(row_of_query, np.int32)).to(DEV)
    h_out = torch.full((B, m.H), float("nan"), device=DEV, dtype=torch.float32)
    lp = torch.full((N, K), float("nan"), device=DEV, dtype=torch.float32)
    rn.rnnlm_step(m, prev_t, h_t, q_t, h_out, lp, row_of_query=roq_t)
    torch.cuda.synchronize()
    return h_out.cpu().numpy(), lp.cpu().numpy()


def gpu_dedup(keys: np.ndarray):
    N = len(keys)
    k_t = keys_tensor(keys) if N else torch.zeros(0, dtype=torch.int64, device=DEV)
    rep = torch.full((N,), -1, device=DEV, dtype=torch.int32)
    inv = torch.full((N,), -1, device=DEV, dtype=torch.int32)
    nu = torch.full((1,), -1, device=DEV, dtype=torch.int32)
    ws = torch.empty(max(rn.rnnlm_dedup_workspace_bytes(N), 16), device=DEV, dtype=torch.uint8)
    rn.rnnlm_dedup(k_t, rep, inv, nu, ws)
    torch.cuda.synchronize()
    U = int(nu.item())
    return U, rep.cpu().numpy()[:U], inv.cpu().numpy()


def gpu_step_dedup(m: rn.RnnlmModel, keys, prev, h_in, query):
    N, K = query.shape
    k_t = keys_tensor(keys)
    prev_t = torch.from_numpy(np.ascontiguousarray(prev, np.int32)).to(DEV)
    h_t = torch.from_numpy(np.ascontiguousarray(h_in, np.float32)).to(DEV)
    q_t = torch.from_numpy(np.ascontiguousarray(query, np.int32)).to(DEV)
    rep = torch.full((N,), -1, device=DEV, dtype=torch.int32)
    inv = torch.full((N,), -1, device=DEV, dtype=torch.int32)
    nu = torch.full((1,), -1, device=DEV, dtype=torch.int32)
    ws = torch.empty(max(rn.rnnlm_dedup_workspace_bytes(N), 16), device=DEV, dtype=torch.uint8)
    h_out = torch.full((N, m.H), float("nan"), device=DEV, dtype=torch.float32)
    lp = torch.full((N, K), float("nan"), device=DEV, dtype=torch.float32)
    rn.rnnlm_step_dedup(m, k_t, prev_t, h_t, q_t, rep, inv, nu, h_out, lp, ws)
    torch.cuda.synchronize()
    U = int(nu.item())
    return {"n_unique": U, "rep": rep.cpu().numpy()[:U], "inverse": inv.cpu().numpy(),
            "h_out": h_out.cpu().numpy()[:U], "h_out_rest": h_out.cpu().numpy()[U:],
            "logprob": lp.cpu().numpy()}


class CachedStepper:
    """Device buffers for repeated rnnlm_step_cached calls of up to N raw queries."""

    def __init__(self, m: rn.RnnlmModel, cache, N: int, K: int):
        self.m, self.cache, self.N, self.K = m, cache, N, K
        self.ws = torch.empty(max(rn.rnnlm_dedup_workspace_bytes(N), 16), device=DEV, dtype=torch.uint8)

    def step(self, keys, prev, h_in, query, base_score=None):
        N, K = query.shape
        k_t = keys_tensor(keys) if N else torch.zeros(0, dtype=torch.int64, device=DEV)
        prev_t = torch.from_numpy(np.ascontiguousarray(prev, np.int32)).to(DEV)
        h_t = torch.from_numpy(np.ascontiguousarray(h_in, np.float32)).to(DEV)
        q_t = torch.from_numpy(np.ascontiguousarray(query, np.int32)).to(DEV)
        b_t = None if base_score is None else torch.from_numpy(np.ascontiguousarray(base_score, np.float32)).to(DEV)
        rep = torch.full((N,), -1, device=DEV, dtype=torch.int32)
        inv = torch.full((N,), -1, device=DEV, dtype=torch.int32)
        nu = torch.full((1,), -1, device=DEV, dtype=torch.int32)
        stats = torch.full((4,), -1, device=DEV, dtype=torch.int32)
        h_out = torch.full((N, self.m.H), float("nan"), device=DEV, dtype=torch.float32)
        score = torch.full((N, K), float("nan"), device=DEV, dtype=torch.float32)
        rn.rnnlm_step_cached(self.m, self.cache, k_t, prev_t, h_t, q_t, rep, inv, nu, h_out, score, self.ws,
                             base_score=b_t, step_stats=stats)
        torch.cuda.synchronize()
        U = int(nu.item())
        return {"n_unique": U, "rep": rep.cpu().numpy()[:U], "inverse": inv.cpu().numpy(),
                "h_out": h_out.cpu().numpy()[:U], "h_out_rest": h_out.cpu().numpy()[U:],
                "score": score.cpu().numpy(), "stats": tuple(int(v) for v in stats.cpu().numpy())}
