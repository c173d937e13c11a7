"""The five seeded workloads and their generators (random draws and gathers only)."""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    """Shape and distribution of one synthetic workload.

    V vocabulary size, H hidden units, B rows (unique histories) per step, K query
    words per raw query, N raw queries per step (N == B when nothing repeats).
    """
    name: str
    V: int
    H: int
    B: int
    K: int
    N: int
    dtype: str                 # "f32" or "bf16": storage type of U, W, O
    sigma: float               # weights ~ N(0, sigma^2)
    zipf_s: Optional[float]    # None: uniform word ids; else bounded Zipf exponent
    h_in: str                  # "uniform" or "sigmoid_normal"
    steps: int
    unique_frac: Optional[float] = None   # fraction of distinct histories (decode trace)
    seed: int = 0

    def scaled(self, **kw) -> "Workload":
        """Same recipe at other sizes (used by tests that need a smaller case)."""
        w = dataclasses.replace(self, **kw)
        if "B" in kw and "N" not in kw and self.unique_frac is None:
            w = dataclasses.replace(w, N=w.B)
        return w


CONFIGS: Dict[int, Workload] = {
    1: Workload("tiny", V=1000, H=64, B=8, K=4, N=8, dtype="f32", sigma=0.1,
                zipf_s=None, h_in="uniform", steps=1, seed=1001),
    2: Workload("wsj_sized", V=20000, H=256, B=256, K=16, N=256, dtype="f32", sigma=0.05,
                zipf_s=1.1, h_in="sigmoid_normal", steps=20, seed=1002),
    3: Workload("large_vocab", V=65536, H=512, B=1024, K=32, N=1024, dtype="bf16", sigma=0.03,
                zipf_s=1.1, h_in="sigmoid_normal", steps=1, seed=1003),
    4: Workload("decode_trace", V=65536, H=512, B=1229, K=8, N=4096, dtype="bf16", sigma=0.03,
                zipf_s=1.1, h_in="sigmoid_normal", steps=50, unique_frac=0.3, seed=1004),
    5: Workload("stress", V=200000, H=1024, B=2048, K=64, N=2048, dtype="bf16", sigma=0.02,
                zipf_s=1.0, h_in="sigmoid_normal", steps=1, seed=1005),
    # Not one of the five given workloads: the regime the paper itself runs in (Section 5.1: about a
    # million words, a hidden layer of 100 units -- 128 here, the next size the matrix cores like) with the
    # few distinct histories per step that its cache leaves (Section 5.2).  Used to set the hierarchical
    # output layer of Section 2.1 beside the full softmax where the former is meant to win.
    6: Workload("paper_regime", V=1000000, H=128, B=64, K=32, N=64, dtype="bf16", sigma=0.05,
                zipf_s=1.1, h_in="sigmoid_normal", steps=1, seed=1006),
}


# --------------------------------------------------------------------------- bf16 helpers
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of float32 values that are already exact in bfloat16."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    if np.any(bits & 0xFFFF):
        raise ValueError("values are not exactly representable in bfloat16")
    return (bits >> 16).astype(np.uint16).reshape(x.shape)


def pack_history_id(ctx_index: np.ndarray, small_lm_index: np.ndarray) -> np.ndarray:
    """One 64-bit value from two 32-bit indices, context index in the high half
    (Section 3.2: the RNNLM context index and the small-LM index travel as one number)."""
    return (np.asarray(ctx_index, dtype=np.uint64) << np.uint64(32)) | \
        np.asarray(small_lm_index, dtype=np.uint64)


# --------------------------------------------------------------------------- draws
def bounded_zipf_ids(rng: np.random.Generator, V: int, s: float, size) -> np.ndarray:
    """Word ids with p(rank r) proportional to r^-s for r = 1..V; id = r - 1.
    Sampled by inverting the explicit cumulative mass (works for s = 1.0 too)."""
    pmf = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(pmf)
    cdf /= cdf[-1]
    u = rng.random(size)
    ids = np.searchsorted(cdf, u, side="right")
    return np.minimum(ids, V - 1).astype(np.int32)


def _word_ids(cfg: Workload, rng, size) -> np.ndarray:
    if cfg.zipf_s is None:
        return rng.integers(0, cfg.V, size=size, dtype=np.int64).astype(np.int32)
    return bounded_zipf_ids(rng, cfg.V, cfg.zipf_s, size)


def _hidden(cfg: Workload, rng, rows: int) -> np.ndarray:
    if cfg.h_in == "uniform":
        return rng.random((rows, cfg.H)).astype(np.float32)
    x = rng.standard_normal((rows, cfg.H))
    return (1.0 / (1.0 + np.exp(-x))).astype(np.float32)   # values in (0,1), like a previous h'


def make_model(cfg: Workload, seed: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Random-init weights: U[V,H], W[H,H] (W[j,i] multiplies h[i]), O[H,V], bias[V] = 0.
    float32 arrays; for dtype "bf16" every value is exactly representable in bfloat16."""
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    out = {}
    for name, shape in (("U", (cfg.V, cfg.H)), ("W", (cfg.H, cfg.H)), ("O", (cfg.H, cfg.V))):
        a = rng.standard_normal(shape, dtype=np.float32)
        a *= np.float32(cfg.sigma)
        out[name] = round_to_bf16(a) if cfg.dtype == "bf16" else a
    out["bias"] = np.zeros(cfg.V, dtype=np.float32)
    return out


def make_step_inputs(cfg: Workload, rng: np.random.Generator) -> Dict[str, np.ndarray]:
    """One step without repeated histories: N == B rows, each with its own id.
    keys[N] u64, prev[B] i32, h_in[B,H] f32, query[N,K] i32."""
    B, K = cfg.B, cfg.K
    if cfg.zipf_s is None and B <= cfg.V:
        prev = rng.permutation(cfg.V)[:B].astype(np.int32)       # all distinct (tiny case)
    else:
        prev = _word_ids(cfg, rng, B)
    keys = pack_history_id(rng.permutation(max(B, 1) * 4)[:B],
                           rng.integers(0, 2 ** 32, size=B, dtype=np.uint64))
    return {
        "keys": keys.astype(np.uint64),
        "prev": prev,
        "h_in": _hidden(cfg, rng, B),
        "query": _word_ids(cfg, rng, (B, K)),
    }


class DecodeTrace:
    """A sequence of steps whose raw queries repeat histories (config 4).

    Each step has U0 = round(unique_frac * N) distinct histories.  Rows 0..U0-1 of the
    pre-shuffle order are the distinct ones; every other row copies (id, prev word, h) of
    a uniformly chosen distinct history; all N rows are then permuted.  From one step to
    the next a seeded half of the distinct histories is carried over unchanged (same id,
    same prev word, same h), so the same id seen in two steps must score identically; the
    other half are new contexts grown from a uniformly chosen raw row n of the step
    before: h_in = that row's updated hidden vector, prev word = its first query word.
    The caller supplies the updated hidden vectors (its own side's), so this class
    never computes anything of the method.
    """

    def __init__(self, cfg: Workload, seed: Optional[int] = None, carry_frac: float = 0.5):
        """carry_frac: expected share of the distinct histories kept from one step to the next
        (one half in the workload as specified; the paper's search finds about nine lookups in
        ten again, Section 5.2)."""
        assert cfg.unique_frac is not None and 0.0 <= carry_frac <= 1.0
        self.cfg = cfg
        self.carry_frac = carry_frac
        self.rng = np.random.default_rng(cfg.seed if seed is None else seed)
        self.U0 = int(round(cfg.unique_frac * cfg.N))
        self._ctx_counter = 0
        self._uniq = None        # dict of the distinct histories of the latest step

    def _fresh_ids(self, n: int) -> np.ndarray:
        ctx = np.arange(self._ctx_counter, self._ctx_counter + n, dtype=np.uint64)
        self._ctx_counter += n
        return pack_history_id(ctx, self.rng.integers(0, 2 ** 32, size=n, dtype=np.uint64))

    def _expand(self, uniq: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
        cfg, rng, U0, N = self.cfg, self.rng, self.U0, self.cfg.N
        src = np.concatenate([np.arange(U0), rng.integers(0, U0, size=N - U0)])
        src = src[rng.permutation(N)]
        self._uniq = uniq
        return {
            "keys": uniq["ids"][src],
            "prev": uniq["prev"][src],
            "h_in": uniq["h"][src],
            "query": _word_ids(cfg, rng, (N, cfg.K)),
            "src_unique": src.astype(np.int32),      # which distinct history each row copies
            "carried": uniq["carried"],              # per distinct history: kept from last step
        }

    def first(self) -> Dict[str, np.ndarray]:
        U0 = self.U0
        uniq = {"ids": self._fresh_ids(U0), "prev": _word_ids(self.cfg, self.rng, U0),
                "h": _hidden(self.cfg, self.rng, U0), "carried": np.zeros(U0, dtype=bool)}
        return self._expand(uniq)

    def next(self, last_inputs: Dict[str, np.ndarray], h_out: np.ndarray,
             inverse: np.ndarray) -> Dict[str, np.ndarray]:
        """last_inputs: what first()/next() returned for the step before; h_out[U,H]: that
        step's updated hidden vectors, one per distinct history; inverse[N]: raw row -> row
        of h_out."""
        rng, U0, N = self.rng, self.U0, self.cfg.N
        old = self._uniq
        carried = rng.random(U0) < self.carry_frac
        grow_from = rng.integers(0, N, size=U0)
        new_ids = self._fresh_ids(U0)
        h_new = np.asarray(h_out, dtype=np.float32)[np.asarray(inverse)[grow_from]]
        uniq = {
            "ids": np.where(carried, old["ids"], new_ids),
            "prev": np.where(carried, old["prev"], last_inputs["query"][grow_from, 0]).astype(np.int32),
            "h": np.where(carried[:, None], old["h"], h_new).astype(np.float32),
            "carried": carried,
        }
        return self._expand(uniq)
