"""CPU oracle (scalar fp64 C) for the batched RNNLM step.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package; the GPU library and its Python binding never do.  The arithmetic lives in
rnnlm_oracle.c (see its header for what is computed and from which passages); this file
compiles it with gcc and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rnnlm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile rnnlm_oracle.c -> liboracle.so (gcc -O2, OpenMP over rows, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        P = ctypes.c_void_p
        I = ctypes.c_int
        lib.oracle_dedup.argtypes = [P, I, P, P]
        lib.oracle_dedup.restype = I
        lib.oracle_step.argtypes = [I, I, I, I, I, P, P, P, P, P, P, P, P, P, P, P, P, I]
        lib.oracle_step.restype = I
        lib.oracle_max_threads.restype = I
        lib.oracle_cache_new.argtypes = [I, I]
        lib.oracle_cache_new.restype = P
        lib.oracle_cache_free.argtypes = [P]
        lib.oracle_cache_free.restype = None
        lib.oracle_cache_reset.argtypes = [P]
        lib.oracle_cache_reset.restype = None
        lib.oracle_cache_stats.argtypes = [P, P]
        lib.oracle_cache_stats.restype = None
        lib.oracle_step_cached.argtypes = [P, I, I, I, I] + [P] * 15 + [I]
        lib.oracle_step_cached.restype = I
        lib.oracle_hs_step_cached.argtypes = [P, I, I, I, I] + [P] * 15
        lib.oracle_hs_step_cached.restype = I
        lib.oracle_pack_ids.argtypes = [P, P, I, P]
        lib.oracle_pack_ids.restype = None
        lib.oracle_huffman_build.argtypes = [I, P, P, P, ctypes.c_longlong]
        lib.oracle_huffman_build.restype = ctypes.c_longlong
        lib.oracle_hs_step.argtypes = [I, I, I, I, I] + [P] * 12 + [I]
        lib.oracle_hs_step.restype = I
        lib.oracle_index_new.argtypes = [I, I]
        lib.oracle_index_new.restype = P
        lib.oracle_index_free.argtypes = [P]
        lib.oracle_index_free.restype = None
        lib.oracle_index_reset.argtypes = [P]
        lib.oracle_index_reset.restype = None
        lib.oracle_index_stats.argtypes = [P, P]
        lib.oracle_index_stats.restype = None
        lib.oracle_index_intern.argtypes = [P, I, P, P, P]
        lib.oracle_index_intern.restype = None
        lib.oracle_index_fetch.argtypes = [P, I, P, P, P]
        lib.oracle_index_fetch.restype = I
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def dedup(keys: np.ndarray):
    """keys u64[N] -> (n_unique, rep i32[n_unique], inverse i32[N]), first-appearance order."""
    keys = _c(keys, np.uint64)
    N = keys.shape[0]
    rep = np.zeros(max(N, 1), dtype=np.int32)
    inverse = np.zeros(max(N, 1), dtype=np.int32)
    U = _load().oracle_dedup(_ptr(keys), N, _ptr(rep), _ptr(inverse))
    return U, rep[:U].copy(), inverse[:N].copy()


def step(model: dict, prev, h_in, query, row_of_query=None, want_full: bool = False,
         num_threads: int = 0) -> dict:
    """One step.  model: dict with float32 U[V,H], W[H,H], O[H,V], bias[V] or None.
    Returns float64 h_out[B,H], lse[B], logprob[N,K] (and full_logp[B,V] if want_full)."""
    U = _c(model["U"], np.float32)
    W = _c(model["W"], np.float32)
    O = _c(model["O"], np.float32)
    bias = model.get("bias")
    bias = None if bias is None else _c(bias, np.float32)
    V, H = U.shape
    assert W.shape == (H, H) and O.shape == (H, V)
    prev = _c(prev, np.int32)
    h_in = _c(h_in, np.float32)
    query = _c(query, np.int32)
    B = prev.shape[0]
    N, K = query.shape
    assert h_in.shape == (B, H)
    if row_of_query is not None:
        row_of_query = _c(row_of_query, np.int32)
        assert row_of_query.shape == (N,)
    else:
        assert N == B
    h_out = np.zeros((B, H), dtype=np.float64)
    lse = np.zeros(B, dtype=np.float64)
    logprob = np.zeros((N, K), dtype=np.float64)
    full = np.zeros((B, V), dtype=np.float64) if want_full else None
    rc = _load().oracle_step(V, H, B, K, N, _ptr(U), _ptr(W), _ptr(O), _ptr(bias),
                             _ptr(prev), _ptr(h_in), _ptr(query), _ptr(row_of_query),
                             _ptr(h_out), _ptr(lse), _ptr(logprob), _ptr(full), num_threads)
    if rc != 0:
        raise ValueError("oracle_step: index out of range" if rc == -1 else "oracle_step: out of memory")
    out = {"h_out": h_out, "lse": lse, "logprob": logprob}
    if want_full:
        out["full_logp"] = full
    return out


class Cache:
    """The cache of RnnlmProb kept between steps (Table 1; Sections 4.2 and 5.3): at most
    `capacity` histories, nothing is ever removed; reset() starts a new utterance."""

    def __init__(self, H: int, capacity: int):
        self._h = _load().oracle_cache_new(int(H), int(capacity))
        if not self._h:
            raise MemoryError("oracle_cache_new failed")
        self.H, self.capacity = int(H), int(capacity)

    def reset(self) -> None:
        _load().oracle_cache_reset(self._h)

    def stats(self) -> dict:
        out = np.zeros(5, dtype=np.int64)
        _load().oracle_cache_stats(self._h, _ptr(out))
        return dict(zip(("entries", "lookups", "hits", "misses", "unstored"), (int(x) for x in out)))

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.oracle_cache_free(self._h)
            self._h = None


def step_cached(model: dict, cache: Optional[Cache], ids, prev, h_in, query, base_score=None,
                num_threads: int = 0) -> dict:
    """One step over N raw queries through the cache (None: no cache outlives the step).
    Returns n_unique, rep, inverse, float64 h_out[n_unique,H], lse[n_unique], score[N,K]
    (log-probability minus base_score) and stats = (distinct, hits, computed, entries)."""
    U = _c(model["U"], np.float32)
    W = _c(model["W"], np.float32)
    O = _c(model["O"], np.float32)
    bias = model.get("bias")
    bias = None if bias is None else _c(bias, np.float32)
    V, H = U.shape
    ids = _c(ids, np.uint64)
    prev = _c(prev, np.int32)
    h_in = _c(h_in, np.float32)
    query = _c(query, np.int32)
    N, K = query.shape
    assert ids.shape == (N,) and prev.shape == (N,) and h_in.shape == (N, H)
    if base_score is not None:
        base_score = _c(base_score, np.float32)
        assert base_score.shape == (N, K)
    n1 = max(N, 1)
    rep = np.zeros(n1, dtype=np.int32)
    inverse = np.zeros(n1, dtype=np.int32)
    h_out = np.zeros((n1, H), dtype=np.float64)
    lse = np.zeros(n1, dtype=np.float64)
    score = np.zeros((N, K), dtype=np.float64)
    stats = np.zeros(4, dtype=np.int32)
    rc = _load().oracle_step_cached(cache._h if cache is not None else None, V, H, N, K,
                                    _ptr(U), _ptr(W), _ptr(O), _ptr(bias), _ptr(ids), _ptr(prev),
                                    _ptr(h_in), _ptr(query), _ptr(base_score), _ptr(rep), _ptr(inverse),
                                    _ptr(h_out), _ptr(lse), _ptr(score), _ptr(stats), num_threads)
    if rc < 0:
        raise ValueError("oracle_step_cached failed (%d)" % rc)
    return {"n_unique": rc, "rep": rep[:rc].copy(), "inverse": inverse[:N].copy(),
            "h_out": h_out[:rc].copy(), "lse": lse[:rc].copy(), "score": score,
            "stats": tuple(int(x) for x in stats)}


def hs_step_cached(model: dict, cache: Optional[Cache], ids, prev, h_in, query, base_score=None) -> dict:
    """step_cached for a model with the hierarchical output layer (model as in hs_step): returns
    n_unique, rep, inverse, float64 h_out[n_unique,H], score[N,K] and stats = (distinct, hits,
    computed, entries)."""
    U = _c(model["U"], np.float32)
    W = _c(model["W"], np.float32)
    theta = _c(model["theta"], np.float32)
    off = _c(model["path_off"], np.int32)
    entry = _c(model["path_entry"], np.int32)
    V, H = U.shape
    assert W.shape == (H, H) and theta.shape == (V - 1, H) and off.shape == (V + 1,)
    ids = _c(ids, np.uint64)
    prev = _c(prev, np.int32)
    h_in = _c(h_in, np.float32)
    query = _c(query, np.int32)
    N, K = query.shape
    assert ids.shape == (N,) and prev.shape == (N,) and h_in.shape == (N, H)
    if base_score is not None:
        base_score = _c(base_score, np.float32)
        assert base_score.shape == (N, K)
    n1 = max(N, 1)
    rep = np.zeros(n1, dtype=np.int32)
    inverse = np.zeros(n1, dtype=np.int32)
    h_out = np.zeros((n1, H), dtype=np.float64)
    score = np.zeros((N, K), dtype=np.float64)
    stats = np.zeros(4, dtype=np.int32)
    rc = _load().oracle_hs_step_cached(cache._h if cache is not None else None, V, H, N, K, _ptr(U), _ptr(W),
                                       _ptr(theta), _ptr(off), _ptr(entry), _ptr(ids), _ptr(prev), _ptr(h_in),
                                       _ptr(query), _ptr(base_score), _ptr(rep), _ptr(inverse), _ptr(h_out),
                                       _ptr(score), _ptr(stats))
    if rc < 0:
        raise ValueError("oracle_hs_step_cached failed (%d)" % rc)
    return {"n_unique": rc, "rep": rep[:rc].copy(), "inverse": inverse[:N].copy(), "h_out": h_out[:rc].copy(),
            "score": score, "stats": tuple(int(x) for x in stats)}


def pack_ids(ctx, small_lm) -> np.ndarray:
    """The packed 8-byte history index of Section 3.2 (context index in the high half)."""
    ctx = _c(ctx, np.uint32)
    small_lm = _c(small_lm, np.uint32)
    assert ctx.shape == small_lm.shape and ctx.ndim == 1
    out = np.zeros(ctx.shape[0], dtype=np.uint64)
    _load().oracle_pack_ids(_ptr(ctx), _ptr(small_lm), ctx.shape[0], _ptr(out))
    return out


class IndexTable:
    """IndexTable and its inverse (Section 3.2; Table 1 steps 5, 7-12): contexts (word, hidden
    vector) stored once, found again by content (all bits), numbered in order of storage."""
    NOT_STORED = 0xFFFFFFFF

    def __init__(self, H: int, capacity: int):
        self._h = _load().oracle_index_new(int(H), int(capacity))
        if not self._h:
            raise MemoryError("oracle_index_new failed")
        self.H, self.capacity = int(H), int(capacity)

    def reset(self) -> None:
        _load().oracle_index_reset(self._h)

    def stats(self) -> dict:
        out = np.zeros(4, dtype=np.int64)
        _load().oracle_index_stats(self._h, _ptr(out))
        return dict(zip(("entries", "lookups", "found", "unstored"), (int(x) for x in out)))

    def intern(self, word, h) -> np.ndarray:
        word = _c(word, np.int32)
        h = _c(h, np.float32)
        N = word.shape[0]
        assert h.shape == (N, self.H)
        out = np.zeros(N, dtype=np.uint32)
        _load().oracle_index_intern(self._h, N, _ptr(word), _ptr(h), _ptr(out))
        return out

    def fetch(self, index):
        index = _c(index, np.uint32)
        N = index.shape[0]
        word = np.zeros(N, dtype=np.int32)
        h = np.zeros((N, self.H), dtype=np.float32)
        if _load().oracle_index_fetch(self._h, N, _ptr(index), _ptr(word), _ptr(h)) != 0:
            raise ValueError("oracle_index_fetch: index not held")
        return word, h

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.oracle_index_free(self._h)
            self._h = None


def huffman_build(freq):
    """Huffman tree over the words (Section 2.1) from their frequencies: returns path_off i32[V+1]
    and path_entry i32[total], the path of word v from the root down being
    path_entry[path_off[v]:path_off[v+1]], each entry = inner node id | code bit << 31."""
    freq = _c(freq, np.float64)
    V = freq.shape[0]
    off = np.zeros(V + 1, dtype=np.int32)
    cap = 64 * V
    entry = np.zeros(cap, dtype=np.int32)
    total = _load().oracle_huffman_build(V, _ptr(freq), _ptr(off), _ptr(entry), cap)
    if total < -1:
        cap = -total - 1
        entry = np.zeros(cap, dtype=np.int32)
        total = _load().oracle_huffman_build(V, _ptr(freq), _ptr(off), _ptr(entry), cap)
    if total < 0:
        raise ValueError("oracle_huffman_build failed")
    return off, entry[:total].copy()


def hs_step(model: dict, prev, h_in, query, row_of_query=None, want_full: bool = False,
            num_threads: int = 0) -> dict:
    """One step with the hierarchical output layer.  model: float32 U[V,H], W[H,H], theta[V-1,H],
    int32 path_off[V+1], path_entry[...].  Returns float64 h_out[B,H], logprob[N,K]."""
    U = _c(model["U"], np.float32)
    W = _c(model["W"], np.float32)
    theta = _c(model["theta"], np.float32)
    off = _c(model["path_off"], np.int32)
    entry = _c(model["path_entry"], np.int32)
    V, H = U.shape
    assert W.shape == (H, H) and theta.shape == (V - 1, H) and off.shape == (V + 1,)
    prev = _c(prev, np.int32)
    h_in = _c(h_in, np.float32)
    query = _c(query, np.int32)
    B = prev.shape[0]
    N, K = query.shape
    if row_of_query is not None:
        row_of_query = _c(row_of_query, np.int32)
    else:
        assert N == B
    h_out = np.zeros((B, H), dtype=np.float64)
    logprob = np.zeros((N, K), dtype=np.float64)
    full = np.zeros((B, V), dtype=np.float64) if want_full else None
    rc = _load().oracle_hs_step(V, H, B, K, N, _ptr(U), _ptr(W), _ptr(theta), _ptr(off), _ptr(entry),
                                _ptr(prev), _ptr(h_in), _ptr(query), _ptr(row_of_query), _ptr(h_out),
                                _ptr(logprob), _ptr(full), num_threads)
    if rc != 0:
        raise ValueError("oracle_hs_step: index out of range")
    out = {"h_out": h_out, "logprob": logprob}
    if want_full:
        out["full_logp"] = full
    return out
