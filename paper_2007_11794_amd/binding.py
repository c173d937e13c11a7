"""ctypes binding of librnnlm.so: argument marshalling only.

Every function mirrors the C entry point of the same name (include/rnnlm.h).  Device
buffers are torch tensors (their data_ptr() is passed through); the stream is torch's
current stream unless one is given.  If the library has not been built this module raises
at import of the symbol table -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

RNNLM_F32, RNNLM_BF16 = 0, 1
FLAG_BAD_PREV_WORD, FLAG_BAD_QUERY_WORD, FLAG_BAD_ROW = 1, 2, 4
OPT_LSE_MODE, OPT_OUTPROJ_KERNEL = 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librnnlm.so")
_lib = None

EXPORTS = ["rnnlm_strerror", "rnnlm_load", "rnnlm_free", "rnnlm_model_share", "rnnlm_set_option", "rnnlm_last_error",
           "rnnlm_dedup_workspace_bytes", "rnnlm_dedup", "rnnlm_dedup_static", "rnnlm_step", "rnnlm_step_dedup",
           "rnnlm_time_outproj", "rnnlm_cache_create", "rnnlm_cache_free", "rnnlm_cache_reset",
           "rnnlm_cache_stats", "rnnlm_step_cached", "rnnlm_pack_ids", "rnnlm_index_create",
           "rnnlm_index_free", "rnnlm_index_reset", "rnnlm_index_intern", "rnnlm_index_fetch",
           "rnnlm_index_stats", "rnnlm_huffman_build", "rnnlm_hs_load", "rnnlm_hs_step", "rnnlm_hs_time_query",
           "rnnlm_probe_mfma_rate", "rnnlm_time_empty_launch", "rnnlm_outproj_kernel_name"]


class RnnlmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, rnnlm_strerror(status), status))


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Load librnnlm.so (built in-tree by paper_2007_11794_amd.build); raise if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("librnnlm.so is not built: run `python -m paper_2007_11794_amd.build` "
                              "(or __graft_entry__.build()); there is no fallback implementation")
        L = ctypes.CDLL(_LIB_PATH)
        P, I, Z = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.rnnlm_strerror.argtypes = [I]
        L.rnnlm_strerror.restype = ctypes.c_char_p
        L.rnnlm_load.argtypes = [I, I, I, P, P, P, P, I, ctypes.POINTER(P)]
        L.rnnlm_load.restype = I
        L.rnnlm_free.argtypes = [P]
        L.rnnlm_free.restype = I
        L.rnnlm_set_option.argtypes = [P, I, I]
        L.rnnlm_set_option.restype = I
        L.rnnlm_last_error.argtypes = [P, P, ctypes.POINTER(I)]
        L.rnnlm_last_error.restype = I
        L.rnnlm_dedup_workspace_bytes.argtypes = [I]
        L.rnnlm_dedup_workspace_bytes.restype = Z
        L.rnnlm_dedup.argtypes = [P, I, P, P, P, P, Z, P]
        L.rnnlm_dedup.restype = I
        L.rnnlm_dedup_static.argtypes = [P, I, P, P, P, P]
        L.rnnlm_dedup_static.restype = I
        L.rnnlm_step.argtypes = [P, I, I, P, P, P, P, I, P, P, P]
        L.rnnlm_step.restype = I
        L.rnnlm_step_dedup.argtypes = [P, I, I, P, P, P, P, P, P, P, P, P, P, Z, P]
        L.rnnlm_step_dedup.restype = I
        L.rnnlm_model_share.argtypes = [P, I, ctypes.POINTER(P)]
        L.rnnlm_model_share.restype = I
        L.rnnlm_time_outproj.argtypes = [P, I, P, I, P, ctypes.POINTER(ctypes.c_float)]
        L.rnnlm_time_outproj.restype = I
        L.rnnlm_time_empty_launch.argtypes = [I, P, ctypes.POINTER(ctypes.c_float)]
        L.rnnlm_time_empty_launch.restype = I
        L.rnnlm_outproj_kernel_name.argtypes = [P, I]
        L.rnnlm_outproj_kernel_name.restype = ctypes.c_char_p
        L.rnnlm_probe_mfma_rate.argtypes = [I, I, I, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.rnnlm_probe_mfma_rate.restype = I
        L.rnnlm_cache_create.argtypes = [P, I, ctypes.POINTER(P)]
        L.rnnlm_cache_create.restype = I
        L.rnnlm_cache_free.argtypes = [P]
        L.rnnlm_cache_free.restype = I
        L.rnnlm_cache_reset.argtypes = [P, P]
        L.rnnlm_cache_reset.restype = I
        L.rnnlm_cache_stats.argtypes = [P, P, ctypes.POINTER(ctypes.c_int64)]
        L.rnnlm_cache_stats.restype = I
        L.rnnlm_step_cached.argtypes = [P, P, I, I, P, P, P, P, P, P, P, P, P, P, P, P, Z, P]
        L.rnnlm_step_cached.restype = I
        L.rnnlm_pack_ids.argtypes = [P, P, I, P, P]
        L.rnnlm_pack_ids.restype = I
        L.rnnlm_huffman_build.argtypes = [I, P, P, P, Z, ctypes.POINTER(Z)]
        L.rnnlm_huffman_build.restype = I
        L.rnnlm_hs_load.argtypes = [I, I, I, P, P, P, P, P, I, ctypes.POINTER(P)]
        L.rnnlm_hs_load.restype = I
        L.rnnlm_hs_step.argtypes = [P, I, I, P, P, P, P, I, P, P, P, P]
        L.rnnlm_hs_step.restype = I
        L.rnnlm_hs_time_query.argtypes = [P, I, I, P, P, I, P, P, I, P, ctypes.POINTER(ctypes.c_float)]
        L.rnnlm_hs_time_query.restype = I
        L.rnnlm_index_create.argtypes = [I, I, I, ctypes.POINTER(P)]
        L.rnnlm_index_create.restype = I
        L.rnnlm_index_free.argtypes = [P]
        L.rnnlm_index_free.restype = I
        L.rnnlm_index_reset.argtypes = [P, P]
        L.rnnlm_index_reset.restype = I
        L.rnnlm_index_intern.argtypes = [P, I, P, P, P, P]
        L.rnnlm_index_intern.restype = I
        L.rnnlm_index_fetch.argtypes = [P, I, P, P, P, P]
        L.rnnlm_index_fetch.restype = I
        L.rnnlm_index_stats.argtypes = [P, P, ctypes.POINTER(ctypes.c_int64)]
        L.rnnlm_index_stats.restype = I
        _lib = L
    return _lib


def rnnlm_strerror(status: int) -> str:
    return lib().rnnlm_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise RnnlmError(status, where)


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _dev(t, dtype, name):
    """Device pointer of a contiguous CUDA tensor of the given torch dtype (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError("%s must be a contiguous device tensor of dtype %s" % (name, dtype))
    return t.data_ptr() or None


def rnnlm_dedup_workspace_bytes(N: int) -> int:
    return int(lib().rnnlm_dedup_workspace_bytes(int(N)))


class RnnlmModel:
    """Handle returned by rnnlm_load; frees the device copy when closed or collected."""

    def __init__(self, handle: int, V: int, H: int, dtype: int, max_B: int):
        self._h = handle
        self.V, self.H, self.dtype, self.max_B = V, H, dtype, max_B

    @property
    def handle(self):
        if not self._h:
            raise ValueError("model already freed")
        return self._h

    def set_option(self, option: int, value: int):
        _check(lib().rnnlm_set_option(self.handle, int(option), int(value)), "rnnlm_set_option")

    def last_error(self, stream=None) -> int:
        f = ctypes.c_int(0)
        _check(lib().rnnlm_last_error(self.handle, _stream(stream), ctypes.byref(f)), "rnnlm_last_error")
        return f.value

    def share(self, max_B: int) -> "RnnlmModel":
        """A further handle on the same weights with scratch of its own, for use on another stream."""
        out = ctypes.c_void_p()
        _check(lib().rnnlm_model_share(self.handle, int(max_B), ctypes.byref(out)), "rnnlm_model_share")
        return RnnlmModel(out.value, self.V, self.H, self.dtype, int(max_B))

    def time_outproj(self, B: int, repeats: int, stream=None, n_rows_dev=None) -> float:
        ms = ctypes.c_float(0)
        import torch
        _check(lib().rnnlm_time_outproj(self.handle, int(B), _dev(n_rows_dev, torch.int32, "n_rows_dev"),
                                        int(repeats), _stream(stream),
                                        ctypes.byref(ms)), "rnnlm_time_outproj")
        return ms.value

    def outproj_kernel_name(self, B: int) -> str:
        """Name of the kernel a launch of the output projection sized for B rows takes."""
        name = lib().rnnlm_outproj_kernel_name(self.handle, int(B))
        if name is None:
            raise ValueError("rnnlm_outproj_kernel_name: bad argument")
        return name.decode()

    def close(self):
        if self._h:
            h, self._h = self._h, None
            _check(lib().rnnlm_free(h), "rnnlm_free")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def rnnlm_time_empty_launch(repeats: int = 1000, stream=None) -> float:
    """Mean time of one launch of an empty kernel, back to back on the stream, in microseconds."""
    us = ctypes.c_float()
    _check(lib().rnnlm_time_empty_launch(int(repeats), _stream(stream), ctypes.byref(us)), "rnnlm_time_empty_launch")
    return float(us.value)


def rnnlm_probe_mfma_rate(feed: int, data: int, launches: int = 20):
    """(TFLOP/s, core GHz) the bf16 matrix cores sustain on the output projection's loop shape."""
    tf, ghz = ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().rnnlm_probe_mfma_rate(int(feed), int(data), int(launches), ctypes.byref(tf), ctypes.byref(ghz)),
           "rnnlm_probe_mfma_rate")
    return tf.value, ghz.value


def rnnlm_load(V: int, H: int, dtype: int, U: np.ndarray, W: np.ndarray, O: np.ndarray,
               bias: Optional[np.ndarray], max_B: int) -> RnnlmModel:
    """Host numpy arrays in: float32 for RNNLM_F32, uint16 bfloat16 bit patterns for RNNLM_BF16."""
    want = np.float32 if dtype == RNNLM_F32 else np.uint16
    arrs = []
    for name, a, shape in (("U", U, (V, H)), ("W", W, (H, H)), ("O", O, (H, V))):
        a = np.ascontiguousarray(a)
        if a.dtype != want or a.shape != shape:
            raise TypeError("%s must be %s of shape %s" % (name, want.__name__, shape))
        arrs.append(a)
    b = None
    if bias is not None:
        b = np.ascontiguousarray(bias, dtype=np.float32)
        if b.shape != (V,):
            raise TypeError("bias must have shape (V,)")
    out = ctypes.c_void_p()
    st = lib().rnnlm_load(V, H, dtype, arrs[0].ctypes.data, arrs[1].ctypes.data, arrs[2].ctypes.data,
                          b.ctypes.data if b is not None else None, int(max_B), ctypes.byref(out))
    _check(st, "rnnlm_load")
    return RnnlmModel(out.value, V, H, dtype, int(max_B))


def rnnlm_dedup(history_ids, rep, inverse, n_unique, workspace, stream=None):
    """history_ids: int64 device tensor holding the u64 bit patterns [N]; rep, inverse int32 [N];
    n_unique int32 [1]; workspace uint8 device tensor of rnnlm_dedup_workspace_bytes(N)."""
    import torch
    N = int(history_ids.shape[0])
    _check(lib().rnnlm_dedup(_dev(history_ids, torch.int64, "history_ids"), N,
                             _dev(rep, torch.int32, "rep"), _dev(inverse, torch.int32, "inverse"),
                             _dev(n_unique, torch.int32, "n_unique"),
                             _dev(workspace, torch.uint8, "workspace"),
                             0 if workspace is None else workspace.numel(), _stream(stream)), "rnnlm_dedup")


DEDUP_STATIC_MAX_N = 65536


def rnnlm_dedup_static(history_ids, rep, inverse, n_unique, stream=None):
    """rnnlm_dedup without a workspace (the library's own fixed device array; N <= DEDUP_STATIC_MAX_N)."""
    import torch
    N = int(history_ids.shape[0])
    _check(lib().rnnlm_dedup_static(_dev(history_ids, torch.int64, "history_ids"), N,
                                    _dev(rep, torch.int32, "rep"), _dev(inverse, torch.int32, "inverse"),
                                    _dev(n_unique, torch.int32, "n_unique"), _stream(stream)), "rnnlm_dedup_static")


def rnnlm_step(model: RnnlmModel, prev_word, h_in, query_word, h_out, logprob,
               row_of_query=None, stream=None):
    import torch
    B = int(prev_word.shape[0])
    N = int(query_word.shape[0])
    K = int(query_word.shape[1]) if query_word.dim() == 2 else 0
    if h_in.shape != (B, model.H) or h_out.shape != (B, model.H) or logprob.shape != (N, K):
        raise TypeError("shape mismatch")
    if row_of_query is not None and row_of_query.shape != (N,):
        raise TypeError("row_of_query must have shape (N,)")
    _check(lib().rnnlm_step(model.handle, B, K, _dev(prev_word, torch.int32, "prev_word"),
                            _dev(h_in, torch.float32, "h_in"), _dev(query_word, torch.int32, "query_word"),
                            _dev(row_of_query, torch.int32, "row_of_query"), N,
                            _dev(h_out, torch.float32, "h_out"), _dev(logprob, torch.float32, "logprob"),
                            _stream(stream)), "rnnlm_step")


def rnnlm_step_dedup(model: RnnlmModel, history_ids, prev_word, h_in, query_word, rep, inverse, n_unique,
                     h_out, logprob, workspace, stream=None):
    import torch
    N = int(history_ids.shape[0])
    K = int(query_word.shape[1]) if query_word.dim() == 2 else 0
    if (prev_word.shape != (N,) or h_in.shape != (N, model.H) or h_out.shape != (N, model.H)
            or query_word.shape[0] != N or logprob.shape != (N, K)
            or rep.shape != (N,) or inverse.shape != (N,)):
        raise TypeError("shape mismatch")
    _check(lib().rnnlm_step_dedup(model.handle, N, K, _dev(history_ids, torch.int64, "history_ids"),
                                  _dev(prev_word, torch.int32, "prev_word"), _dev(h_in, torch.float32, "h_in"),
                                  _dev(query_word, torch.int32, "query_word"), _dev(rep, torch.int32, "rep"),
                                  _dev(inverse, torch.int32, "inverse"), _dev(n_unique, torch.int32, "n_unique"),
                                  _dev(h_out, torch.float32, "h_out"), _dev(logprob, torch.float32, "logprob"),
                                  _dev(workspace, torch.uint8, "workspace"),
                                  0 if workspace is None else workspace.numel(), _stream(stream)),
           "rnnlm_step_dedup")


class RnnlmCache:
    """Handle returned by rnnlm_cache_create."""

    def __init__(self, handle: int, capacity: int):
        self._h = handle
        self.capacity = capacity

    @property
    def handle(self):
        if not self._h:
            raise ValueError("cache already freed")
        return self._h

    def reset(self, stream=None):
        _check(lib().rnnlm_cache_reset(self.handle, _stream(stream)), "rnnlm_cache_reset")

    def stats(self, stream=None) -> dict:
        out = (ctypes.c_int64 * 5)()
        _check(lib().rnnlm_cache_stats(self.handle, _stream(stream), out), "rnnlm_cache_stats")
        return dict(zip(("entries", "lookups", "hits", "misses", "unstored"), (int(x) for x in out)))

    def close(self):
        if self._h:
            h, self._h = self._h, None
            _check(lib().rnnlm_cache_free(h), "rnnlm_cache_free")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def rnnlm_cache_create(model: RnnlmModel, capacity: int) -> RnnlmCache:
    out = ctypes.c_void_p()
    _check(lib().rnnlm_cache_create(model.handle, int(capacity), ctypes.byref(out)), "rnnlm_cache_create")
    return RnnlmCache(out.value, int(capacity))


def rnnlm_step_cached(model: RnnlmModel, cache: Optional[RnnlmCache], history_ids, prev_word, h_in,
                      query_word, rep, inverse, n_unique, h_out, score, workspace, base_score=None,
                      step_stats=None, stream=None):
    import torch
    N = int(history_ids.shape[0])
    K = int(query_word.shape[1]) if query_word.dim() == 2 else 0
    if (prev_word.shape != (N,) or h_in.shape != (N, model.H) or h_out.shape != (N, model.H)
            or query_word.shape[0] != N or score.shape != (N, K)
            or rep.shape != (N,) or inverse.shape != (N,)):
        raise TypeError("shape mismatch")
    if base_score is not None and base_score.shape != (N, K):
        raise TypeError("base_score must have shape (N, K)")
    if step_stats is not None and step_stats.shape != (4,):
        raise TypeError("step_stats must have shape (4,)")
    _check(lib().rnnlm_step_cached(model.handle, cache.handle if cache is not None else None, N, K,
                                   _dev(history_ids, torch.int64, "history_ids"),
                                   _dev(prev_word, torch.int32, "prev_word"), _dev(h_in, torch.float32, "h_in"),
                                   _dev(query_word, torch.int32, "query_word"),
                                   _dev(base_score, torch.float32, "base_score"),
                                   _dev(rep, torch.int32, "rep"), _dev(inverse, torch.int32, "inverse"),
                                   _dev(n_unique, torch.int32, "n_unique"),
                                   _dev(h_out, torch.float32, "h_out"), _dev(score, torch.float32, "score"),
                                   _dev(step_stats, torch.int32, "step_stats"),
                                   _dev(workspace, torch.uint8, "workspace"),
                                   0 if workspace is None else workspace.numel(), _stream(stream)),
           "rnnlm_step_cached")


def rnnlm_pack_ids(ctx_idx, small_lm_idx, ids, stream=None):
    """ctx_idx, small_lm_idx: int32 device tensors holding u32 bit patterns [N]; ids int64 [N] out."""
    import torch
    N = int(ctx_idx.shape[0])
    if small_lm_idx.shape != (N,) or ids.shape != (N,):
        raise TypeError("shape mismatch")
    _check(lib().rnnlm_pack_ids(_dev(ctx_idx, torch.int32, "ctx_idx"), _dev(small_lm_idx, torch.int32, "small_lm_idx"),
                                N, _dev(ids, torch.int64, "ids"), _stream(stream)), "rnnlm_pack_ids")


INDEX_NOT_STORED, INDEX_COLLISION = 0xFFFFFFFF, 0xFFFFFFFE


class RnnlmIndexTable:
    """Handle returned by rnnlm_index_create."""

    def __init__(self, handle: int, H: int, capacity: int, max_N: int):
        self._h = handle
        self.H, self.capacity, self.max_N = H, capacity, max_N

    @property
    def handle(self):
        if not self._h:
            raise ValueError("index table already freed")
        return self._h

    def reset(self, stream=None):
        _check(lib().rnnlm_index_reset(self.handle, _stream(stream)), "rnnlm_index_reset")

    def stats(self, stream=None) -> dict:
        out = (ctypes.c_int64 * 6)()
        _check(lib().rnnlm_index_stats(self.handle, _stream(stream), out), "rnnlm_index_stats")
        return dict(zip(("entries", "lookups", "found", "unstored", "collisions", "bad_fetch"),
                        (int(x) for x in out)))

    def close(self):
        if self._h:
            h, self._h = self._h, None
            _check(lib().rnnlm_index_free(h), "rnnlm_index_free")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def rnnlm_index_create(H: int, capacity: int, max_N: int) -> RnnlmIndexTable:
    out = ctypes.c_void_p()
    _check(lib().rnnlm_index_create(int(H), int(capacity), int(max_N), ctypes.byref(out)), "rnnlm_index_create")
    return RnnlmIndexTable(out.value, int(H), int(capacity), int(max_N))


def rnnlm_index_intern(table: RnnlmIndexTable, word, h, index, stream=None):
    """word int32 [N], h float32 [N,H], index int32 [N] out (u32 bit patterns); device tensors."""
    import torch
    N = int(word.shape[0])
    if h.shape != (N, table.H) or index.shape != (N,):
        raise TypeError("shape mismatch")
    _check(lib().rnnlm_index_intern(table.handle, N, _dev(word, torch.int32, "word"), _dev(h, torch.float32, "h"),
                                    _dev(index, torch.int32, "index"), _stream(stream)), "rnnlm_index_intern")


def rnnlm_index_fetch(table: RnnlmIndexTable, index, word, h, stream=None):
    import torch
    N = int(index.shape[0])
    if h.shape != (N, table.H) or word.shape != (N,):
        raise TypeError("shape mismatch")
    _check(lib().rnnlm_index_fetch(table.handle, N, _dev(index, torch.int32, "index"), _dev(word, torch.int32, "word"),
                                   _dev(h, torch.float32, "h"), _stream(stream)), "rnnlm_index_fetch")


def rnnlm_huffman_build(frequency: np.ndarray):
    """Host-side Huffman tree over the words: returns (path_offset i32[V+1], path_entry i32[total])."""
    f = np.ascontiguousarray(frequency, dtype=np.float64)
    V = int(f.shape[0])
    off = np.zeros(V + 1, dtype=np.int32)
    need = ctypes.c_size_t(0)
    st = lib().rnnlm_huffman_build(V, f.ctypes.data, off.ctypes.data, None, 0, ctypes.byref(need))
    if st not in (0, -4):
        _check(st, "rnnlm_huffman_build")
    entry = np.zeros(max(need.value, 1), dtype=np.int32)
    _check(lib().rnnlm_huffman_build(V, f.ctypes.data, off.ctypes.data, entry.ctypes.data, need.value,
                                     ctypes.byref(need)), "rnnlm_huffman_build")
    return off, entry[:need.value]


def rnnlm_hs_load(V: int, H: int, dtype: int, U: np.ndarray, W: np.ndarray, Theta: np.ndarray,
                  path_offset: np.ndarray, path_entry: np.ndarray, max_B: int) -> RnnlmModel:
    want = np.float32 if dtype == RNNLM_F32 else np.uint16
    arrs = []
    for name, a, shape in (("U", U, (V, H)), ("W", W, (H, H)), ("Theta", Theta, (V - 1, H))):
        a = np.ascontiguousarray(a)
        if a.dtype != want or a.shape != shape:
            raise TypeError("%s must be %s of shape %s" % (name, want.__name__, shape))
        arrs.append(a)
    off = np.ascontiguousarray(path_offset, dtype=np.int32)
    ent = np.ascontiguousarray(path_entry, dtype=np.int32)
    if off.shape != (V + 1,) or ent.shape != (int(off[-1]),):
        raise TypeError("path arrays have the wrong size")
    out = ctypes.c_void_p()
    _check(lib().rnnlm_hs_load(V, H, dtype, arrs[0].ctypes.data, arrs[1].ctypes.data, arrs[2].ctypes.data,
                               off.ctypes.data, ent.ctypes.data, int(max_B), ctypes.byref(out)), "rnnlm_hs_load")
    return RnnlmModel(out.value, V, H, dtype, int(max_B))


def rnnlm_hs_step(model: RnnlmModel, prev_word, h_in, query_word, h_out, logprob, row_of_query=None,
                  base_score=None, stream=None):
    import torch
    B = int(prev_word.shape[0])
    N = int(query_word.shape[0])
    K = int(query_word.shape[1]) if query_word.dim() == 2 else 0
    if h_in.shape != (B, model.H) or h_out.shape != (B, model.H) or logprob.shape != (N, K):
        raise TypeError("shape mismatch")
    _check(lib().rnnlm_hs_step(model.handle, B, K, _dev(prev_word, torch.int32, "prev_word"),
                               _dev(h_in, torch.float32, "h_in"), _dev(query_word, torch.int32, "query_word"),
                               _dev(row_of_query, torch.int32, "row_of_query"), N,
                               _dev(base_score, torch.float32, "base_score"),
                               _dev(h_out, torch.float32, "h_out"), _dev(logprob, torch.float32, "logprob"),
                               _stream(stream)), "rnnlm_hs_step")


def rnnlm_hs_time_query(model: RnnlmModel, query_word, h_out, logprob, repeats: int, row_of_query=None,
                        stream=None) -> float:
    import torch
    B, (N, K) = int(h_out.shape[0]), query_word.shape
    ms = ctypes.c_float(0)
    _check(lib().rnnlm_hs_time_query(model.handle, B, int(K), _dev(query_word, torch.int32, "query_word"),
                                     _dev(row_of_query, torch.int32, "row_of_query"), int(N),
                                     _dev(h_out, torch.float32, "h_out"), _dev(logprob, torch.float32, "logprob"),
                                     int(repeats), _stream(stream), ctypes.byref(ms)), "rnnlm_hs_time_query")
    return ms.value
