"""rnnlm_dedup_static -- the entry point that allocates nothing -- through the C ABI against
rnnlm_dedup on the same ids: bit-exact, on two calls in a row of which the second is smaller
(the library's fixed device array keeps the first call's contents), on sizes that use the array
(the many-launch path above 7168 ids) and one that does not."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2007_11794_amd as rn

from harness import DEV, gpu_dedup, keys_tensor

pytestmark = pytest.mark.gpu


def static_dedup(keys: np.ndarray):
    """One raw call of the C symbol: plain pointers and sizes, no workspace."""
    N = len(keys)
    k_t = keys_tensor(keys) if N else torch.zeros(0, dtype=torch.int64, device=DEV)
    rep = torch.full((max(N, 1),), -1, device=DEV, dtype=torch.int32)
    inv = torch.full((max(N, 1),), -1, device=DEV, dtype=torch.int32)
    nu = torch.full((1,), -1, device=DEV, dtype=torch.int32)
    stream = torch.cuda.current_stream().cuda_stream
    st = rn.lib().rnnlm_dedup_static(ctypes.c_void_p(k_t.data_ptr() if N else 0), N, ctypes.c_void_p(rep.data_ptr()),
                                     ctypes.c_void_p(inv.data_ptr()), ctypes.c_void_p(nu.data_ptr()),
                                     ctypes.c_void_p(stream))
    assert st == 0, st
    torch.cuda.synchronize()
    U = int(nu.item())
    return U, rep.cpu().numpy()[:U], inv.cpu().numpy()[:N]


def ids(N, distinct, seed):
    rng = np.random.default_rng(seed)
    pool = rng.integers(0, 2 ** 64, size=distinct, dtype=np.uint64)
    keys = pool[rng.integers(0, distinct, size=N)]
    keys[: min(N, distinct)] = pool[: min(N, distinct)]
    return keys[rng.permutation(N)]


def test_two_calls_in_a_row_second_smaller_match_rnnlm_dedup():
    for N, distinct, seed in ((60000, 20000, 1), (9000, 2500, 2), (65536, 65536, 3), (7169, 5, 4), (3000, 900, 5),
                              (0, 1, 6), (20000, 19000, 7)):
        keys = ids(N, distinct, seed) if N else np.zeros(0, np.uint64)
        U, rep, inv = static_dedup(keys)
        U0, rep0, inv0 = gpu_dedup(keys)
        assert U == U0 == (len(np.unique(keys)) if N else 0), (N, U, U0)
        assert np.array_equal(rep, rep0) and np.array_equal(inv, inv0), N
        if N:
            assert np.array_equal(keys[rep][inv], keys)


def test_sizes_beyond_the_maximum_are_refused():
    N = rn.DEDUP_STATIC_MAX_N + 1
    t = torch.zeros(N, dtype=torch.int64, device=DEV)
    o = torch.zeros(N, dtype=torch.int32, device=DEV)
    nu = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(rn.RnnlmError) as e:
        rn.rnnlm_dedup_static(t, o, o.clone(), nu)
    assert e.value.status == -4
    rn.rnnlm_dedup_static(t[: rn.DEDUP_STATIC_MAX_N], o, o.clone(), nu)      # the maximum itself is served
    torch.cuda.synchronize()
    assert int(nu.item()) == 1
