"""The library's host-side Huffman builder against the oracle's (no GPU needed): the
construction rule is fixed (two queues, ties: word before inner node, lower id first), so the
trees must be identical, entry for entry."""
import ctypes

import numpy as np
import pytest

import oracle
import paper_2007_11794_amd as rn


@pytest.mark.parametrize("V,kind", [(2, "flat"), (3, "zipf"), (6, "textbook"), (257, "flat"), (1000, "zipf"),
                                    (4096, "ties"), (65536, "zipf"), (200000, "zipf1")])
def test_same_tree_as_the_oracle(V, kind):
    rng = np.random.default_rng(V)
    if kind == "flat":
        f = np.ones(V)
    elif kind == "textbook":
        f = np.array([5, 9, 12, 13, 16, 45], dtype=np.float64)
    elif kind == "ties":
        f = rng.integers(1, 5, V).astype(np.float64)           # many equal weights
    else:
        f = np.arange(1, V + 1, dtype=np.float64) ** (-1.0 if kind == "zipf1" else -1.1)
        f = f[rng.permutation(V)]
    off_l, ent_l = rn.rnnlm_huffman_build(f)
    off_o, ent_o = oracle.huffman_build(f)
    assert np.array_equal(off_l, off_o) and np.array_equal(ent_l, ent_o)


def test_errors_and_size_query():
    L = rn.lib()
    off = np.zeros(4, np.int32)
    f = np.array([1.0, 2.0, 3.0])
    need = ctypes.c_size_t(0)
    assert L.rnnlm_huffman_build(3, f.ctypes.data, off.ctypes.data, None, 0, ctypes.byref(need)) == -4
    assert need.value == 5 and off.tolist() == [0, 2, 4, 5]
    ent = np.zeros(4, np.int32)
    assert L.rnnlm_huffman_build(3, f.ctypes.data, off.ctypes.data, ent.ctypes.data, 4, None) == -4   # too small
    assert L.rnnlm_huffman_build(1, f.ctypes.data, off.ctypes.data, ent.ctypes.data, 4, None) == -1
    bad = np.array([1.0, -1.0, 3.0])
    assert L.rnnlm_huffman_build(3, bad.ctypes.data, off.ctypes.data, ent.ctypes.data, 4, None) == -1
    bad[1] = np.nan
    assert L.rnnlm_huffman_build(3, bad.ctypes.data, off.ctypes.data, ent.ctypes.data, 4, None) == -1
