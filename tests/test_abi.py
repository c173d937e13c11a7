"""The C-ABI library without a GPU: it loads, exports what include/rnnlm.h and include/rnnlm_diag.h declare, and
rejects host-checkable mistakes before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2007_11794_amd as rn
from paper_2007_11794_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    for header in ("rnnlm.h", "rnnlm_diag.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(rnnlm_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = rn.lib()
    names = declared_functions()
    assert "rnnlm_load" in names and "rnnlm_dedup" in names and "rnnlm_step" in names
    for n in names:
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == names


def test_strerror_texts():
    assert rn.rnnlm_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert rn.rnnlm_strerror(code) not in ("ok", "unknown status")
    assert rn.rnnlm_strerror(-99) == "unknown status"


def test_workspace_bytes():
    assert rn.rnnlm_dedup_workspace_bytes(0) == 0
    assert rn.rnnlm_dedup_workspace_bytes(-3) == 0
    small, big = rn.rnnlm_dedup_workspace_bytes(10), rn.rnnlm_dedup_workspace_bytes(100000)
    assert 0 < small < big
    assert big >= 100000 * (8 * 2 + 4)          # table of >= 2N slots of key+2 ints, plus N slot ids
    assert big % 256 == 0


def test_host_checked_errors_return_before_any_device_work():
    L = rn.lib()
    out = ctypes.c_void_p()
    buf = (ctypes.c_float * 16)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    EINVAL, ERANGE, EWORKSPACE = -1, -4, -5
    assert L.rnnlm_load(0, 4, 0, p, p, p, None, 1, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_load(4, 0, 0, p, p, p, None, 1, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_load(4, 4, 7, p, p, p, None, 1, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_load(4, 4, 0, None, p, p, None, 1, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_load(4, 4, 0, p, p, p, None, 0, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_load(4, 4, 0, p, p, p, None, 1, None) == EINVAL
    assert out.value is None
    assert L.rnnlm_free(None) == 0
    assert L.rnnlm_set_option(None, 1, 0) == EINVAL
    assert L.rnnlm_step(None, 1, 1, p, p, p, None, 1, p, p, None) == EINVAL
    assert L.rnnlm_step_dedup(None, 1, 1, p, p, p, p, p, p, p, p, p, p, 1 << 20, None) == EINVAL
    assert L.rnnlm_dedup(p, -1, p, p, p, p, 1 << 20, None) == EINVAL
    assert L.rnnlm_dedup(None, 4, p, p, p, p, 1 << 20, None) == EINVAL
    assert L.rnnlm_dedup(p, 4, p, p, None, p, 1 << 20, None) == EINVAL
    assert L.rnnlm_dedup(p, 4, p, p, p, None, 1 << 20, None) == EWORKSPACE
    assert L.rnnlm_dedup(p, 4, p, p, p, p, 8, None) == EWORKSPACE
    assert L.rnnlm_dedup(p, 4, p, p, p, ctypes.c_void_p(p.value + 4), 1 << 20, None) == EWORKSPACE
    assert L.rnnlm_dedup(p, (1 << 28) + 1, p, p, p, p, 1 << 20, None) == ERANGE
    ms = ctypes.c_float()
    assert L.rnnlm_time_outproj(None, 1, None, 1, None, ctypes.byref(ms)) == EINVAL
    assert L.rnnlm_model_share(None, 4, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_model_share(None, 4, None) == EINVAL
    assert L.rnnlm_dedup_static(p, -1, p, p, p, None) == EINVAL
    assert L.rnnlm_dedup_static(None, 4, p, p, p, None) == EINVAL
    assert L.rnnlm_dedup_static(p, 4, p, p, None, None) == EINVAL
    assert L.rnnlm_dedup_static(p, 65537, p, p, p, None) == ERANGE
    us = ctypes.c_float()
    assert L.rnnlm_time_empty_launch(0, None, ctypes.byref(us)) == EINVAL
    assert L.rnnlm_time_empty_launch(10, None, None) == EINVAL
    L.rnnlm_outproj_kernel_name.restype = ctypes.c_char_p
    assert L.rnnlm_outproj_kernel_name(None, 4) is None
    tf = ctypes.c_double()
    assert L.rnnlm_probe_mfma_rate(2, 0, 1, ctypes.byref(tf), None) == EINVAL
    assert L.rnnlm_probe_mfma_rate(0, -1, 1, ctypes.byref(tf), None) == EINVAL
    assert L.rnnlm_probe_mfma_rate(0, 0, 0, ctypes.byref(tf), None) == EINVAL
    assert L.rnnlm_probe_mfma_rate(0, 0, 1001, ctypes.byref(tf), None) == EINVAL
    assert L.rnnlm_probe_mfma_rate(0, 0, 1, None, None) == EINVAL


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        rn.rnnlm_dedup(torch.zeros(4, dtype=torch.int64), torch.zeros(4, dtype=torch.int32),
                       torch.zeros(4, dtype=torch.int32), torch.zeros(1, dtype=torch.int32),
                       torch.zeros(1024, dtype=torch.uint8), stream=0)


def test_host_checked_errors_of_the_cache_index_and_tree_entry_points():
    L = rn.lib()
    out = ctypes.c_void_p()
    buf = (ctypes.c_float * 16)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    EINVAL, ERANGE = -1, -4
    assert L.rnnlm_cache_create(None, 10, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_cache_create(None, 10, None) == EINVAL
    assert L.rnnlm_cache_free(None) == 0
    assert L.rnnlm_cache_reset(None, None) == EINVAL
    assert L.rnnlm_cache_stats(None, None, None) == EINVAL
    assert L.rnnlm_index_create(0, 10, 10, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_index_create(8, -1, 10, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_index_create(8, 10, 0, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_index_create(8, 1 << 27, 10, ctypes.byref(out)) == ERANGE
    assert L.rnnlm_index_free(None) == 0
    assert L.rnnlm_index_intern(None, 1, p, p, p, None) == EINVAL
    assert L.rnnlm_index_fetch(None, 1, p, p, p, None) == EINVAL
    assert L.rnnlm_pack_ids(None, None, 1, None, None) == EINVAL
    assert L.rnnlm_pack_ids(None, None, 0, None, None) == 0
    assert L.rnnlm_pack_ids(None, None, -1, None, None) == EINVAL
    off = (ctypes.c_int32 * 4)(0, 1, 2, 3)
    ent = (ctypes.c_int32 * 3)(0, 0, 0)
    assert L.rnnlm_hs_load(1, 4, 0, p, p, p, off, ent, 1, ctypes.byref(out)) == EINVAL      # V < 2
    assert L.rnnlm_hs_load(3, 4, 0, p, p, p, None, ent, 1, ctypes.byref(out)) == EINVAL
    bad_off = (ctypes.c_int32 * 4)(0, 1, 1, 2)                                              # an empty path
    assert L.rnnlm_hs_load(3, 4, 0, p, p, p, bad_off, ent, 1, ctypes.byref(out)) == EINVAL
    bad_ent = (ctypes.c_int32 * 3)(0, 2, 0)                                                 # node 2 of a 3-word tree
    assert L.rnnlm_hs_load(3, 4, 0, p, p, p, off, bad_ent, 1, ctypes.byref(out)) == EINVAL
    assert L.rnnlm_hs_step(None, 1, 1, p, p, p, None, 1, None, p, p, None) == EINVAL
    assert L.rnnlm_step_cached(None, None, 1, 1, p, p, p, p, None, p, p, p, p, p, None, p, 64, None) == EINVAL
    assert out.value is None


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N > 1 says so and exits before it touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
