"""The C-ABI library loads without a GPU and exports every symbol include/dllmc.h declares."""
import ctypes
import os
import re

import pytest

from paper_2506_06295_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dllmc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dllmc_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_boundary_calls():
    syms = declared_symbols()
    for s in ("dllmc_create", "dllmc_step", "dllmc_destroy", "dllmc_workspace_bytes"):
        assert s in syms
    assert set(syms) == set(binding.EXPORTS)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libdllmc.so not built in this tree")
    L = binding.lib()
    for s in declared_symbols():
        assert hasattr(L, s), s


def test_host_only_calls_work_without_a_gpu():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libdllmc.so not built in this tree")
    L = binding.lib()
    assert L.dllmc_strerror(0) == b"ok"
    assert b"workspace" in L.dllmc_strerror(-4)
    m = binding.dllmc_model(32, 4096, 32, 32, 128, 12288, 1, binding.DLLMC_BF16, 1e-5, 10000.0)
    nbytes = L.dllmc_workspace_bytes(ctypes.byref(m), 512, 256)
    # caches alone: 4 tensors x layers x tokens x d, bf16 (storage-overhead proof of the paper)
    assert nbytes > 2 * 4 * 32 * 768 * 4096
    assert nbytes < 3 * 2 * 4 * 32 * 768 * 4096
    bad = binding.dllmc_model(32, 4096, 32, 5, 128, 12288, 1, binding.DLLMC_BF16, 1e-5, 10000.0)
    assert L.dllmc_workspace_bytes(ctypes.byref(bad), 512, 256) == 0   # 5 does not divide 32
    assert L.dllmc_workspace_bytes(ctypes.byref(m), 512, 0) == 0
    h = ctypes.c_void_p()
    assert L.dllmc_create(ctypes.byref(h), ctypes.byref(m), None, 512, 256, 0.25, 50, 7, None, 0, None) == -1
    assert L.dllmc_step(None, None, 0, None, None, None) == -1
    assert L.dllmc_destroy(None) == -1


def test_argument_checks_of_the_later_entry_points_need_no_gpu():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libdllmc.so not built in this tree")
    L = binding.lib()
    assert L.dllmc_set_layer_rho(None, None, 0) == -1
    assert L.dllmc_layer_num_selected(None, 0) == -1
    assert L.dllmc_set_policy(None, 0, 0, 0, 0, 0) == -1
    assert L.dllmc_probe_copy(None, None, 1024, None) == -1
    assert L.dllmc_probe_read(None, 1024, None, None) == -1
    assert L.dllmc_probe_mfma(0, 0, None, None, None) == -1
    assert L.dllmc_gen_destroy(None) == -1
