"""Host-side logic of the paged cache layout, no GPU: the page-id allocator and the closed forms
of the pool size through the C ABI, and the same sources (allocator, row-map construction) built
with AddressSanitizer + UndefinedBehaviorSanitizer and run as a plain program."""
import ctypes as C
import os
import shutil
import subprocess

import pytest

from paper_2506_06295_amd import binding
from paper_2506_06295_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_pool_allocator_through_the_abi():
    pool = binding.PagePool(12)
    assert pool.available == 12
    a = pool.alloc(5)
    assert a == [0, 1, 2, 3, 4] and pool.available == 7
    with pytest.raises(binding.DllmcError, match="ENOMEM"):
        pool.alloc(8)
    assert pool.available == 7
    for bad in ([1, 1], [12], [9], [-1]):
        with pytest.raises(binding.DllmcError, match="EINVAL"):
            pool.free(bad)
        assert pool.available == 7
    pool.free([3, 1])
    assert pool.alloc(3) == [1, 3, 5]
    assert pool.alloc(0) == []
    pool.close()
    with pytest.raises(binding.DllmcError):
        binding.PagePool(0)


@pytest.mark.parametrize("name", ["llada8b", "dream7b", "llada8b_long"])
def test_pool_bytes_is_the_storage_closed_form(name):
    """Storage-overhead proof of the paper: four tensors of tokens x width per layer; here in pages
    (K and V are d_kv wide for grouped KV heads), bf16."""
    cfg = I.CONFIGS[name]
    m = binding.dllmc_model(cfg.T, cfg.d, cfg.H_q, cfg.H_kv, cfg.d_h, cfg.m, cfg.B, 1, cfg.rms_eps, cfg.rope_theta)
    page_rows, pool_pages = 64, 3 * ((cfg.n + 63) // 64)
    want = cfg.T * page_rows * pool_pages * (2 * cfg.d_kv + 2 * cfg.d) * 2
    assert binding.pool_bytes(m, page_rows, pool_pages) == want
    assert binding.pool_bytes(m, 0, pool_pages) == 0 and binding.pool_bytes(m, page_rows, 0) == 0
    L = binding.lib()
    pps = (cfg.n + page_rows - 1) // page_rows
    table = (C.c_int32 * (cfg.B * pps))(*range(cfg.B * pps))
    inside = binding.dllmc_paging(page_rows, pool_pages, table, None, 0)
    outside = binding.dllmc_paging(page_rows, pool_pages, table, 256, want)   # any non-null pool pointer
    w_in = L.dllmc_workspace_bytes_paged(C.byref(m), cfg.L_p, cfg.L_r, C.byref(inside))
    w_out = L.dllmc_workspace_bytes_paged(C.byref(m), cfg.L_p, cfg.L_r, C.byref(outside))
    assert w_in - w_out == want            # a caller-owned pool takes the caches out of the workspace
    flat = L.dllmc_workspace_bytes(C.byref(m), cfg.L_p, cfg.L_r)
    exact_pool = binding.dllmc_paging(page_rows, cfg.B * pps, table, None, 0)
    w_exact = L.dllmc_workspace_bytes_paged(C.byref(m), cfg.L_p, cfg.L_r, C.byref(exact_pool))
    # a pool that holds exactly the sequences' pages costs the flat layout plus page round-up and the row map
    assert 0 <= w_exact - flat <= cfg.T * cfg.B * (pps * page_rows - cfg.n) * (2 * cfg.d_kv + 2 * cfg.d) * 2 + cfg.B * cfg.n * 4 + 4096


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_paging_host_logic_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "paging_driver")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-pthread", os.path.join(ROOT, "tests", "host_san", "paging_driver.cpp"),
           os.path.join(ROOT, "paper_2506_06295_amd", "csrc", "page_pool.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", UBSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "paging host logic ok" in r.stdout, r.stdout + r.stderr
