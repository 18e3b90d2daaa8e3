"""Host-side logic of the library that needs no GPU: the GEMM slice planner never plans more
float32 partial sums than the slice buffer holds (an overflow there is an out-of-bounds write
on the device), for every shape the workloads produce and for random ones."""
import ctypes
import os

import numpy as np
import pytest

from paper_2506_06295_amd import binding, inputs as I

pytestmark = pytest.mark.skipif(not os.path.exists(binding.LIB_PATH), reason="libdllmc.so not built")


def workspace_cws_floats(cfg):
    # mirrors make_layout(): rows padded to 128 times the widest GEMM output, plus 640 tiles
    rows = cfg.B * cfg.n
    n_max = max(2 * cfg.m, cfg.d_q + cfg.d_kv, cfg.d)
    return (rows + 127) // 128 * 128 * n_max + 640 * 128 * 128


def step_gemm_shapes(cfg):
    k = int(np.floor(cfg.rho * cfg.L_r + 1e-6))
    for P in (False, True):
        for Rf in (False, True):
            Mc = cfg.B * ((cfg.L_p if P else 0) + cfg.L_r)
            M_R = cfg.B * ((cfg.L_p if P else 0) + (cfg.L_r if Rf else k))
            yield Mc, cfg.d_kv, cfg.d_kv, cfg.d
            if M_R:
                yield M_R, cfg.d_q + cfg.d_kv, cfg.d_q, cfg.d
                yield M_R, cfg.d, cfg.d, cfg.d_q
                yield M_R, 2 * cfg.m, cfg.m, cfg.d
                yield M_R, cfg.d, cfg.d, cfg.m


@pytest.mark.parametrize("name", list(I.CONFIGS))
def test_planned_slices_fit_the_workspace_for_every_step_kind(name):
    cfg = I.CONFIGS[name]
    L = binding.lib()
    cap = workspace_cws_floats(cfg)
    dt = 1 if cfg.dtype == "bf16" else 0
    for rho in (cfg.rho, 0.05, 0.5, 1.0):
        c = cfg.replace(rho=rho)
        for M, N, N0, K in step_gemm_shapes(c):
            S = L.dllmc_plan_gemm_slices(dt, M, N, N0, K, cap)
            assert 1 <= S <= 8, (M, N, K, S)
            assert S * M * N <= cap, (M, N, K, S)


def test_planned_slices_respect_any_capacity():
    L = binding.lib()
    r = np.random.default_rng(0)
    for _ in range(3000):
        M = int(r.integers(1, 20000))
        N = int(r.choice([128, 256, 512, 1024, 4096, 8192, 24576, 37888, 200, 704]))
        K = int(r.choice([128, 256, 512, 896, 1024, 3584, 4096, 12288, 18944, 72]))
        cap = int(r.integers(1, 9)) * M * N + int(r.integers(0, 1000)) - (M * N if r.random() < 0.1 else 0)
        for dt in (0, 1):
            S = L.dllmc_plan_gemm_slices(dt, M, N, N, K, max(cap, 0))
            if cap < M * N:
                assert S == 0
            else:
                assert S >= 1 and S * M * N <= cap


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU; asking for more ends with a message, before anything touches a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=60)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
