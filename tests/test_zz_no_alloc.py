"""The entry point that allocates nothing (dllmc_op_linear_static: the float32 slices of the
split contraction live in a buffer inside the library's device image) against dllmc_op_linear,
through the C ABI: two calls in a row, the second smaller, so that the first call's leftovers
in the shared buffer would show; results must be bit-identical while M * N <= 2^20 (same slices)
and within float32 summation noise above; sizes beyond the buffer are refused."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2506_06295_amd import binding

pytestmark = pytest.mark.gpu


def _operands(M, N, K, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    a = torch.randn((M + 19, K), device="cuda", generator=g).to(torch.bfloat16)
    w = (0.05 * torch.randn((N, K), device="cuda", generator=g)).to(torch.bfloat16)
    idx = torch.randperm(M + 19, device="cuda", generator=g)[:M].to(torch.int32)
    return a, w, idx


def test_static_scratch_linear_matches_op_linear_twice_in_a_row():
    cases = [(200, 4096, 1024), (64, 1024, 4096)]           # the second call is the smaller one
    outs = []
    for seed, (M, N, K) in enumerate(cases):
        a, w, idx = _operands(M, N, K, seed)
        out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        binding.op_linear_static("bf16", a, w, out, idx)
        outs.append((out, a, w, idx))
    torch.cuda.synchronize()
    for out, a, w, idx in outs:
        want = binding.op_linear("bf16", a, w, idx)
        torch.cuda.synchronize()
        assert torch.equal(out, want)
        ref = a.float()[idx.long()].double() @ w.double().T
        assert float((out.double() - ref).norm() / ref.norm()) < 1e-5


def test_static_scratch_linear_above_the_common_slice_count_and_float32():
    # M * N > 2^20: fewer slices fit the static buffer than op_linear's own scratch
    M, N, K = 1500, 2048, 512
    a, w, idx = _operands(M, N, K, 7)
    out = torch.empty((M, N), dtype=torch.float32, device="cuda")
    binding.op_linear_static("bf16", a, w, out, idx)
    want = binding.op_linear("bf16", a, w, idx)
    torch.cuda.synchronize()
    assert float((out - want).norm() / want.norm()) < 1e-5
    # then a small float32 problem (plain kernel) through the same buffer
    a32 = torch.randn((40, 72), device="cuda")
    w32 = torch.randn((100, 72), device="cuda")
    out32 = torch.empty((40, 100), dtype=torch.float32, device="cuda")
    binding.op_linear_static("f32", a32, w32, out32)
    torch.cuda.synchronize()
    assert torch.equal(out32, binding.op_linear("f32", a32, w32))


def test_static_scratch_linear_refuses_what_does_not_fit():
    L = binding.lib()
    cap = L.dllmc_op_linear_static_max_elements()
    assert cap == 8 << 20
    a = torch.zeros((8, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(8, dtype=torch.float32, device="cuda")
    M, N = 4096, 4096                      # 16 Mi elements: nothing may be launched
    rc = L.dllmc_op_linear_static(1, a.data_ptr(), None, M, a.data_ptr(), N, 128, out.data_ptr(), None)
    assert rc == -5 and b"static scratch" in L.dllmc_strerror(rc)
    with pytest.raises(binding.DllmcError):
        binding.op_linear_static("bf16", a, a, out, torch.zeros(0, dtype=torch.int32, device="cuda"))
