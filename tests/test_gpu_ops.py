"""GPU parity of the single operations behind the C ABI against the CPU oracle.

Sizes span several workgroup tiles and leave ragged tails (row counts that are not multiples
of 16 or 64, key counts that are not multiples of 32).  Integer results must match exactly;
float32 results to 1e-4 relative (Frobenius), bf16 results to 2e-2.
"""
import numpy as np
import pytest
import torch

from oracle import dllm_cache_oracle as O
from paper_2506_06295_amd import binding
from paper_2506_06295_amd.inputs import to_bf16_grid
from tests.parity_util import rel_err

pytestmark = pytest.mark.gpu


def dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t


def grid(a, dtype):
    return to_bf16_grid(a).astype(np.float64) if dtype == "bf16" else np.asarray(a, np.float32).astype(np.float64)


# ------------------------------------------------------------------ select
def check_select(scores, k):
    got = binding.op_select(torch.from_numpy(scores).cuda(), k)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    for b in range(scores.shape[0]):
        want = O.bottom_k(scores[b].astype(np.float64), k)
        assert got[b].tolist() == want.tolist(), f"row {b}, k={k}"


@pytest.mark.parametrize("B,L,k", [(1, 32, 8), (1, 256, 64), (1, 512, 51), (16, 256, 12),
                                   (16, 256, 128), (16, 256, 256), (3, 1000, 333), (2, 5000, 1234),
                                   (1, 1, 1), (1, 7, 0), (4, 257, 256),
                                   (2, 8192, 2048),     # the longest sequence whose keys stay in LDS
                                   (2, 8193, 100), (1, 20000, 5000)])  # beyond it: keys re-read from memory
def test_select_random_scores(B, L, k):
    r = np.random.default_rng(L * 31 + k)
    check_select(r.uniform(-1, 1, size=(B, L)).astype(np.float32), k)


def test_select_exact_ties_take_lowest_indices():
    s = np.ones((2, 256), dtype=np.float32)
    check_select(s, 64)
    s[0, [200, 13, 77]] = [0.5, -0.25, 0.999]
    s[1, 100:140] = 0.75          # a tie block straddling the cut
    s[1, [5, 250]] = 0.1
    check_select(s, 10)
    check_select(s, 41)
    check_select(s, 42)
    check_select(s, 43)


def test_select_few_distinct_values_many_ties():
    r = np.random.default_rng(3)
    for L, k in [(256, 64), (300, 75), (1024, 100)]:
        s = (r.integers(0, 4, size=(5, L)) / 4.0).astype(np.float32)
        check_select(s, k)


def test_select_controlled_gaps_signs_and_zeros():
    r = np.random.default_rng(4)
    L = 256
    # scores clustered just below 1 with gaps of one float32 ulp, as random-init models give
    base = np.float32(1.0) - np.arange(L, dtype=np.float32) * np.float32(2.0 ** -24)
    s = np.stack([r.permutation(base) for _ in range(4)])
    check_select(s, 64)
    # negative values, both zeros (they tie), denormals, large magnitudes
    s2 = r.standard_normal((3, L)).astype(np.float32)
    s2[:, ::7] = 0.0
    s2[:, 3::7] = -0.0
    s2[0, 5] = 1e-42
    s2[1, 9] = -3e38
    check_select(s2, 64)
    check_select(s2, 150)


def test_select_rejects_bad_k():
    s = torch.zeros((1, 8), device="cuda")
    with pytest.raises(binding.DllmcError):
        binding.op_select(s, 9)


# ------------------------------------------------------------------ linear (gather GEMM)
@pytest.mark.parametrize("dtype,M,N,K,gather", [
    ("f32", 8, 256, 256, False), ("f32", 96, 704, 256, True), ("f32", 33, 100, 72, True),
    ("bf16", 64, 4096, 4096, True),      # MFMA streaming kernel, one row tile, split contraction
    ("bf16", 51, 1024, 1024, True),      # ragged rows
    ("bf16", 200, 512, 3584, True),      # several row tiles, K = 28 * 128
    ("bf16", 20, 2432, 896, False),      # N = 19 * 128
    ("bf16", 40, 896, 2432, False),
    ("bf16", 17, 200, 72, True),         # falls back to the plain kernel
    ("bf16", 100, 1024, 1024, True),     # streaming kernel, 128 rows per workgroup
    ("bf16", 128, 512, 896, False),      # the same with phases of 128
    ("bf16", 150, 512, 1024, True),      # two such tiles, the second ragged
    ("bf16", 256, 1024, 4096, True),     # 128 x 128 LDS-direct kernel, split contraction
    ("bf16", 300, 512, 896, True),       # tile kernel, ragged last row tile, K = 14 * 64
    ("bf16", 768, 2432, 1024, False),    # tile kernel, N = 19 * 128
])
def test_linear_matches_matmul(dtype, M, N, K, gather):
    run_linear_case(dtype, M, N, K, gather)


@pytest.mark.parametrize("M,N,K", [(256, 1024, 4096), (300, 512, 896), (768, 2432, 1024)])
def test_linear_tile_kernel(M, N, K):
    binding.set_gemm_tuning(tile_min_m=128)
    try:
        run_linear_case("bf16", M, N, K, True)
    finally:
        binding.set_gemm_tuning(tile_min_m=192)


@pytest.mark.parametrize("M,N,K", [(256, 1024, 4096), (300, 512, 896), (768, 2304, 1024), (100, 256, 512)])
def test_linear_fat_kernel(M, N, K):
    binding.set_gemm_tuning(fat_min_m=64)
    try:
        run_linear_case("bf16", M, N, K, True)
    finally:
        binding.set_gemm_tuning(fat_min_m=512)


@pytest.mark.parametrize("K", [128, 256, 384, 512, 768, 1024, 1280, 1536])
@pytest.mark.parametrize("M,N", [(40, 128), (64, 256)])
def test_linear_streaming_kernel_phase_counts(M, N, K):
    """One slice, so that the workgroup walks K / 256 (or K / 128) phases: one to six, through the
    paired loop and each of its tails."""
    binding.set_gemm_tuning(force_s=1)
    try:
        run_linear_case("bf16", M, N, K, True)
    finally:
        binding.set_gemm_tuning(force_s=0)


@pytest.mark.parametrize("nw", [8, 4])
@pytest.mark.parametrize("M,N,K", [(256, 1024, 4096), (200, 512, 896), (300, 2304, 1024), (512, 1024, 512)])
def test_linear_streaming_kernel_with_256_rows_per_workgroup(M, N, K, nw):
    binding.set_gemm_tuning(tall_max_m=512, nw=nw)
    try:
        run_linear_case("bf16", M, N, K, True)
    finally:
        binding.set_gemm_tuning(tall_max_m=128, nw=8)


def run_linear_case(dtype, M, N, K, gather):
    r = np.random.default_rng(M + N + K)
    rows_total = M + 37
    a = r.standard_normal((rows_total, K)).astype(np.float32)
    w = (0.05 * r.standard_normal((N, K))).astype(np.float32)
    idx = r.permutation(rows_total)[:M].astype(np.int32) if gather else None
    got = binding.op_linear(dtype, dev(a, dtype), dev(w, dtype),
                            None if idx is None else torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    A = grid(a, dtype)
    want = (A[idx] if gather else A[:M]) @ grid(w, dtype).T
    got = got.cpu().numpy()
    if not gather:
        got = got[:M]
    assert got.shape == want.shape
    assert rel_err(got, want) < 1e-5
    assert np.max(np.abs(got - want)) < 1e-4 * np.max(np.abs(want))


# ------------------------------------------------------------------ V-verify
@pytest.mark.parametrize("dtype,rows,d,d_kv", [("f32", 32, 256, 256), ("f32", 50, 96, 40),
                                               ("bf16", 256, 1024, 1024), ("bf16", 80, 896, 128),
                                               ("bf16", 100, 4096, 512)])
def test_vverify_scores_and_cache_overwrite(dtype, rows, d, d_kv):
    r = np.random.default_rng(rows + d)
    h = r.standard_normal((rows, d)).astype(np.float32)
    wv = (0.05 * r.standard_normal((d_kv, d))).astype(np.float32)
    H, W = grid(h, dtype), grid(wv, dtype)
    v_true = H @ W.T
    # cached rows: some identical to the new ones, some slightly moved, some unrelated, one zero
    v_old = v_true.copy()
    v_old[rows // 4: rows // 2] += 0.05 * r.standard_normal((rows // 2 - rows // 4, d_kv))
    v_old[rows // 2: 3 * rows // 4] = r.standard_normal((3 * rows // 4 - rows // 2, d_kv))
    v_old[-1] = 0.0
    v_old = grid(v_old, dtype)
    cache = dev(v_old, dtype)
    got = binding.op_vverify(dtype, dev(h, dtype), dev(wv, dtype), cache)
    torch.cuda.synchronize()
    v_new = O.round_bf16(v_true) if dtype == "bf16" else v_true
    want = O.cosine_scores(v_new, v_old)
    got = got.cpu().numpy().astype(np.float64)
    assert got[-1] == 0.0 and want[-1] == 0.0
    # bf16: a last-bit difference of one V element moves a score by at most ~2^-8/sqrt(d_kv)
    tol = 1e-5 if dtype == "f32" else 2e-4
    assert np.max(np.abs(got - want)) < tol
    if dtype == "f32":
        assert np.all(np.abs(got[: rows // 4] - 1.0) < 1e-6)
    new_cache = cache.float().cpu().numpy().astype(np.float64)
    assert rel_err(new_cache, v_new) < (1e-6 if dtype == "f32" else 1e-3)
    if dtype == "bf16":
        # at most isolated last-bit differences from float32 vs float64 accumulation
        mism = np.mean(new_cache != v_new)
        assert mism < 0.01


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("dtype,B,Mq,n,H_q,H_kv,d_h", [
    ("f32", 1, 8, 96, 4, 4, 64),
    ("f32", 2, 5, 45, 4, 2, 16),
    ("bf16", 1, 64, 768, 4, 4, 128),     # adaptive-step shape: key range split over wavefronts
    ("bf16", 2, 20, 176, 8, 8, 128),     # ragged queries and keys
    ("bf16", 1, 51, 333, 7, 1, 128),     # grouped KV heads
    ("bf16", 3, 200, 200, 28, 4, 128),   # many queries: 128-query tiles, second tile and last key block ragged
    ("bf16", 1, 256, 768, 4, 4, 128),    # 128-query tiles with the keys split six ways and merged
    ("bf16", 2, 130, 1000, 8, 2, 128),   # the same with grouped KV heads, two queries in the second tile
    ("bf16", 1, 128, 64, 2, 2, 128),     # exactly one tile and one key block
    ("bf16", 1, 300, 40, 2, 1, 128),     # 128-query tiles, fewer keys than one block
    ("bf16", 1, 40, 2500, 2, 2, 128),    # long key ranges: 16 ranges of 5 blocks, the last one shorter
    ("bf16", 2, 70, 1100, 8, 2, 128),    # the same with grouped KV heads and two query tiles
    ("bf16", 1, 7, 5, 2, 2, 128),        # fewer keys than one block
    ("bf16", 1, 9, 70, 2, 1, 64),        # head width without an MFMA kernel
])
@pytest.mark.parametrize("split_keys", [True, False])
def test_attention_matches_oracle(dtype, B, Mq, n, H_q, H_kv, d_h, split_keys):
    r = np.random.default_rng(Mq * 7 + n)
    q = r.standard_normal((B, Mq, H_q * d_h)).astype(np.float32)
    k = r.standard_normal((B, n, H_kv * d_h)).astype(np.float32)
    v = r.standard_normal((B, n, H_kv * d_h)).astype(np.float32)
    # make the softmax peaky for some queries and flat for others
    q[:, ::3] *= 0.05
    got = binding.op_attention(dtype, dev(q, dtype), dev(k, dtype), dev(v, dtype), H_q, H_kv, d_h,
                               split_keys=split_keys)
    torch.cuda.synchronize()
    got = got.float().cpu().numpy()
    for b in range(B):
        want = O.attention(grid(q[b], dtype), grid(k[b], dtype), grid(v[b], dtype), H_q, H_kv, d_h)
        e = rel_err(got[b], want)
        assert e < (1e-5 if dtype == "f32" else 1e-2), f"seq {b}: rel err {e:.3e}"


# ------------------------------------------------------------------ achievable-peak probes
@pytest.mark.parametrize("nbytes", [16, 16 * 12345, 1 << 24])
def test_probe_copy_copies_and_probe_read_writes_nothing(nbytes):
    r = np.random.default_rng(nbytes)
    src = torch.from_numpy(r.integers(0, 256, nbytes, dtype=np.uint8)).cuda()
    dst = torch.zeros_like(src)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    keep = src.clone()
    binding.probe_copy(src, dst)
    binding.probe_read(src, sink)
    torch.cuda.synchronize()
    assert torch.equal(dst, keep) and torch.equal(src, keep)
    with pytest.raises(binding.DllmcError):
        binding.probe_copy(src[:8], dst[:8])


def test_probe_mfma_result_follows_the_instruction_layout():
    """The loop's operands are small dyadic numbers, so its result is exact: 8 accumulators x
    iters x (A @ B), with A, B and the result spread over the 64 lanes as the 16x16x32 MFMA
    defines (A: row = lane % 16, k = 8 * (lane / 16) + i; B alike with the column; result:
    row = 4 * (lane / 16) + i, column = lane % 16)."""
    iters = 3
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    flops = binding.probe_mfma(iters, sink)
    torch.cuda.synchronize()
    A = np.zeros((16, 32))
    Bm = np.zeros((32, 16))
    for lane in range(64):
        for i in range(8):
            A[lane % 16, 8 * (lane // 16) + i] = ((lane + i) & 7) / 8.0
            Bm[8 * (lane // 16) + i, lane % 16] = ((3 * lane + i) & 7) / 8.0
    Cm = 8 * iters * (A @ Bm)
    want = np.array([Cm[4 * (lane // 16) + i, lane % 16] for lane in range(64) for i in range(4)])
    assert np.array_equal(sink.cpu().numpy().astype(np.float64), want)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flops == cus * 8 * 4 * iters * 8 * 2 * 16 * 16 * 32


def test_probe_mfma_32x32x16_result_follows_the_instruction_layout():
    """Shape 1 of the MFMA loop: four accumulators x iters x (A @ B) with 32 x 16 and 16 x 32
    operands (A: row = lane % 32, k = 8 * (lane / 32) + i; B alike with the column); a lane
    writes the sum of its 16 results: column lane % 32, rows 8 * (e / 4) + 4 * (lane / 32) + e % 4."""
    iters = 2
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    flops = binding.probe_mfma(iters, sink, shape=1)
    torch.cuda.synchronize()
    A = np.zeros((32, 16))
    Bm = np.zeros((16, 32))
    for lane in range(64):
        for i in range(8):
            A[lane % 32, 8 * (lane // 32) + i] = ((lane + i) & 7) / 8.0
            Bm[8 * (lane // 32) + i, lane % 32] = ((3 * lane + i) & 7) / 8.0
    Cm = 4 * iters * (A @ Bm)
    want = np.array([sum(Cm[8 * (e // 4) + 4 * (lane // 32) + e % 4, lane % 32] for e in range(16))
                     for lane in range(64)])
    assert np.array_equal(sink[:64].cpu().numpy().astype(np.float64), want)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flops == cus * 8 * 4 * iters * 4 * 2 * 32 * 32 * 16
    with pytest.raises(binding.DllmcError):
        binding.probe_mfma(1, sink, shape=2)
