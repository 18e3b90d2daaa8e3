"""The paged cache layout on the GPU: the four per-layer cache tensors in a pool of row pages
behind a page table (the memory-management direction the paper's Limitations paragraph names).
The oracle's model of the caches is the flat one; a paged context must reproduce the flat
context bit for bit (outputs, selected sets, scores, every cache tensor read back in logical
order), and it is compared with the oracle under the same bars as the flat layout."""
import numpy as np
import pytest
import torch

from paper_2506_06295_amd import binding, inputs as I
from tests import parity_util as PU
from tests.test_gpu_step import MINI_DREAM, MINI_LLADA

pytestmark = pytest.mark.gpu


def shuffled_table(cfg, page_rows, pool_pages, seed):
    pps = (cfg.n + page_rows - 1) // page_rows
    ids = np.random.default_rng(seed).permutation(pool_pages)[: cfg.B * pps]
    return ids.reshape(cfg.B, pps).tolist()


def paging_for(cfg, page_rows, slack=1.5, seed=0):
    pps = (cfg.n + page_rows - 1) // page_rows
    pool_pages = int(cfg.B * pps * slack) + 1
    return dict(page_rows=page_rows, pool_pages=pool_pages,
                page_table=shuffled_table(cfg, page_rows, pool_pages, seed))


def make_gpu(cfg, dev_ws, paging=None, **over):
    den = binding.CachedDenoiser(
        n_layers=cfg.T, d_model=cfg.d, n_q_heads=cfg.H_q, n_kv_heads=cfg.H_kv, head_dim=cfg.d_h,
        d_ffn=cfg.m, batch=cfg.B, dtype=cfg.dtype, weights=dev_ws, L_p=cfg.L_p, L_r=cfg.L_r,
        rho=over.get("rho", cfg.rho), K_p=over.get("K_p", cfg.K_p), K_r=over.get("K_r", cfg.K_r),
        rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta, paging=paging)
    policy = {k: over[k] for k in ("metric", "selection", "v_update", "seed", "source") if k in over}
    if policy:
        den.set_policy(**policy)
    return den


def assert_same_state(cfg, a, b, what):
    for l in range(cfg.T):
        for which in range(4):
            ca, cb = a.read_cache(l, which), b.read_cache(l, which)
            torch.cuda.synchronize()
            assert torch.equal(ca, cb), f"{what}: layer {l} cache {which}"


def run_twins(cfg, hidden, steps, paging, **over):
    """The same steps on a flat and on a paged context; everything must agree bit for bit."""
    ws = over.pop("weights")
    flat, paged = make_gpu(cfg, ws, None, **over), make_gpu(cfg, ws, paging, **over)
    K_r = over.get("K_r", cfg.K_r)
    for i in steps:
        o1, n1 = flat.step(hidden(i), i)
        o2, n2 = paged.step(hidden(i), i)
        torch.cuda.synchronize()
        assert n1 == n2 and torch.equal(o1, o2), f"step {i}: output"
        assert torch.equal(flat.sel_idx[:, :, :n1], paged.sel_idx[:, :, :n2]), f"step {i}: selected sets"
        if i % K_r:
            s1, s2 = flat.read_scores(), paged.read_scores()
            torch.cuda.synchronize()
            assert torch.equal(s1, s2), f"step {i}: scores"
    assert_same_state(cfg, flat, paged, "after the schedule")
    return flat, paged


VARIANTS = [dict(), dict(source="k"), dict(v_update="selected", metric="l2")]


@pytest.mark.parametrize("over", VARIANTS, ids=["default", "k_verify", "selected_only_l2"])
@pytest.mark.parametrize("cfg,page_rows", [(I.CONFIGS["toy"], 8), (MINI_LLADA, 16), (MINI_DREAM, 32), (MINI_DREAM, 5)],
                         ids=["toy_f32", "mini_llada", "mini_dream", "mini_dream_odd_pages"])
def test_paged_context_reproduces_the_flat_one(cfg, page_rows, over):
    ws = [{k: PU.to_device(cfg, v) for k, v in w.items()} for w in I.all_weights(cfg)]
    sched = I.TokenSchedule(cfg, stress=True)
    hid = {i: PU.to_device(cfg, sched.hidden_in(i)) for i in range(cfg.steps)}
    flat, paged = run_twins(cfg, lambda i: hid[i], range(cfg.steps), paging_for(cfg, page_rows, seed=page_rows),
                            weights=ws, **over)
    flat.close()
    paged.close()


def test_paged_context_matches_the_oracle():
    cfg = MINI_LLADA
    ws = I.all_weights(cfg)
    gpu, ora = PU.make_pair(cfg, ws, paging=paging_for(cfg, 16, seed=3))
    sched = I.TokenSchedule(cfg, stress=True)
    st = PU.ParityStats()
    for i in range(cfg.steps):
        PU.run_step_pair(cfg, gpu, ora, sched.hidden_in(i), i, st)
    assert st.failed == 0 and st.exact > 0
    PU.compare_caches(cfg, gpu, ora, st)
    gpu.close()


def test_long_prompt_at_full_width_paged():
    """L_p = 4096, L_r = 512 at the LLaDA-8B width (two layers): 72 pages of 64 rows scattered
    over a pool of 100; all four step kinds; bit-identical to the flat context."""
    cfg = I.CONFIGS["llada8b_long"].replace(T=2)
    ws = I.device_weights(cfg)
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    base = torch.randn((cfg.B, cfg.n, cfg.d), device="cuda", generator=g).to(torch.bfloat16)
    noise = [0.5 * torch.randn((cfg.B, cfg.L_r // 3, cfg.d), device="cuda", generator=g).to(torch.bfloat16)
             for _ in range(5)]
    rows = [torch.randperm(cfg.L_r, device="cuda", generator=g)[: cfg.L_r // 3] + cfg.L_p for _ in range(5)]

    def hidden(i):
        h = base.clone()
        h[:, rows[i]] += noise[i]
        return h

    paging = dict(page_rows=64, pool_pages=100, page_table=shuffled_table(cfg, 64, 100, 7))
    flat, paged = run_twins(cfg, hidden, range(5), paging, weights=ws, K_p=4, K_r=3)
    flat.close()
    paged.close()


def test_shared_pool_eviction_and_remap():
    """Two contexts share one caller-owned pool through the host allocator; when the first
    generation is over its pages go back to the pool and the second context is moved onto them
    (a new page table; the next step must then be step 0)."""
    cfg = MINI_LLADA.replace(B=1)
    ws = [{k: PU.to_device(cfg, v) for k, v in w.items()} for w in I.all_weights(cfg)]
    page_rows = 16
    pps = (cfg.n + page_rows - 1) // page_rows
    pool_pages = 2 * pps + 3
    alloc = binding.PagePool(pool_pages)
    ref = make_gpu(cfg, ws)
    nbytes = binding.pool_bytes(ref.model, page_rows, pool_pages)
    pool = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ids_a, ids_b = alloc.alloc(pps), alloc.alloc(pps)
    mk = lambda ids: make_gpu(cfg, ws, dict(page_rows=page_rows, pool_pages=pool_pages, page_table=[ids], pool=pool))
    a, b = mk(ids_a), mk(ids_b)
    sched_a, sched_b = I.TokenSchedule(cfg, stress=True), I.TokenSchedule(cfg.replace(seed=cfg.seed + 1), stress=True)
    ha = [PU.to_device(cfg, sched_a.hidden_in(i)) for i in range(4)]
    hb = [PU.to_device(cfg, sched_b.hidden_in(i)) for i in range(4)]
    want_a, want_b = [], []
    for i in range(4):
        want_a.append(ref.step(ha[i], i)[0].clone())
    for i in range(4):
        want_b.append(ref.step(hb[i], i)[0].clone())      # step 0 starts a new generation
    for i in range(2):                                    # interleaved: neither touches the other's pages
        assert torch.equal(a.step(ha[i], i)[0], want_a[i])
        assert torch.equal(b.step(hb[i], i)[0], want_b[i])
    for i in range(2, 4):
        assert torch.equal(a.step(ha[i], i)[0], want_a[i])
    torch.cuda.synchronize()
    # generation A is over: evict it, hand its pages to B
    a.close()
    alloc.free(ids_a)
    alloc.free(ids_b)
    assert alloc.available == pool_pages
    ids_new = alloc.alloc(pps)
    with pytest.raises(binding.DllmcError, match="EINVAL"):
        b.set_page_table([ids_new[:-1] + [ids_new[0]]])   # a page listed twice: nothing changes
    assert torch.equal(b.step(hb[2], 2)[0], want_b[2])
    b.set_page_table([list(reversed(ids_new))])
    with pytest.raises(binding.DllmcError, match="ESTATE"):
        b.step(hb[3], 3)                                  # the caches are void: step 0 first
    for i in range(4):
        assert torch.equal(b.step(hb[i], i)[0], want_b[i])
    torch.cuda.synchronize()
    b.close()
    ref.close()
    alloc.close()


def test_paging_argument_errors():
    cfg = MINI_LLADA
    ws = [{k: PU.to_device(cfg, v) for k, v in w.items()} for w in I.all_weights(cfg)]
    good = paging_for(cfg, 16)
    pps = (cfg.n + 15) // 16
    for bad in (dict(good, page_rows=0), dict(good, pool_pages=0),
                dict(good, page_table=[[0] * pps, list(range(1, pps + 1))]),            # a page twice
                dict(good, page_table=[list(range(pps)), [good["pool_pages"]] + list(range(pps, 2 * pps - 1))]),  # out of range
                dict(good, pool=torch.empty(1024, dtype=torch.uint8, device="cuda"))):  # pool too small
        with pytest.raises(binding.DllmcError):
            make_gpu(cfg, ws, bad)
    flat = make_gpu(cfg, ws)
    with pytest.raises(binding.DllmcError, match="EINVAL"):
        flat.set_page_table(good["page_table"])            # not a paged context
    flat.close()
