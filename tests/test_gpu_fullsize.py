"""Parity at the headline workload's full size (LLaDA-8B shape: 32 layers, d 4096, L_p 512,
L_r 256, bf16), in the launch configuration bench.py times: the first denoising steps of the
schedule (a full refresh, adaptive steps, a response refresh) on device-drawn random weights against the
oracle, plus properties that hold at any size on the wider shapes (Dream-7B GQA widths, long
prompt).  The oracle runs on the host cores; each test prints its progress.
"""
import time

import numpy as np
import pytest
import torch

from oracle import dllm_cache_oracle as O
from paper_2506_06295_amd import binding, inputs as I
from tests import parity_util as PU

pytestmark = pytest.mark.gpu


def make_gpu(cfg, weights, **over):
    return binding.CachedDenoiser(
        n_layers=cfg.T, d_model=cfg.d, n_q_heads=cfg.H_q, n_kv_heads=cfg.H_kv, head_dim=cfg.d_h,
        d_ffn=cfg.m, batch=cfg.B, dtype=cfg.dtype, weights=weights, L_p=cfg.L_p, L_r=cfg.L_r,
        rho=over.get("rho", cfg.rho), K_p=over.get("K_p", cfg.K_p), K_r=over.get("K_r", cfg.K_r),
        rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta)


def test_llada8b_full_depth_first_steps_match_oracle():
    """All four step kinds at the headline size: a full refresh, six adaptive steps, the first
    response refresh (K_r = 7) and, with K_p lowered to 8, a step that refreshes the prompt while
    the response is updated adaptively.  Every layer's four cache tensors and the step output are
    held to bars derived from the oracle-only noise floor of that very tensor."""
    cfg = I.CONFIGS["llada8b"]
    floor = PU.load_floor("llada8b")
    K_p = 8
    t0 = time.time()
    dev_w = I.device_weights(cfg)
    host_w = [{k: v.float().cpu().numpy() for k, v in w.items()} for w in dev_w]   # float32, 28 GB
    print(f"\n[fullsize] weights ready {time.time() - t0:.1f}s", flush=True)
    gpu = make_gpu(cfg, dev_w, K_p=K_p)
    ora = O.CachedDenoiser(PU.oracle_model(cfg), host_w, cfg.B, cfg.L_p, cfg.L_r, cfg.rho, K_p,
                           cfg.K_r, storage="bf16")
    sched = I.TokenSchedule(cfg, stress=True)
    stats = PU.ParityStats(floor=floor)
    kinds = []
    for i in range(9):
        PU.run_step_pair(cfg, gpu, ora, sched.hidden_in(i), i, stats)
        kinds.append(("P" if i % K_p == 0 else "-") + ("R" if i % cfg.K_r == 0 else "a"))
        print(f"[fullsize] step {i} [{kinds[-1]}]: rel err {stats.rel_per_step[-1]:.3e}  t={time.time() - t0:.1f}s",
              flush=True)
    assert kinds == ["PR"] + ["-a"] * 6 + ["-R", "Pa"]
    print(f"[fullsize] selection exact={stats.exact} tied_same={stats.tied_same} "
          f"followed={stats.followed} failed={stats.failed}; worst |ds| {stats.worst_score_dev:.2e} "
          f"({stats.worst_score_dev_over_tol:.2f} of its tolerance)", flush=True)
    assert stats.failed == 0, stats.failures
    # 7 adaptive steps x 32 layers: nearly every margin is decisive under the stressed schedule
    assert stats.exact >= 188 and stats.followed <= 4
    assert stats.worst_rel <= PU.stated_tol(cfg)
    PU.compare_caches(cfg, gpu, ora, stats, verbose=True)
    print(f"[fullsize] worst distance / bar over all tensors: {stats.worst_over_bar:.2f}", flush=True)
    last = floor["layers"][cfg.T - 1]["FFNOut"]["frob"]
    print(f"[fullsize] note: the last layers' FFNOut floors exceed the stated 2e-2 (layer {cfg.T - 1}: "
          f"{last:.3e} between two oracle evaluations); those tensors are held to 1.5 x floor", flush=True)
    gpu.close()


WIDE = [("dream7b", None), ("llada8b_long", None), ("llada8b_b16", [3, 12])]


@pytest.mark.parametrize("name,seqs", WIDE, ids=[w[0] for w in WIDE])
def test_wide_shapes_match_oracle_at_full_width(name, seqs):
    """Full width and length, two layers, against the oracle: a full refresh, two adaptive steps,
    a response refresh and a prompt refresh with adaptive response (K_p = 4, K_r = 3), i.e. the
    grouped-KV Dream widths (d 3584, FFN 18944), the 4608-row long prompt, and two of the sixteen
    batched sequences.  Bars from tests/golden/noise_floor_<name>_T2.json (oracle only)."""
    cfg = I.CONFIGS[name].replace(T=2)
    floor = PU.load_floor(f"{name}_T2")
    K_p, K_r = floor["K_p"], floor["K_r"]
    t0 = time.time()
    dev_w = I.device_weights(cfg)
    host_w = [{k: v.float().cpu().numpy() for k, v in w.items()} for w in dev_w]
    gpu = make_gpu(cfg, dev_w, K_p=K_p, K_r=K_r)
    nb = cfg.B if seqs is None else len(seqs)
    ora = O.CachedDenoiser(PU.oracle_model(cfg), host_w, nb, cfg.L_p, cfg.L_r, cfg.rho, K_p, K_r,
                           storage="bf16")
    sched = I.TokenSchedule(cfg, stress=True)
    stats = PU.ParityStats(floor=floor)
    for i in range(len(floor["step_kinds"])):
        PU.run_step_pair(cfg, gpu, ora, sched.hidden_in(i), i, stats, seqs=seqs)
        print(f"\n[{name}] step {i} [{floor['step_kinds'][i]}]: rel err {stats.rel_per_step[-1]:.3e}  "
              f"t={time.time() - t0:.1f}s", flush=True)
    PU.compare_caches(cfg, gpu, ora, stats, seqs=seqs, verbose=True)
    print(f"[{name}] selection exact={stats.exact} tied_same={stats.tied_same} followed={stats.followed}; "
          f"worst |ds| {stats.worst_score_dev:.2e}; worst distance / bar {stats.worst_over_bar:.2f}", flush=True)
    assert stats.failed == 0, stats.failures
    assert stats.exact > 0
    assert stats.worst_rel <= PU.stated_tol(cfg)
    gpu.close()


@pytest.mark.parametrize("name,layers", [("dream7b", 3), ("llada8b_long", 2), ("llada8b_b16", 2)])
def test_wide_shapes_properties_at_size(name, layers):
    """Reduced depth, full width and length: refresh == uncached forward on the GPU itself,
    bit-reproducibility, selection exactly the bottom-k of the GPU's scores, untouched rows."""
    cfg = I.CONFIGS[name].replace(T=layers)
    dev_w = I.device_weights(cfg)
    tdt = torch.bfloat16
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    h0 = torch.randn((cfg.B, cfg.n, cfg.d), device="cuda", generator=g).to(tdt)
    h1 = h0.clone()
    rows = torch.randperm(cfg.L_r, device="cuda", generator=g)[: cfg.L_r // 3] + cfg.L_p
    h1[:, rows] += 0.5 * torch.randn((cfg.B, rows.numel(), cfg.d), device="cuda", generator=g).to(tdt)

    runs = []
    for _ in range(2):
        den = make_gpu(cfg, dev_w, K_p=8, K_r=8)
        out0, _ = den.step(h0, 0)
        out0 = out0.clone()
        before = [den.read_cache(layers - 1, w).clone() for w in range(4)]
        out1, n_sel = den.step(h1, 1)
        torch.cuda.synchronize()
        sel = den.sel_idx[:, :, :n_sel].clone()
        scores = den.read_scores()
        after = [den.read_cache(layers - 1, w) for w in range(4)]
        torch.cuda.synchronize()
        runs.append((out0, out1.clone(), sel, scores.clone()))
        k = den.num_selected
        assert n_sel == k == O.num_selected(cfg.rho, cfg.L_r)
        sc_host, sel_host = scores.cpu().numpy().astype(np.float64), sel.cpu().numpy()
        for l in range(layers):
            for b in range(cfg.B):
                assert sel_host[l, b].tolist() == O.bottom_k(sc_host[l, b], k).tolist()
        for b in range(cfg.B):
            rest = np.setdiff1d(np.arange(cfg.L_r), sel_host[layers - 1, b]) + cfg.L_p
            for w in (0, 2, 3):
                assert torch.equal(after[w][b, rest], before[w][b, rest])
                assert torch.equal(after[w][b, :cfg.L_p], before[w][b, :cfg.L_p])
        den.close()
    assert all(torch.equal(a, b) for a, b in zip(runs[0], runs[1]))

    # a full-refresh step equals the uncached configuration (rho = 1, K_p = K_r = 1) bit for bit
    unc = make_gpu(cfg, dev_w, rho=1.0, K_p=1, K_r=1)
    u0, _ = unc.step(h0, 0)
    torch.cuda.synchronize()
    assert torch.equal(u0, runs[0][0])
    # and against the oracle on sampled rows of the first layer's V cache
    v_gpu = unc.read_cache(0, 1)[0].float().cpu().numpy()
    w0 = {k: v.float().cpu().numpy().astype(np.float64) for k, v in dev_w[0].items()}
    x = h0[0].float().cpu().numpy().astype(np.float64)
    sample = np.random.default_rng(0).permutation(cfg.n)[:64]
    hs = O.round_bf16(O.rmsnorm(x[sample], w0["attn_norm_g"], cfg.rms_eps))
    v_ref = O.round_bf16(hs @ w0["wv"].T)
    assert PU.rel_err(v_gpu[sample], v_ref) < 1e-3
    unc.close()


@pytest.mark.parametrize("name,M", [("llada8b", 256), ("llada8b", 4), ("dream7b", 100)])
def test_head_at_full_vocabulary_sampled_rows(name, M):
    """The mask-predictor head at the workload's vocabulary and width (126464 x 4096, 152064 x
    3584): every row's greedy token and confidence from the GPU, the oracle on sampled rows."""
    from oracle import dllm_generate_oracle as G
    cfg = I.CONFIGS[name]
    hw = I.device_head_weights(cfg)
    g = torch.Generator(device="cuda")
    g.manual_seed(cfg.seed + M)
    hidden = torch.randn((M + 5, cfg.d), dtype=torch.float32, device="cuda", generator=g).to(torch.bfloat16)
    rows = torch.randperm(M + 5, device="cuda", generator=g)[:M].to(torch.int32)
    x0, conf = binding.op_head(cfg.dtype, hidden, hw["final_norm_g"], hw["lm_head"], cfg.rms_eps, rows)
    torch.cuda.synchronize()
    x0, conf = x0.cpu().numpy(), conf.cpu().numpy().astype(np.float64)
    assert x0.min() >= 0 and x0.max() < cfg.vocab and np.all((conf > 0) & (conf <= 1))
    sample = np.unique(np.linspace(0, M - 1, 6).astype(int))
    hid = hidden.float().cpu().numpy()[rows.cpu().numpy()[sample]]
    gain = hw["final_norm_g"].float().cpu().numpy()
    logits = np.empty((sample.size, cfg.vocab))
    for v0 in range(0, cfg.vocab, 16384):     # the projection in slabs: 16384 x d float64 at a time
        w = hw["lm_head"][v0:v0 + 16384].float().cpu().numpy()
        logits[:, v0:v0 + w.shape[0]] = G.head_logits(hid, gain, w, cfg.rms_eps, "bf16")
    want_x0, want_conf = G.greedy_with_confidence(logits)
    for t, i in enumerate(sample):
        top = logits[t, want_x0[t]]
        assert x0[i] == want_x0[t] or top - logits[t, x0[i]] <= 2e-3, f"row {i}"
    assert np.allclose(conf[sample], want_conf, rtol=5e-3, atol=0), np.abs(conf[sample] / want_conf - 1).max()
    print(f"\n[head {name} M={M}] sampled rows {sample.tolist()}: tokens equal "
          f"{int(np.sum(x0[sample] == want_x0))}/{sample.size}, conf rel err "
          f"{np.abs(conf[sample] / want_conf - 1).max():.2e}", flush=True)


def test_llada8b_closed_loop_first_steps_match_oracle():
    """The closed loop at the headline size (32 layers, vocabulary 126464): a full-refresh step
    and an adaptive step driven by the model's own predictions, every decision checked by
    tests/test_gpu_generate.run_loop's rules against the oracle."""
    from oracle import dllm_generate_oracle as G
    from tests.test_gpu_generate import run_loop
    cfg = I.CONFIGS["llada8b"]
    floor = PU.load_floor("llada8b")
    t0 = time.time()
    dev_w = I.device_weights(cfg)
    host_w = [{k: v.float().cpu().numpy() for k, v in w.items()} for w in dev_w]
    hw = I.device_head_weights(cfg)
    host_hw = {k: v.float().cpu().numpy() for k, v in hw.items()}
    print(f"\n[fullsize loop] weights ready {time.time() - t0:.1f}s", flush=True)
    gpu = make_gpu(cfg, dev_w)
    ora = O.CachedDenoiser(PU.oracle_model(cfg), host_w, cfg.B, cfg.L_p, cfg.L_r, cfg.rho, cfg.K_p,
                           cfg.K_r, storage="bf16")
    ggen = binding.Generator(gpu, hw["embed"], hw["final_norm_g"], hw["lm_head"], cfg.steps)
    ogen = G.Generator(ora, host_hw["embed"], host_hw["final_norm_g"], host_hw["lm_head"], cfg.vocab,
                       cfg.steps)
    st, tally, tokens = run_loop(cfg, steps=2, loop=(gpu, ora, ggen, ogen), floor=floor)
    print(f"[fullsize loop] rel {st.worst_rel:.3e} {tally} selection exact/tied/followed/failed "
          f"{st.exact}/{st.tied_same}/{st.followed}/{st.failed}  t={time.time() - t0:.1f}s", flush=True)
    assert st.failed == 0, st.failures
    assert tally["tokens_exact"] > 0
    assert int(np.sum(tokens[:, cfg.L_p:] != cfg.vocab)) == 2 * cfg.B * (cfg.L_r // cfg.steps)
    ggen.close()
    gpu.close()
