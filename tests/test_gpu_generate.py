"""GPU parity of the closed denoising loop (embedding gather, cached step, mask-predictor head,
low-confidence remasking) against oracle/dllm_generate_oracle.py, through the C ABI.

Integer decisions (greedy token, revealed positions, the token update itself) are compared
exactly wherever the oracle's margin decides; inside a near-tie (top-2 logit gap or the
confidence gap at the reveal boundary within the band below) any admissible choice is accepted
and the oracle continues from the GPU's token state, so that later steps are compared on equal
terms.  Bands: the two sides' logits differ by float32-vs-float64 accumulation (1e-4 floor) and
by what the difference e of the step's output rows (relative, measured in the same step) does to
a logit: a perturbation of relative size e in a random direction moves a logit by about
e * sigma, sigma the spread of that row's logits; the band is 8 of those.  A confidence moves
by at most (exp(2 dl) - 1) of itself when every logit moves by dl.
"""
import numpy as np
import pytest
import torch

from oracle import dllm_cache_oracle as O
from oracle import dllm_generate_oracle as G
from paper_2506_06295_amd import binding, inputs as I
from tests import parity_util as PU
from tests.test_gpu_step import MINI_LLADA, MINI_LONG

pytestmark = pytest.mark.gpu


def logit_band(e_step, logits):
    return max(1e-4, 8.0 * e_step * float(np.std(logits)))


def conf_rel_tol(band):
    return max(5e-4, 4.0 * band)


# ---- the head as a single operation ---------------------------------------------------------

def head_case(dtype, M, vocab, d, gather, seed=0, dup=False, flat=False):
    r = np.random.default_rng(seed + M + vocab)
    rows_total = M + 11
    hidden = r.standard_normal((rows_total, d)).astype(np.float32)
    gain = (1.0 + 0.1 * r.standard_normal(d)).astype(np.float32)
    w = (0.05 * r.standard_normal((vocab, d))).astype(np.float32)
    if dtype == "bf16":
        hidden, gain, w = I.to_bf16_grid(hidden), I.to_bf16_grid(gain), I.to_bf16_grid(w)
    if dup:    # every logit appears twice: the lower id must win
        w[vocab // 2:2 * (vocab // 2)] = w[:vocab // 2]
    if flat:   # all logits equal: token 0 with probability 1/vocab
        w[:] = w[0]
    rows = r.permutation(rows_total)[:M].astype(np.int32) if gather else None
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    dev = lambda a: torch.from_numpy(a).cuda().to(tdt).contiguous()
    x0, conf = binding.op_head(dtype, dev(hidden), dev(gain), dev(w), 1e-5,
                               None if rows is None else torch.from_numpy(rows).cuda())
    torch.cuda.synchronize()
    x0, conf = x0.cpu().numpy().astype(np.int64), conf.cpu().numpy().astype(np.float64)
    src = hidden if rows is None else hidden[rows]
    logits = G.head_logits(src, gain, w, 1e-5, "bf16" if dtype == "bf16" else "f64")
    want_x0, want_conf = G.greedy_with_confidence(logits)
    return x0, conf, want_x0, want_conf, logits


@pytest.mark.parametrize("dtype,M,vocab,d,gather", [
    ("f32", 5, 1000, 96, False),      # plain GEMM kernel, vector path of the finalize
    ("f32", 9, 1001, 64, True),       # odd vocabulary: scalar path
    ("bf16", 70, 4096, 1024, True),   # streaming kernel, two row tiles
    ("bf16", 4, 4096, 512, False),    # a handful of rows (late steps of a generation)
    ("bf16", 256, 8192, 512, True),   # 128 x 128 LDS-direct kernel
    ("bf16", 200, 2432, 1024, False), # 19 column tiles: remapped part + tail of the tile order
])
def test_head_matches_oracle(dtype, M, vocab, d, gather):
    x0, conf, want_x0, want_conf, logits = head_case(dtype, M, vocab, d, gather)
    band = 1e-4 if dtype == "f32" else 2e-3   # single op: no depth amplification
    decided = 0
    for i in range(M):
        top = logits[i, want_x0[i]]
        if x0[i] == want_x0[i]:
            decided += 1
        else:
            assert top - logits[i, x0[i]] <= band, f"row {i}: token {x0[i]} is {top - logits[i, x0[i]]:.3e} below the maximum"
    assert decided >= M - max(1, M // 20)
    rtol = 5e-5 if dtype == "f32" else 5e-3
    assert np.allclose(conf, want_conf, rtol=rtol, atol=0), np.max(np.abs(conf / want_conf - 1))


@pytest.mark.parametrize("dtype,vocab", [("f32", 1000), ("f32", 1001), ("bf16", 4096)])
def test_head_exact_ties_go_to_the_lower_token(dtype, vocab):
    x0, conf, want_x0, want_conf, logits = head_case(dtype, 33, vocab, 128, False, dup=True)
    assert np.all(x0 < vocab // 2)
    assert np.array_equal(x0, want_x0)
    x0, conf, want_x0, want_conf, logits = head_case(dtype, 7, vocab, 128, False, flat=True)
    assert np.all(x0 == 0)
    assert np.allclose(conf, 1.0 / vocab, rtol=1e-5)


# ---- the closed loop -------------------------------------------------------------------------

def make_loop(cfg, block_len=0):
    ws = I.all_weights(cfg)
    gpu, ora = PU.make_pair(cfg, ws)
    hw = I.head_weights(cfg)
    dev = lambda a: PU.to_device(cfg, a)
    ggen = binding.Generator(gpu, dev(hw["embed"]), dev(hw["final_norm_g"]), dev(hw["lm_head"]),
                             cfg.steps, block_len)
    ogen = G.Generator(ora, hw["embed"], hw["final_norm_g"], hw["lm_head"], cfg.vocab, cfg.steps,
                       block_len or None)
    return gpu, ora, ggen, ogen


def run_loop(cfg, block_len=0, steps=None, loop=None, floor=None):
    """loop: (gpu, ora, ggen, ogen) built by the caller (full-size runs draw their weights on the
    device); floor: stored oracle-only noise floor of the model (default: measured on the fly)."""
    gpu, ora, ggen, ogen = loop if loop is not None else make_loop(cfg, block_len)
    tokens = I.initial_tokens(cfg)
    tok_dev = torch.from_numpy(tokens.astype(np.int32)).cuda()
    st = PU.ParityStats(floor=floor)
    tally = dict(tokens_exact=0, tokens_tied=0, reveal_exact=0, reveal_tied=0, worst_conf=0.0)
    L_p, L_r = cfg.L_p, cfg.L_r
    for i in range(steps or cfg.steps):
        before = tok_dev.clone()
        n_rev, n_sel = ggen.step(tok_dev, i)
        torch.cuda.synchronize()
        chk = PU.SelectionCheck(cfg, gpu, ora, i, n_sel, st)
        new_ora, rep = ogen.step(tokens, i, on_layer=chk.on_layer)
        chk.finish(ogen.embed[tokens], rep.step_report, rep.hidden_out)
        sel = chk.sel
        PU.check_selection_shape(cfg, ora, rep.step_report, sel, n_sel)
        assert n_rev == rep.n_unmask
        x0, conf, chosen, hout = ggen.read(hidden=True)
        torch.cuda.synchronize()
        x0, conf = x0.cpu().numpy().astype(np.int64), conf.cpu().numpy().astype(np.float64)
        chosen = chosen.cpu().numpy().astype(np.int64)[:, :n_rev]
        e = PU.check_tensor(st, cfg, f"step {i} hidden_out", hout.float().cpu().numpy(), rep.hidden_out,
                            st.current_floor()["hidden_out"], ceiling=PU.stated_tol(cfg))["frob"]
        st.worst_rel = max(st.worst_rel, e)
        new_gpu = tok_dev.cpu().numpy().astype(np.int64)
        old = before.cpu().numpy().astype(np.int64)
        assert np.array_equal(old, tokens)                     # both sides start the step equal
        for b in range(cfg.B):
            band = logit_band(e, rep.logits[b])
            elig = np.flatnonzero(tokens[b, L_p:][rep.lo:rep.hi] == cfg.vocab) + rep.lo
            other = np.setdiff1d(np.arange(L_r), elig)
            assert np.all(x0[b, other] == -1) and np.all(np.isneginf(conf[b, other]))
            # greedy tokens and confidences of the eligible positions
            for j in elig:
                top = rep.logits[b][j, rep.x0[b, j]]
                if x0[b, j] == rep.x0[b, j]:
                    tally["tokens_exact" if rep.logit_gap[b, j] > band else "tokens_tied"] += 1
                else:
                    assert top - rep.logits[b][j, x0[b, j]] <= band, f"step {i} seq {b} pos {j}: token not admissible"
                    tally["tokens_tied"] += 1
            rel = np.abs(conf[b, elig] / rep.conf[b, elig] - 1.0)
            tally["worst_conf"] = max(tally["worst_conf"], float(rel.max()))
            assert rel.max() <= conf_rel_tol(band), f"step {i} seq {b}: confidence off by {rel.max():.3e}"
            # revealed positions: exactly the top n of the GPU's own confidences (integer part) ...
            own = np.lexsort((elig, -conf[b, elig]))[:n_rev]
            assert chosen[b].tolist() == sorted(elig[own].tolist()), f"step {i} seq {b}: reveal selection"
            # ... and the oracle's set wherever its margin decides
            srt = np.sort(rep.conf[b, elig])[::-1]
            margin = (srt[n_rev - 1] - srt[n_rev]) if 0 < n_rev < elig.size else np.inf
            cband = 2.0 * float(np.max(np.abs(conf[b, elig] - rep.conf[b, elig])))
            if chosen[b].tolist() == rep.chosen[b].tolist():
                tally["reveal_exact" if margin > cband else "reveal_tied"] += 1
            else:
                assert margin <= cband, f"step {i} seq {b}: decisive margin {margin:.3e} but reveal sets differ"
                tau = srt[n_rev - 1]
                assert np.all(rep.conf[b, chosen[b]] >= tau - cband)
                assert set(elig[rep.conf[b, elig] > tau + cband].tolist()) <= set(chosen[b].tolist())
                tally["reveal_tied"] += 1
            # the update itself: chosen positions take the GPU's greedy token, nothing else moves
            want = old[b].copy()
            want[L_p + chosen[b]] = x0[b, chosen[b]]
            assert np.array_equal(new_gpu[b], want)
        tokens = new_gpu                                        # the oracle follows the GPU's state
    return st, tally, tokens


def test_closed_loop_toy_fp32():
    cfg = I.CONFIGS["toy"]
    st, tally, tokens = run_loop(cfg)
    print(f"\n[toy loop] rel {st.worst_rel:.2e} {tally} selection exact/tied/followed/failed "
          f"{st.exact}/{st.tied_same}/{st.followed}/{st.failed}")
    assert st.failed == 0, st.failures
    assert not np.any(tokens == cfg.vocab)
    assert tally["tokens_exact"] > 0 and tally["reveal_exact"] > 0


@pytest.mark.parametrize("block_len", [0, 8])
def test_closed_loop_toy_blocks(block_len):
    cfg = I.CONFIGS["toy"].replace(B=2)
    st, tally, tokens = run_loop(cfg, block_len)
    assert st.failed == 0, st.failures
    assert not np.any(tokens == cfg.vocab)


@pytest.mark.parametrize("cfg,block_len", [(MINI_LLADA, 0), (MINI_LLADA, 20), (MINI_LONG, 0)],
                         ids=["mini_llada", "mini_llada_blocks", "mini_long"])
def test_closed_loop_bf16(cfg, block_len):
    if cfg.L_r % max(block_len, 1) or (block_len and cfg.steps % (cfg.L_r // block_len)):
        pytest.skip("schedule does not divide")
    st, tally, tokens = run_loop(cfg, block_len)
    print(f"\n[{cfg.name} loop, block {block_len or cfg.L_r}] rel {st.worst_rel:.2e} {tally} selection "
          f"exact/tied/followed/failed {st.exact}/{st.tied_same}/{st.followed}/{st.failed}")
    assert st.failed == 0, st.failures
    assert not np.any(tokens == cfg.vocab)
    assert tally["tokens_exact"] > 0


def test_gen_argument_errors():
    cfg = I.CONFIGS["toy"]
    ws = I.all_weights(cfg)
    gpu, _ = PU.make_pair(cfg, ws)
    hw = I.head_weights(cfg)
    dev = lambda a: PU.to_device(cfg, a)
    e, g, w = dev(hw["embed"]), dev(hw["final_norm_g"]), dev(hw["lm_head"])
    with pytest.raises(binding.DllmcError):
        binding.Generator(gpu, e, g, w, cfg.steps, block_len=5)       # does not divide L_r
    with pytest.raises(binding.DllmcError):
        binding.Generator(gpu, e, g, w, 7, block_len=8)               # 4 blocks do not divide 7 steps
    gen = binding.Generator(gpu, e, g, w, cfg.steps)
    tok = torch.from_numpy(I.initial_tokens(cfg).astype(np.int32)).cuda()
    with pytest.raises(binding.DllmcError):
        gen.step(tok, cfg.steps)                                      # past the schedule
    with pytest.raises(binding.DllmcError):
        gen.step(tok, 3)                                              # step 0 first
    gen.close()
    gpu.close()
