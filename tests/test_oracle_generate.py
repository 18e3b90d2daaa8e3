"""Pins of the closed-loop oracle (oracle/dllm_generate_oracle.py), CPU only.

Each piece is checked against something other than itself: library routines (scipy softmax,
numpy argmax / sort), closed forms of the unmask schedule, a brute-force rewrite of the
transition on tiny inputs, and invariants of the loop that Sec. 3.1 fixes (fully masked start,
tokens only ever revealed, everything revealed after the last step).
"""
import itertools

import numpy as np
import pytest
from scipy.special import softmax

from oracle import dllm_cache_oracle as O
from oracle import dllm_generate_oracle as G
from paper_2506_06295_amd import inputs as I


def test_greedy_token_and_confidence_match_library_softmax():
    r = np.random.default_rng(0)
    logits = r.standard_normal((37, 501)) * 3.0
    x0, conf = G.greedy_with_confidence(logits)
    p = softmax(logits, axis=-1)
    assert np.array_equal(x0, np.argmax(p, axis=-1))
    assert np.allclose(conf, p.max(axis=-1), rtol=1e-12)
    assert np.allclose(conf, p[np.arange(37), x0], rtol=1e-12)


def test_greedy_ties_go_to_the_lower_token_id_and_shift_invariance():
    logits = np.array([[0.5, 2.0, 2.0, -1.0], [7.0, 7.0, 7.0, 7.0]])
    x0, conf = G.greedy_with_confidence(logits)
    assert x0.tolist() == [1, 0]
    assert np.isclose(conf[1], 0.25)
    x1, conf1 = G.greedy_with_confidence(logits + 1234.5)  # softmax is shift invariant, no overflow
    assert np.array_equal(x0, x1) and np.allclose(conf, conf1)
    one_hot = np.full((1, 9), -1e9)
    one_hot[0, 4] = 0.0
    assert G.greedy_with_confidence(one_hot)[1][0] == pytest.approx(1.0)


@pytest.mark.parametrize("block_len,spb", [(256, 64), (8, 8), (32, 5), (7, 3), (3, 7), (1, 1)])
def test_unmask_schedule_closed_form(block_len, spb):
    c = G.unmask_counts(block_len, spb)
    assert len(c) == spb and sum(c) == block_len
    assert all(a >= b for a, b in zip(c, c[1:]))           # remainder goes to the first steps
    assert max(c) - min(c) <= 1
    assert c == [(block_len + spb - 1 - t) // spb for t in range(spb)]  # ceil((L - t) / spb)


def test_block_of_step_walks_blocks_left_to_right():
    L_r, bl, steps = 32, 8, 16
    seen = []
    for i in range(steps):
        lo, hi, n = G.block_of_step(i, L_r, bl, steps)
        assert hi - lo == bl and lo == (i // 4) * bl and n == 2
        seen.append((lo, n))
    assert sum(n for _, n in seen) == L_r
    with pytest.raises(ValueError):
        G.block_of_step(0, 30, 8, 16)
    with pytest.raises(ValueError):
        G.block_of_step(0, 32, 8, 6)


def brute_transition(tokens, x0, conf, mask_id, lo, hi, n):
    """All subsets of the eligible positions of size n; the best one under the total order
    (higher confidence first, then lower position) compared element-wise after sorting."""
    elig = [j for j in range(lo, hi) if tokens[j] == mask_id]
    key = lambda j: (-conf[j], j)
    best = min((sorted(c, key=key) for c in itertools.combinations(elig, n)),
               key=lambda c: [key(j) for j in c])
    out = list(tokens)
    for j in best:
        out[j] = x0[j]
    return out, sorted(best)


@pytest.mark.parametrize("seed", range(6))
def test_transition_against_brute_force(seed):
    r = np.random.default_rng(seed)
    L, mask = 10, 99
    tokens = np.where(r.random(L) < 0.6, mask, r.integers(0, 50, L))
    x0 = r.integers(0, 50, L)
    conf = np.round(r.random(L), 1)          # coarse grid: exact ties occur
    lo, hi = 2, 9
    n_elig = int(np.sum(tokens[lo:hi] == mask))
    for n in range(0, n_elig + 1):
        got, chosen = G.low_confidence_transition(tokens, x0, conf, mask, lo, hi, n)
        want, want_chosen = brute_transition(tokens.tolist(), x0.tolist(), conf.tolist(), mask, lo, hi, n)
        assert got.tolist() == want and chosen.tolist() == want_chosen
    with pytest.raises(ValueError):
        G.low_confidence_transition(tokens, x0, conf, mask, lo, hi, n_elig + 1)


def test_transition_invariants():
    r = np.random.default_rng(3)
    L, mask = 64, 1000
    tokens = np.where(r.random(L) < 0.7, mask, r.integers(0, 900, L))
    x0, conf = r.integers(0, 900, L), r.random(L)
    lo, hi, n = 16, 48, 5
    got, chosen = G.low_confidence_transition(tokens, x0, conf, mask, lo, hi, n)
    assert chosen.size == n and np.all((chosen >= lo) & (chosen < hi))
    assert np.all(tokens[chosen] == mask) and np.array_equal(got[chosen], x0[chosen])
    untouched = np.setdiff1d(np.arange(L), chosen)
    assert np.array_equal(got[untouched], tokens[untouched])   # revealed tokens frozen, rest still masked
    # every position passed over is no more confident than every chosen one
    passed = [j for j in range(lo, hi) if tokens[j] == mask and j not in set(chosen.tolist())]
    assert max(conf[passed]) <= min(conf[chosen])
    # a block covering everything is plain global top-n over the masked positions
    g2, c2 = G.low_confidence_transition(tokens, x0, conf, mask, 0, L, n)
    masked = np.flatnonzero(tokens == mask)
    assert c2.tolist() == sorted(masked[np.argsort(-conf[masked], kind="stable")[:n]].tolist())


def toy_generator(rho, K_p, K_r, block_len=None, storage="f64"):
    cfg = I.CONFIGS["toy"]
    ws = [{k: np.asarray(v, dtype=np.float64) for k, v in w.items()} for w in I.all_weights(cfg)]
    mo = O.Model(cfg.T, cfg.d, cfg.H_q, cfg.H_kv, cfg.d_h, cfg.m, cfg.rms_eps, cfg.rope_theta)
    den = O.CachedDenoiser(mo, ws, cfg.B, cfg.L_p, cfg.L_r, rho, K_p, K_r, storage=storage)
    hw = I.head_weights(cfg)
    gen = G.Generator(den, hw["embed"], hw["final_norm_g"], hw["lm_head"], cfg.vocab, cfg.steps, block_len)
    return cfg, mo, ws, hw, gen


@pytest.mark.parametrize("block_len", [None, 8])
def test_loop_reveals_tokens_monotonically_and_finishes(block_len):
    cfg, mo, ws, hw, gen = toy_generator(0.25, 4, 2, block_len)
    tokens = I.initial_tokens(cfg)
    assert np.all(tokens[:, cfg.L_p:] == cfg.vocab)            # fully masked start (Sec. 3.1)
    prompt = tokens[:, :cfg.L_p].copy()
    for i in range(cfg.steps):
        new, rep = gen.step(tokens, i)
        was_masked = tokens[:, cfg.L_p:] == cfg.vocab
        now_masked = new[:, cfg.L_p:] == cfg.vocab
        assert np.array_equal(new[:, :cfg.L_p], prompt)
        assert np.all(new[:, cfg.L_p:][~was_masked] == tokens[:, cfg.L_p:][~was_masked])
        assert int(np.sum(was_masked) - np.sum(now_masked)) == cfg.B * rep.n_unmask
        for b in range(cfg.B):
            ch = rep.chosen[b]
            assert np.all((ch >= rep.lo) & (ch < rep.hi))
            assert np.array_equal(new[b, cfg.L_p + ch], rep.x0[b, ch])
            assert np.all((rep.conf[b] > 0) & (rep.conf[b] <= 1))
            assert np.all(rep.x0[b] < cfg.vocab)               # the mask id is never predicted
        tokens = new
    assert not np.any(tokens == cfg.vocab)                      # everything revealed at the end


def test_uncached_loop_feeds_the_head_the_plain_forward():
    """rho = 1, K_p = K_r = 1: the hidden rows behind every prediction are the uncached
    forward of the embedded tokens, so greedy tokens follow from library pieces alone."""
    cfg, mo, ws, hw, gen = toy_generator(1.0, 1, 1)
    tokens = I.initial_tokens(cfg)
    for i in range(3):
        hidden = np.asarray(hw["embed"], dtype=np.float64)[tokens]
        ref = O.uncached_forward(mo, ws, hidden, "f64", np.float64)
        z = ref[:, cfg.L_p:] / np.sqrt(np.mean(ref[:, cfg.L_p:] ** 2, axis=-1, keepdims=True) + cfg.rms_eps)
        p = softmax(z @ np.asarray(hw["lm_head"], dtype=np.float64).T, axis=-1)
        new, rep = gen.step(tokens, i)
        assert np.array_equal(rep.x0, np.argmax(p, axis=-1))
        assert np.allclose(rep.conf, p.max(axis=-1), rtol=1e-9)
        tokens = new


def test_forced_decisions_are_followed():
    cfg, mo, ws, hw, gen = toy_generator(0.25, 4, 2)
    tokens = I.initial_tokens(cfg)
    forced = [np.array([3, 5, 7, 11])]
    new, rep = gen.step(tokens, 0, forced_chosen=forced)
    assert rep.chosen[0].tolist() == [3, 5, 7, 11]
    assert np.array_equal(new[0, cfg.L_p + forced[0]], rep.x0[0, forced[0]])
    assert int(np.sum(new[0, cfg.L_p:] != cfg.vocab)) == 4
