"""Pins of the selection / update variants the paper compares against its default (Sec. 4.3
selection strategies; appendix "Impact of Similarity Metric", "Design Choice Between Full
V-Cache Overwrite and Selective Update"), CPU only."""
import numpy as np
import pytest

from oracle import dllm_cache_oracle as O
from paper_2506_06295_amd import inputs as I
from tests.test_oracle_cache_rules import make, small_cfg


def test_l2_scores_are_minus_the_library_norm():
    r = np.random.default_rng(0)
    a, b = r.standard_normal((40, 33)), r.standard_normal((40, 33))
    s = O.l2_scores(a, b)
    assert np.allclose(s, -np.linalg.norm(a - b, axis=1), rtol=1e-13)
    assert np.all(O.l2_scores(a, a) == 0.0)
    assert np.allclose(O.l2_scores(a, b), O.l2_scores(b, a))
    # scaling both rows scales the distance; the cosine would not move
    assert np.allclose(O.l2_scores(3 * a, 3 * b), 3 * s)
    # the row that moved farthest has the lowest score and is selected first
    c = a.copy()
    c[7] += 100.0
    assert O.bottom_k(O.l2_scores(c, a), 1).tolist() == [7]


def test_fmix32_is_a_bijection_with_avalanche():
    xs = np.arange(1 << 16, dtype=np.uint64)
    hs = np.array([O._fmix32(int(x)) for x in xs], dtype=np.uint64)
    assert np.unique(hs).size == xs.size                      # no collisions on consecutive inputs
    assert O._fmix32(0) == 0                                  # the one fixed point every xor-shift-multiply mix has
    # known values of MurmurHash3's 32-bit finalizer
    assert O._fmix32(1) == 0x514E28B7 and O._fmix32(0xFFFFFFFF) == 0x81F16F39
    # flipping one input bit flips about half of the output bits
    flips = []
    for bit in range(32):
        d = np.array([O._fmix32(int(x) ^ (1 << bit)) for x in xs[:2048]], dtype=np.uint64) ^ hs[:2048]
        flips.append(np.mean([bin(int(v)).count("1") for v in d]))
    assert 14.0 < min(flips) and max(flips) < 18.0


def test_random_scores_are_uniform_and_keyed():
    s = np.concatenate([O.random_scores(123, st, l, b, 256) for st in range(8) for l in range(4) for b in range(2)])
    assert s.min() >= 0.0 and s.max() < 1.0
    assert np.all(s * 2 ** 24 == np.floor(s * 2 ** 24))       # 24-bit grid: exact in float32
    counts, _ = np.histogram(s, bins=16, range=(0, 1))
    expected = s.size / 16
    assert np.sum((counts - expected) ** 2 / expected) < 40.0   # chi-square, 15 dof: p ~ 4e-4
    base = O.random_scores(123, 3, 1, 0, 64)
    assert np.array_equal(base, O.random_scores(123, 3, 1, 0, 64))
    for other in (O.random_scores(124, 3, 1, 0, 64), O.random_scores(123, 4, 1, 0, 64),
                  O.random_scores(123, 3, 2, 0, 64), O.random_scores(123, 3, 1, 1, 64)):
        assert not np.array_equal(base, other)
    # every position is selected with probability k / L_r
    hits = np.zeros(32)
    trials = 4000
    for t in range(trials):
        hits[O.bottom_k(O.random_scores(7, t, 0, 0, 32), 8)] += 1
    assert np.all(np.abs(hits / trials - 0.25) < 0.04)


def test_random_selection_ignores_the_activations_and_follows_the_hash():
    cfg = small_cfg(K_p=8, K_r=8, L_r=16, rho=0.25)
    ws = I.all_weights(cfg)
    den = make(cfg, ws, selection="random", seed=99)
    sched = I.TokenSchedule(cfg, stress=True)
    den.step(sched.hidden_in(0).astype(np.float64), 0)
    _, rep = den.step(sched.hidden_in(1).astype(np.float64), 1)
    for l in range(cfg.T):
        want = O.bottom_k(O.random_scores(99, 1, l, 0, cfg.L_r), den.k_sel)
        assert rep.selected[l][0].tolist() == want.tolist()


def test_l2_policy_selects_by_distance():
    cfg = small_cfg(K_p=8, K_r=8, L_r=16, rho=0.25)
    ws = I.all_weights(cfg)
    den = make(cfg, ws, metric="l2")
    sched = I.TokenSchedule(cfg, stress=True)
    den.step(sched.hidden_in(0).astype(np.float64), 0)
    v_before = [v.copy() for v in den.V]
    _, rep = den.step(sched.hidden_in(1).astype(np.float64), 1)
    # layer 0: V_new is a function of the input alone, so the scores can be recomputed from the caches
    d = np.linalg.norm(den.V[0][0, cfg.L_p:] - v_before[0][0, cfg.L_p:], axis=1)
    assert np.allclose(rep.scores[0][0], -d, rtol=1e-12)
    assert rep.selected[0][0].tolist() == sorted(np.lexsort((np.arange(cfg.L_r), -d))[:den.k_sel].tolist())


def test_selected_only_v_update_keeps_the_other_rows():
    cfg = small_cfg(K_p=8, K_r=8, L_r=16, rho=0.25)
    ws = I.all_weights(cfg)
    sel_only, full = make(cfg, ws, v_update="selected"), make(cfg, ws)
    sched = I.TokenSchedule(cfg, stress=True)
    for den in (sel_only, full):
        den.step(sched.hidden_in(0).astype(np.float64), 0)
    assert all(np.array_equal(a, b) for a, b in zip(sel_only.V, full.V))     # refresh steps are identical
    v_before = [v.copy() for v in sel_only.V]
    _, rep = sel_only.step(sched.hidden_in(1).astype(np.float64), 1)
    full.step(sched.hidden_in(1).astype(np.float64), 1)
    for l in range(cfg.T):
        S = rep.selected[l][0]
        rest = np.setdiff1d(np.arange(cfg.L_r), S)
        assert np.array_equal(sel_only.V[l][0, cfg.L_p + rest], v_before[l][0, cfg.L_p + rest])
        assert not np.array_equal(sel_only.V[l][0, cfg.L_p + S], v_before[l][0, cfg.L_p + S])
    # layer 0 sees the same input and the same cache in both variants: same selection, and the
    # selected rows' new Values equal the whole-overwrite variant's
    S0 = rep.selected[0][0]
    assert np.array_equal(sel_only.V[0][0, cfg.L_p + S0], full.V[0][0, cfg.L_p + S0])
    # rho = 1 selects everything: the two variants coincide
    a, b = make(cfg, ws, rho=1.0, v_update="selected"), make(cfg, ws, rho=1.0)
    for i in range(3):
        oa, _ = a.step(sched.hidden_in(i).astype(np.float64), i)
        ob, _ = b.step(sched.hidden_in(i).astype(np.float64), i)
        assert np.array_equal(oa, ob)


def test_unknown_policy_is_rejected():
    cfg = small_cfg()
    with pytest.raises(ValueError):
        make(cfg, I.all_weights(cfg), metric="manhattan")


def test_k_verify_is_the_mirror_image_of_v_verify():
    cfg = small_cfg(K_p=8, K_r=8, L_r=16, rho=0.25)
    ws = I.all_weights(cfg)
    kv, vv = make(cfg, ws, source="k"), make(cfg, ws)
    sched = I.TokenSchedule(cfg, stress=True)
    o_k, _ = kv.step(sched.hidden_in(0).astype(np.float64), 0)
    o_v, _ = vv.step(sched.hidden_in(0).astype(np.float64), 0)
    assert np.array_equal(o_k, o_v)                       # refresh steps do not depend on the variant
    k_before = [k.copy() for k in kv.K]
    v_before = [v.copy() for v in kv.V]
    _, rep = kv.step(sched.hidden_in(1).astype(np.float64), 1)
    # layer 0: the scores are the cosines between the Keys now in the cache and those before
    s0 = O.cosine_scores(kv.K[0][0, cfg.L_p:], k_before[0][0, cfg.L_p:])
    assert np.allclose(rep.scores[0][0], s0, rtol=1e-12)
    assert rep.selected[0][0].tolist() == O.bottom_k(s0, kv.k_sel).tolist()
    for l in range(cfg.T):
        S = rep.selected[l][0]
        rest = np.setdiff1d(np.arange(cfg.L_r), S)
        # every response Key is rewritten, Values only for the selected rows
        assert not np.any(np.all(kv.K[l][0, cfg.L_p:] == k_before[l][0, cfg.L_p:], axis=1))
        assert np.array_equal(kv.V[l][0, cfg.L_p + rest], v_before[l][0, cfg.L_p + rest])
        assert not np.array_equal(kv.V[l][0, cfg.L_p + S], v_before[l][0, cfg.L_p + S])
        # the prompt side is untouched on a step that does not refresh it
        assert np.array_equal(kv.K[l][0, :cfg.L_p], k_before[l][0, :cfg.L_p])
    # the rotation does not change a row's norm, so the cached Keys have the norms of the plain projection
    mo = kv.model
    x = sched.hidden_in(1).astype(np.float64)[0, cfg.L_p:]
    h = O.rmsnorm(x, np.asarray(ws[0]["attn_norm_g"], dtype=np.float64), mo.rms_eps)
    plain = h @ np.asarray(ws[0]["wk"], dtype=np.float64).T
    assert np.allclose(np.linalg.norm(kv.K[0][0, cfg.L_p:], axis=1), np.linalg.norm(plain, axis=1), rtol=1e-12)


def test_k_verify_with_every_row_selected_equals_the_default():
    cfg = small_cfg(K_p=3, K_r=4, L_r=16, rho=1.0)
    ws = I.all_weights(cfg)
    a, b = make(cfg, ws, source="k"), make(cfg, ws)
    sched = I.TokenSchedule(cfg, stress=True)
    for i in range(6):
        oa, _ = a.step(sched.hidden_in(i).astype(np.float64), i)
        ob, _ = b.step(sched.hidden_in(i).astype(np.float64), i)
        assert np.allclose(oa, ob, rtol=1e-12, atol=1e-12)
    assert a.macs == b.macs


# ---- update ratio per layer (appendix "Layer-wise token selection" / cross-layer allocation) ----
def test_linear_allocation_matches_the_table_ends_and_budget():
    for first, last in ((0.375, 0.125), (0.125, 0.375)):
        for T in (2, 3, 28, 32):
            r = O.linear_rho_allocation(T, first, last)
            assert len(r) == T and r[0] == first and r[-1] == pytest.approx(last)
            assert np.mean(r) == pytest.approx(0.25)                 # the table's common budget
            steps = np.diff(r)
            assert np.allclose(steps, steps[0]) and np.sign(steps[0]) == np.sign(last - first)
    assert O.linear_rho_allocation(1, 0.375, 0.125) == [0.25]
    assert O.linear_rho_allocation(5, 0.25, 0.25) == [0.25] * 5
    # the front-heavy and the back-heavy allocation are each other's reversal
    a, b = O.linear_rho_allocation(32, 0.375, 0.125), O.linear_rho_allocation(32, 0.125, 0.375)
    assert np.allclose(a, b[::-1])


def test_equal_ratios_per_layer_reproduce_the_global_ratio():
    cfg = small_cfg(T=3, K_p=4, K_r=3, L_r=16, rho=0.25)
    ws = I.all_weights(cfg)
    a, b = make(cfg, ws, rho_layers=[0.25] * 3), make(cfg, ws)
    sched = I.TokenSchedule(cfg, stress=True)
    for i in range(6):
        oa, ra = a.step(sched.hidden_in(i).astype(np.float64), i)
        ob, rb = b.step(sched.hidden_in(i).astype(np.float64), i)
        assert np.array_equal(oa, ob)
        assert all(np.array_equal(x[0], y[0]) for x, y in zip(ra.selected, rb.selected))
    with pytest.raises(ValueError):
        make(cfg, ws, rho_layers=[0.25, 0.25])
    with pytest.raises(ValueError):
        make(cfg, ws, rho_layers=[0.25, 1.5, 0.0])


def test_each_layer_recomputes_its_own_share():
    cfg = small_cfg(T=4, K_p=8, K_r=8, L_r=16, rho=0.25)
    ws = I.all_weights(cfg)
    ratios = [0.5, 0.0, 1.0, 0.13]
    den = make(cfg, ws, rho_layers=ratios)
    ref_full = make(cfg, ws, rho=1.0)           # recomputes every response row at every layer
    sched = I.TokenSchedule(cfg, stress=True)
    for d in (den, ref_full):
        d.step(sched.hidden_in(0).astype(np.float64), 0)
    before = {name: [c.copy() for c in getattr(den, name)] for name in ("K", "V", "AttnOut", "FFNOut")}
    macs0 = den.macs
    _, rep = den.step(sched.hidden_in(1).astype(np.float64), 1)
    ref_full.step(sched.hidden_in(1).astype(np.float64), 1)
    Lp, Lr = cfg.L_p, cfg.L_r
    assert [rep.selected[l][0].size for l in range(4)] == [8, 0, 16, 2]   # floor(rho_l * 16)
    for l in range(4):
        S = rep.selected[l][0]
        rest = np.setdiff1d(np.arange(Lr), S)
        for name in ("K", "AttnOut", "FFNOut"):
            now, old = getattr(den, name)[l][0, Lp:], before[name][l][0, Lp:]
            assert np.array_equal(now[rest], old[rest])
            assert not np.any(np.all(now[S] == old[S], axis=1))
        # V is overwritten for the whole response at every layer, whatever its ratio
        assert not np.any(np.all(den.V[l][0, Lp:] == before["V"][l][0, Lp:], axis=1))
    # layer 0 sees the step's input: its selected rows' Keys equal a full recomputation's
    S0 = rep.selected[0][0]
    assert np.array_equal(den.K[0][0, Lp + S0], ref_full.K[0][0, Lp + S0])
    # multiply-accumulates of the step: V for all rows plus Q, K, attention, O, FFN per selected row
    mo = den.model
    per_row = mo.d * (mo.d_q + mo.d_kv) + 2 * cfg.n * mo.d_q + mo.d_q * mo.d + 3 * mo.d * mo.m
    want = sum(Lr * mo.d * mo.d_kv + k * per_row for k in (8, 0, 16, 2))
    assert den.macs - macs0 == want
    # a refresh step ignores the ratios
    _, rep8 = den.step(sched.hidden_in(8 % cfg.steps).astype(np.float64), 8)
    assert all(rep8.selected[l][0].size == Lr for l in range(4))
