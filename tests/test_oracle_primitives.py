"""Pins for the oracle's building blocks (CPU only).

Each check ties a function of oracle/dllm_cache_oracle.py to something that is
not the oracle itself: a torch library routine, a closed form, an identity, or
a brute-force loop on tiny inputs.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import dllm_cache_oracle as O


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- bf16 grid
def test_round_bf16_matches_torch_conversion():
    a = rng(0).standard_normal(20000).astype(np.float32) * np.float32(3.0)
    a = np.concatenate([a, np.float32([0.0, -0.0, 1e-30, 3.3e38, -3.3e38, 65504.0])])
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = O.round_bf16(a)
    assert got.dtype == np.float32
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_round_bf16_ties_to_even_known_values():
    # bf16 has 7 fraction bits: spacing 2^-7 in [1, 2)
    assert O.round_bf16(np.float64([1.0 + 2.0 ** -8]))[0] == 1.0            # tie -> even (1.0)
    assert O.round_bf16(np.float64([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6   # tie -> even
    assert O.round_bf16(np.float64([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    assert O.round_bf16(np.float64([-2.5]))[0] == -2.5


# ---------------------------------------------------------------- rmsnorm
def test_rmsnorm_matches_torch_rms_norm():
    x = rng(1).standard_normal((7, 96))
    g = rng(2).standard_normal(96)
    want = F.rms_norm(torch.from_numpy(x), (96,), weight=torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(O.rmsnorm(x, g, 1e-5), want, rtol=1e-13, atol=1e-13)


def test_rmsnorm_unit_rms_and_scale_invariance():
    x = rng(3).standard_normal((5, 64))
    y = O.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=1)), 1.0, atol=1e-14)
    assert np.allclose(O.rmsnorm(7.5 * x, np.ones(64), 0.0), y, atol=1e-13)


# ---------------------------------------------------------------- RoPE
def rope_complex(x, pos, d_h, theta):
    """Independent formulation: pair (t, t+d_h/2) as a complex number times e^{i pos w_t}."""
    rows, width = x.shape
    H, half = width // d_h, d_h // 2
    xt = torch.from_numpy(x).reshape(rows, H, d_h)
    z = torch.complex(xt[..., :half], xt[..., half:])
    w = torch.tensor([theta ** (-2.0 * t / d_h) for t in range(half)], dtype=torch.float64)
    ang = torch.from_numpy(np.asarray(pos, dtype=np.float64))[:, None] * w[None, :]
    z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1).reshape(rows, width).numpy()


def test_rope_matches_complex_rotation():
    x = rng(4).standard_normal((9, 3 * 16))
    pos = np.array([0, 1, 2, 5, 17, 100, 511, 768, 4607])
    assert np.allclose(O.rope(x, pos, 16, 10000.0), rope_complex(x, pos, 16, 10000.0),
                       rtol=1e-12, atol=1e-12)


def test_rope_closed_form_two_dims():
    # d_h = 2: a single pair rotated by angle pos * theta^0 = pos
    x = np.array([[1.0, 0.0], [0.0, 1.0]])
    out = O.rope(x, np.array([0.5, 0.5]), 2, 10000.0)
    assert np.allclose(out[0], [math.cos(0.5), math.sin(0.5)])
    assert np.allclose(out[1], [-math.sin(0.5), math.cos(0.5)])


def test_rope_position_zero_is_identity_and_norm_preserved():
    x = rng(5).standard_normal((4, 64))
    assert np.allclose(O.rope(x, np.zeros(4), 32, 10000.0), x)
    y = O.rope(x, np.array([3, 77, 1000, 4000]), 32, 10000.0)
    assert np.allclose(np.linalg.norm(y.reshape(4, 2, 32), axis=-1),
                       np.linalg.norm(x.reshape(4, 2, 32), axis=-1))


def test_rope_inner_product_depends_on_relative_position_only():
    q = rng(6).standard_normal((1, 32))
    k = rng(7).standard_normal((1, 32))
    def ip(pq, pk):
        return (O.rope(q, np.array([pq]), 32, 10000.0) @ O.rope(k, np.array([pk]), 32, 10000.0).T).item()
    assert abs(ip(10, 3) - ip(107, 100)) < 1e-10
    assert abs(ip(10, 3) - ip(3, 10)) > 1e-3  # and it is not symmetric in the offset's sign


# ---------------------------------------------------------------- attention
def brute_attention(Q, K, V, H_q, H_kv, d_h):
    q, n = len(Q), len(K)
    out = [[0.0] * (H_q * d_h) for _ in range(q)]
    for a in range(H_q):
        kv = a // (H_q // H_kv)
        for i in range(q):
            logit = []
            for j in range(n):
                acc = 0.0
                for t in range(d_h):
                    acc += Q[i][a * d_h + t] * K[j][kv * d_h + t]
                logit.append(acc / math.sqrt(d_h))
            mx = max(logit)
            w = [math.exp(v - mx) for v in logit]
            z = sum(w)
            for t in range(d_h):
                out[i][a * d_h + t] = sum(w[j] * V[j][kv * d_h + t] for j in range(n)) / z
    return np.array(out)


@pytest.mark.parametrize("H_q,H_kv", [(2, 2), (4, 2), (4, 1)])
def test_attention_matches_brute_force_loops(H_q, H_kv):
    d_h, q, n = 4, 3, 7
    r = rng(8)
    Q = r.standard_normal((q, H_q * d_h))
    K = r.standard_normal((n, H_kv * d_h))
    V = r.standard_normal((n, H_kv * d_h))
    want = brute_attention(Q.tolist(), K.tolist(), V.tolist(), H_q, H_kv, d_h)
    assert np.allclose(O.attention(Q, K, V, H_q, H_kv, d_h), want, rtol=1e-12, atol=1e-12)


def test_attention_matches_torch_sdpa_with_grouped_heads():
    H_q, H_kv, d_h, q, n = 8, 2, 16, 5, 33
    r = rng(9)
    Q = r.standard_normal((q, H_q * d_h))
    K = r.standard_normal((n, H_kv * d_h))
    V = r.standard_normal((n, H_kv * d_h))
    tq = torch.from_numpy(Q).reshape(1, q, H_q, d_h).transpose(1, 2)
    tk = torch.from_numpy(K).reshape(1, n, H_kv, d_h).transpose(1, 2)
    tv = torch.from_numpy(V).reshape(1, n, H_kv, d_h).transpose(1, 2)
    want = F.scaled_dot_product_attention(tq, tk, tv, enable_gqa=True)
    want = want.transpose(1, 2).reshape(q, H_q * d_h).numpy()
    assert np.allclose(O.attention(Q, K, V, H_q, H_kv, d_h), want, rtol=1e-11, atol=1e-12)


def test_attention_uniform_when_keys_equal_and_is_order_free():
    # identical keys -> output is the mean of the values; permuting keys changes nothing
    r = rng(10)
    Q = r.standard_normal((2, 8))
    K = np.tile(r.standard_normal((1, 8)), (6, 1))
    V = r.standard_normal((6, 8))
    out = O.attention(Q, K, V, 1, 1, 8)
    assert np.allclose(out, np.tile(V.mean(axis=0), (2, 1)))
    K2 = r.standard_normal((6, 8))
    perm = r.permutation(6)
    assert np.allclose(O.attention(Q, K2, V, 1, 1, 8), O.attention(Q, K2[perm], V[perm], 1, 1, 8))


# ---------------------------------------------------------------- SiLU
def test_silu_matches_torch():
    x = np.linspace(-30, 30, 301)
    assert np.allclose(O.silu(x), F.silu(torch.from_numpy(x)).numpy(), rtol=1e-13, atol=1e-300)
    assert O.silu(np.array([0.0]))[0] == 0.0


# ---------------------------------------------------------------- cosine score
def test_cosine_identities():
    r = rng(11)
    u = r.standard_normal((6, 40))
    assert np.allclose(O.cosine_scores(u, u), 1.0, atol=1e-15)
    assert np.allclose(O.cosine_scores(u, -u), -1.0, atol=1e-15)
    e = np.eye(40)[:6]
    assert np.allclose(O.cosine_scores(e, np.roll(e, 1, axis=1)), 0.0)
    v = r.standard_normal((6, 40))
    base = O.cosine_scores(u, v)
    assert np.allclose(O.cosine_scores(3.0 * u, 0.25 * v), base)
    assert np.allclose(O.cosine_scores(-2.0 * u, 5.0 * v), -base)
    # 3-4-5 triangle: cos between (1,0) and (3,4) is 0.6
    assert np.allclose(O.cosine_scores(np.array([[1.0, 0.0]]), np.array([[3.0, 4.0]])), 0.6)


def test_cosine_matches_torch_and_zero_row_scores_zero():
    r = rng(12)
    u, v = r.standard_normal((9, 64)), r.standard_normal((9, 64))
    want = F.cosine_similarity(torch.from_numpy(u), torch.from_numpy(v), dim=1, eps=1e-8).numpy()
    assert np.allclose(O.cosine_scores(u, v), want, rtol=1e-13)
    u[3] = 0.0
    assert O.cosine_scores(u, v)[3] == 0.0


# ---------------------------------------------------------------- selection
def brute_bottom_k(scores, k):
    order = sorted(range(len(scores)), key=lambda j: (scores[j], j))
    return sorted(order[:k])


def test_num_selected_is_floor_of_rho_times_response_length():
    assert O.num_selected(0.25, 32) == 8
    assert O.num_selected(0.25, 256) == 64
    assert O.num_selected(0.1, 512) == 51      # floor(51.2)
    assert O.num_selected(0.05, 256) == 12     # floor(12.8)
    assert O.num_selected(0.5, 256) == 128
    assert O.num_selected(1.0, 256) == 256
    assert O.num_selected(0.0, 256) == 0
    assert O.num_selected(0.3, 10) == 3        # 0.3*10 = 2.9999999999999996 in binary64


@pytest.mark.parametrize("seed", range(6))
def test_bottom_k_matches_full_sort_with_ties(seed):
    r = rng(100 + seed)
    L = int(r.integers(1, 70))
    # few distinct values -> many exact ties
    s = r.integers(0, 5, size=L).astype(np.float64) / 4.0
    for k in {0, 1, L // 4, L // 2, L - 1, L} - {-1}:
        if 0 <= k <= L:
            assert O.bottom_k(s, k).tolist() == brute_bottom_k(s.tolist(), k)


def test_bottom_k_picks_changed_rows_and_breaks_ties_low():
    s = np.ones(16)
    s[[11, 3]] = [0.2, -0.5]
    assert O.bottom_k(s, 2).tolist() == [3, 11]
    assert O.bottom_k(s, 4).tolist() == [0, 1, 3, 11]   # two of the tied ones: lowest indices
    assert O.bottom_k(np.ones(8), 3).tolist() == [0, 1, 2]


def test_boundary_gap_is_margin_between_kth_and_next():
    s = np.array([0.9, 0.1, 0.5, 0.7])
    assert O.boundary_gap(s, 2) == pytest.approx(0.2)   # sorted: .1 .5 | .7 .9
    assert O.boundary_gap(s, 0) == float("inf") and O.boundary_gap(s, 4) == float("inf")


def test_selection_admissibility_band():
    s = np.array([0.10, 0.50, 0.50005, 0.9, 0.95])
    assert O.selection_is_admissible(s, 2, np.array([0, 1]))
    assert O.selection_is_admissible(s, 2, np.array([0, 2]))      # near-tie inside the band
    assert not O.selection_is_admissible(s, 2, np.array([0, 3]))  # clearly above the cut
    assert not O.selection_is_admissible(s, 2, np.array([1, 2]))  # misses a clear member
    assert not O.selection_is_admissible(s, 2, np.array([0, 0]))
