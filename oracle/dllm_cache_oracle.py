"""CPU oracle for the dLLM-Cache denoising step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, by-eye-checkable numpy implementation of what the cached
bidirectional-transformer denoising step computes.  Only tests, the smoke check
and the benchmark's CPU-baseline leg may import it; the product (the HIP
library and its Python binding) never does, and this file imports nothing from
the product.

What it follows
---------------
* Cache contents and schedule: Sec. 3.2 ("Initialization", "Iterative Steps"),
  Sec. 3.2.1 (prompt cache) and Sec. 3.2.2 (response cache: full refresh,
  adaptive partial update with the V-verify score of Eq. (cos_sim), bottom
  floor(rho*|y|) selection, whole-V overwrite, K / AttnOut / FFNOut scattered
  for the selected rows only).
* Per-layer selection and the boundary margin Delta: appendix "Cross-Layer
  Behavior of Token Selection".
* Cost model: appendix "Complexity and Latency Analysis"; storage: appendix
  "Proof of Storage Overhead of Caching".
* The transformer block itself (pre-RMSNorm, rotate-half RoPE, bidirectional
  softmax attention with optional grouped KV heads, SwiGLU) is the architecture
  named by the workloads; the paper only names "bidirectional attention" and
  the three SwiGLU matmuls.

Arithmetic is float64 by default.  `storage="bf16_cache"` rounds only what is
written into a cache and the step's output (the narrowest reading of the
paper's bf16 caches).  `storage="bf16"` rounds every tensor that a
bf16 implementation materialises (normed rows, Q, K, V, attention rows,
AttnOut, FFN-normed rows, the SwiGLU product, FFNOut, the step's output) to the
bf16 grid once, at the point it is produced; the residual stream inside a step
and all accumulations stay in the working precision.  The paper states that
the caches are held in bfloat16 (storage-overhead proof).

Pins (tests/test_oracle_*.py): uncached forward against a torch float64 model
built from library ops with a complex-multiplication RoPE; brute-force
attention on tiny inputs; cosine identities and torch's cosine_similarity;
selection against a full sort by (score, index) with engineered ties; rho=1 /
K_p=K_r=1 and refresh steps equal the uncached forward; a repeated input right
after a refresh reproduces the output with all scores 1; cache rows outside the
selected set stay bit-identical; MAC counts and cache bytes against the paper's
closed forms; update ratios per layer: equal ratios reproduce the global one,
each layer rewrites exactly its own share of rows, the linear allocation has
the appendix table's end values and average.  The absolute activation values of an adaptive step have no
printed worked example in the paper: beyond those invariants they are
"parity unpinned".
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence

import numpy as np


# ----------------------------------------------------------------------------
# model description
# ----------------------------------------------------------------------------
@dataclass
class Model:
    T: int          # layers
    d: int          # hidden width
    H_q: int        # query heads
    H_kv: int       # key/value heads (H_q for MHA)
    d_h: int        # head width
    m: int          # FFN width
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def d_q(self) -> int:
        return self.H_q * self.d_h

    @property
    def d_kv(self) -> int:
        return self.H_kv * self.d_h


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Nearest bf16 value, ties to even, via binary32; result in a's dtype."""
    a = np.asarray(a)
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = ((u + 0x7FFF + lsb) >> 16) << 16
    r = u.astype(np.uint32).view(np.float32).reshape(f.shape)
    r = np.where(np.isfinite(f), r, f)
    return r.astype(a.dtype if a.dtype.kind == "f" else np.float64)


# ----------------------------------------------------------------------------
# transformer primitives
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """Row-wise x / sqrt(mean(x^2) + eps) * g."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x: np.ndarray, pos: np.ndarray, d_h: int, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing (t, t + d_h/2) inside every head.

    x: [rows, H*d_h], pos: [rows] absolute positions.
    Pair t of a head is rotated by the angle pos * theta^(-2t/d_h).
    """
    rows, width = x.shape
    H = width // d_h
    half = d_h // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d_h)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    xh = x.reshape(rows, H, d_h)
    x1, x2 = xh[..., :half], xh[..., half:]
    out = np.empty_like(xh)
    out[..., :half] = x1 * c - x2 * s
    out[..., half:] = x2 * c + x1 * s
    return out.reshape(rows, width)


def attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, H_q: int, H_kv: int,
              d_h: int) -> np.ndarray:
    """Bidirectional softmax attention of query rows over ALL key rows, no mask.

    Q: [q, H_q*d_h], K, V: [n, H_kv*d_h].  Query head a reads KV head
    a // (H_q/H_kv).  Returns [q, H_q*d_h] (heads concatenated).
    """
    q = Q.shape[0]
    group = H_q // H_kv
    out = np.empty((q, H_q * d_h), dtype=Q.dtype)
    scale = 1.0 / math.sqrt(d_h)
    for a in range(H_q):
        kv = a // group
        Qa = Q[:, a * d_h:(a + 1) * d_h]
        Ka = K[:, kv * d_h:(kv + 1) * d_h]
        Va = V[:, kv * d_h:(kv + 1) * d_h]
        logits = (Qa @ Ka.T) * scale
        logits = logits - logits.max(axis=1, keepdims=True)
        p = np.exp(logits)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, a * d_h:(a + 1) * d_h] = p @ Va
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def cosine_scores(v_new: np.ndarray, v_old: np.ndarray) -> np.ndarray:
    """Eq. (cos_sim): per-row cosine over the whole d_kv-wide Value row.

    The denominator is clamped at 1e-8 so an all-zero row scores 0.
    """
    dot = np.sum(v_new * v_old, axis=1)
    den = np.sqrt(np.sum(v_new * v_new, axis=1)) * np.sqrt(np.sum(v_old * v_old, axis=1))
    return dot / np.maximum(den, 1e-8)


def l2_scores(v_new: np.ndarray, v_old: np.ndarray) -> np.ndarray:
    """Score of the L2-distance variant of V-verify (appendix "Impact of Similarity Metric"):
    minus the Euclidean distance between the current and the cached Value row, so that, as with
    the cosine, the lowest scores mark the rows that changed most."""
    diff = v_new - v_old
    return -np.sqrt(np.sum(diff * diff, axis=1))


def _fmix32(x: int) -> int:
    """Finalizer of MurmurHash3 (32-bit): a bijective avalanche mix."""
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x85EBCA6B) & 0xFFFFFFFF
    x ^= x >> 13
    x = (x * 0xC2B2AE35) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def random_scores(seed: int, step: int, layer: int, seq: int, L_r: int) -> np.ndarray:
    """Scores of the random-selection baseline (Sec. 4.3, selection strategies): a counter-based
    uniform in [0, 1) per (seed, step, layer, sequence, position), 24 bits, exactly representable
    in float32.  h = seed; for each of step, layer, sequence, position: h = fmix32(h xor value)."""
    out = np.empty(L_r, dtype=np.float64)
    h0 = seed & 0xFFFFFFFF
    for v in (step, layer, seq):
        h0 = _fmix32(h0 ^ (v & 0xFFFFFFFF))
    for j in range(L_r):
        out[j] = (_fmix32(h0 ^ j) >> 8) * 2.0 ** -24
    return out


def num_selected(rho: float, L_r: int) -> int:
    """floor(rho * |y|) with |y| the response length (Sec. 3.2.2)."""
    return int(math.floor(float(rho) * L_r + 1e-6))


def linear_rho_allocation(T: int, first: float, last: float) -> List[float]:
    """Update ratio per layer for the cross-layer allocation study (appendix table
    "Cross-layer update ratio allocation"): the table gives the two end values of a
    front-heavy and of a back-heavy allocation with a common average; read here as a straight
    line over the layer index, rho_l = first + (last - first) * l / (T - 1), whose average is
    (first + last) / 2."""
    if T < 1:
        raise ValueError("need at least one layer")
    if T == 1:
        return [0.5 * (first + last)]
    return [first + (last - first) * l / (T - 1) for l in range(T)]


def bottom_k(scores: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k lowest scores; equal scores go to the lower index.

    Returned ascending by index.
    """
    if k <= 0:
        return np.zeros(0, dtype=np.int64)
    order = np.lexsort((np.arange(scores.size), scores))  # primary: score, then index
    return np.sort(order[:k]).astype(np.int64)


def boundary_gap(scores: np.ndarray, k: int) -> float:
    """Delta of the cross-layer appendix: s_(k+1) - s_(k) in ascending order."""
    if k <= 0 or k >= scores.size:
        return float("inf")
    s = np.sort(scores)
    return float(s[k] - s[k - 1])


# ----------------------------------------------------------------------------
# the plain forward pass (no caching anywhere)
# ----------------------------------------------------------------------------
def uncached_forward(model: Model, weights: Sequence[Dict[str, np.ndarray]],
                     hidden_in: np.ndarray, storage: str = "f64",
                     dtype=np.float64) -> np.ndarray:
    """Textbook pre-norm bidirectional transformer over all n rows of each sequence.

    hidden_in: [B, n, d].  Returns the residual stream after the last block.
    """
    st, stc = _store_fn(storage), _cache_store_fn(storage)
    B, n, d = hidden_in.shape
    out = np.empty((B, n, d), dtype=dtype)
    pos = np.arange(n)
    for b in range(B):
        x = np.asarray(hidden_in[b], dtype=dtype)
        for l in range(model.T):
            W = _as(weights[l], dtype)
            h = st(rmsnorm(x, W["attn_norm_g"], model.rms_eps))
            q = st(rope(h @ W["wq"].T, pos, model.d_h, model.rope_theta))
            k = stc(rope(h @ W["wk"].T, pos, model.d_h, model.rope_theta))
            v = stc(h @ W["wv"].T)
            a = st(attention(q, k, v, model.H_q, model.H_kv, model.d_h))
            x = x + stc(a @ W["wo"].T)
            g = st(rmsnorm(x, W["ffn_norm_g"], model.rms_eps))
            u = st(silu(g @ W["w_gate"].T) * (g @ W["w_up"].T))
            x = x + stc(u @ W["w_down"].T)
        out[b] = stc(x)
    return out


def _store_fn(storage: str):
    """Rounding applied where a bf16 implementation materialises an intermediate tensor."""
    if storage in ("f64", "bf16_cache"):
        return lambda a: a
    if storage == "bf16":
        return round_bf16
    raise ValueError("storage must be 'f64', 'bf16' or 'bf16_cache'")


def _cache_store_fn(storage: str):
    """Rounding applied to what is written into a cache (K, V, AttnOut, FFNOut) and to the
    step's output.  'bf16_cache' is the narrowest reading of the paper's statement that the
    caches are held in bfloat16 (storage-overhead proof): only those tensors are rounded, every
    intermediate stays in the working precision."""
    if storage == "f64":
        return lambda a: a
    if storage in ("bf16", "bf16_cache"):
        return round_bf16
    raise ValueError("storage must be 'f64', 'bf16' or 'bf16_cache'")


def _as(W: Dict[str, np.ndarray], dtype) -> Dict[str, np.ndarray]:
    return {k: np.asarray(v, dtype=dtype) for k, v in W.items()}


# ----------------------------------------------------------------------------
# the cached denoiser
# ----------------------------------------------------------------------------
@dataclass
class StepReport:
    prompt_refresh: bool
    response_refresh: bool
    selected: List[List[np.ndarray]]      # [layer][sequence] -> ascending response indices
    scores: List[List[Optional[np.ndarray]]]  # [layer][sequence] -> s_j (None on refresh)
    gaps: List[List[float]]               # [layer][sequence] -> boundary margin Delta


class CachedDenoiser:
    """State and step rule of dLLM-Cache for a batch of independent sequences.

    Caches per layer l (Sec. 3.2): K (after RoPE), V, AttnOut (after the output
    projection, before the residual add) and FFNOut (after the down projection,
    before the residual add), each [B, n, width]; rows [0, L_p) form the prompt
    cache C_p, rows [L_p, n) the response cache C_r.
    """

    def __init__(self, model: Model, weights: Sequence[Dict[str, np.ndarray]], B: int,
                 L_p: int, L_r: int, rho: float, K_p: int, K_r: int,
                 storage: str = "f64", dtype=np.float64, metric: str = "cosine",
                 selection: str = "verify", v_update: str = "all", seed: int = 0,
                 source: str = "v", rho_layers: Optional[Sequence[float]] = None):
        """rho_layers, if given, replaces rho layer by layer (the paper's selection is local to a
        layer, appendix "Layer-wise token selection"; its cross-layer study gives layers
        different ratios): layer l recomputes floor(rho_layers[l] * L_r) response rows.
        metric / selection / v_update / source pick the variants the paper compares with its
        default (cosine V-verify, whole-V overwrite): metric "l2" (appendix "Impact of
        Similarity Metric"), selection "random" (Sec. 4.3), v_update "selected" (appendix
        "Design Choice Between Full V-Cache Overwrite and Selective Update": only the selected
        rows of the verified tensor are written back, the others keep the cached ones), source
        "k" (K-verify, Sec. 4.3: the roles of K and V are exchanged: the Key rows, after RoPE,
        of all response rows are computed, scored against the cached Keys and written back,
        and the Values are recomputed and scattered for the selected rows only; the paper names
        the strategy without spelling it out, this is the mirror image of its V-verify)."""
        if not (0.0 <= rho <= 1.0) or K_p < 1 or K_r < 1:
            raise ValueError("need 0 <= rho <= 1 and K_p, K_r >= 1")
        if metric not in ("cosine", "l2") or selection not in ("verify", "random") or \
                v_update not in ("all", "selected") or source not in ("v", "k"):
            raise ValueError("unknown policy")
        self.metric, self.selection, self.v_update, self.seed = metric, selection, v_update, seed
        self.source = source
        self.model, self.weights = model, weights
        self.B, self.L_p, self.L_r, self.n = B, L_p, L_r, L_p + L_r
        self.rho, self.K_p, self.K_r = rho, K_p, K_r
        self.k_sel = num_selected(rho, L_r)
        if rho_layers is None:
            self.k_layers = [self.k_sel] * model.T
        else:
            if len(rho_layers) != model.T or any(not (0.0 <= r <= 1.0) for r in rho_layers):
                raise ValueError("need one ratio in [0, 1] per layer")
            self.k_layers = [num_selected(r, L_r) for r in rho_layers]
        self.storage, self.dtype = storage, dtype
        self._st = _store_fn(storage)
        self._stc = _cache_store_fn(storage)
        T, n = model.T, self.n
        z = lambda w: [np.zeros((B, n, w), dtype=dtype) for _ in range(T)]
        self.K, self.V = z(model.d_kv), z(model.d_kv)
        self.AttnOut, self.FFNOut = z(model.d), z(model.d)
        self.prompt_hidden_out = np.zeros((B, L_p, model.d), dtype=dtype)
        self.initialised = False
        self.macs = 0  # multiply-accumulates actually performed, all steps so far

    # -- schedule (Sec. 3.2, "Iterative Steps"); step index i counts up from 0 --
    def step_kind(self, i: int):
        prompt_refresh = (i % self.K_p == 0)
        response_refresh = (i % self.K_r == 0)
        return prompt_refresh, response_refresh

    def step(self, hidden_in: np.ndarray, i: int,
             forced_sel: Optional[Sequence[Sequence[np.ndarray]]] = None,
             on_layer=None):
        """One denoising step.  hidden_in: [B, n, d] embedded tokens.

        forced_sel[l][b], if given, replaces the oracle's own selection at layer
        l (used to continue along another valid choice among near-ties).
        on_layer(l, b, scores, own_selection), if given, is called before the
        selection is applied and may return a replacement index array.
        Returns (hidden_out [B, n, d], StepReport).
        """
        mo, st, stc, dt = self.model, self._st, self._stc, self.dtype
        L_p, L_r, n = self.L_p, self.L_r, self.n
        P, Rf = self.step_kind(i)
        if i == 0:
            P = Rf = True
        if not self.initialised and not (P and Rf):
            raise RuntimeError("the first step must be step 0 (it fills both caches)")
        rep = StepReport(P, Rf, [[None] * self.B for _ in range(mo.T)],
                         [[None] * self.B for _ in range(mo.T)],
                         [[float("inf")] * self.B for _ in range(mo.T)])
        hidden_out = np.empty((self.B, n, mo.d), dtype=dt)
        for b in range(self.B):
            # rows carried through the layers: the response, plus the prompt on a prompt refresh
            C = np.arange(0 if P else L_p, n)
            off = C[0]                       # row r of the sequence sits at x[r - off]
            x = np.asarray(hidden_in[b, C], dtype=dt)
            resp_in_C = np.arange(L_p - off, n - off)
            for l in range(mo.T):
                W = _as(self.weights[l], dt)
                h = st(rmsnorm(x, W["attn_norm_g"], mo.rms_eps))
                # the verified tensor (V by default, K after RoPE for K-verify) of every carried row
                k_src = self.source == "k"
                if k_src:
                    T_new = stc(rope(h @ W["wk"].T, C, mo.d_h, mo.rope_theta))
                    cache = self.K[l]
                else:
                    T_new = stc(h @ W["wv"].T)
                    cache = self.V[l]
                self.macs += h.shape[0] * mo.d * mo.d_kv
                if Rf:
                    S = np.arange(L_r)
                else:
                    if self.selection == "random":
                        s = random_scores(self.seed, i, l, b, L_r)
                    elif self.metric == "l2":
                        s = l2_scores(T_new[resp_in_C], cache[b, L_p:])
                    else:
                        s = cosine_scores(T_new[resp_in_C], cache[b, L_p:])
                    S = bottom_k(s, self.k_layers[l])
                    rep.scores[l][b] = s
                    rep.gaps[l][b] = boundary_gap(s, self.k_layers[l])
                    if on_layer is not None:
                        alt = on_layer(l, b, s, S)
                        if alt is not None:
                            S = np.sort(np.asarray(alt, dtype=np.int64))
                    if forced_sel is not None:
                        S = np.sort(np.asarray(forced_sel[l][b], dtype=np.int64))
                rep.selected[l][b] = S
                # rows whose other projections, AttnOut and FFNOut are recomputed
                R = np.concatenate([np.arange(L_p) if P else np.zeros(0, dtype=np.int64),
                                    L_p + S]).astype(np.int64)
                if self.v_update == "all" or Rf:
                    # the whole verified tensor of the response (and of a refreshed prompt) is overwritten
                    cache[b, C] = T_new
                else:
                    # variant: only the selected rows (and a refreshed prompt) take their new rows
                    cache[b, R] = T_new[R - off]
                if R.size:
                    hR = h[R - off]
                    Q_R = st(rope(hR @ W["wq"].T, R, mo.d_h, mo.rope_theta))
                    if k_src:
                        self.V[l][b, R] = stc(hR @ W["wv"].T)
                    else:
                        self.K[l][b, R] = stc(rope(hR @ W["wk"].T, R, mo.d_h, mo.rope_theta))
                    self.macs += R.size * mo.d * (mo.d_q + mo.d_kv)
                    # queries in R attend to all n cached keys/values (updated above)
                    A_R = st(attention(Q_R, self.K[l][b], self.V[l][b], mo.H_q, mo.H_kv, mo.d_h))
                    self.macs += 2 * R.size * n * mo.d_q
                    self.AttnOut[l][b, R] = stc(A_R @ W["wo"].T)
                    self.macs += R.size * mo.d_q * mo.d
                # residual: fresh rows and cached rows alike come from the cache
                x = x + self.AttnOut[l][b, C]
                if R.size:
                    g = st(rmsnorm(x[R - off], W["ffn_norm_g"], mo.rms_eps))
                    u = st(silu(g @ W["w_gate"].T) * (g @ W["w_up"].T))
                    self.FFNOut[l][b, R] = stc(u @ W["w_down"].T)
                    self.macs += 3 * R.size * mo.d * mo.m
                x = x + self.FFNOut[l][b, C]
            x = stc(x)
            if P:
                self.prompt_hidden_out[b] = x[:L_p]
            hidden_out[b, :L_p] = self.prompt_hidden_out[b]
            hidden_out[b, L_p:] = x[resp_in_C]
        self.initialised = True
        return hidden_out, rep


def selection_is_admissible(scores: np.ndarray, k: int, candidate: np.ndarray,
                            tol: float = 1e-4) -> bool:
    """Is `candidate` a valid bottom-k set up to near-ties of width `tol`?

    With tau the k-th smallest score: every row scoring below tau - tol must be
    in the set, no row scoring above tau + tol may be, and the set has k
    distinct in-range members.
    """
    cand = np.asarray(candidate, dtype=np.int64)
    if cand.size != k or np.unique(cand).size != k:
        return False
    if k == 0:
        return True
    if cand.min() < 0 or cand.max() >= scores.size:
        return False
    tau = np.sort(scores)[k - 1]
    inside = np.zeros(scores.size, dtype=bool)
    inside[cand] = True
    must = scores < tau - tol
    never = scores > tau + tol
    return bool(np.all(inside[must]) and not np.any(inside[never]))


# ----------------------------------------------------------------------------
# closed forms of the paper's appendices
# ----------------------------------------------------------------------------
def flops_uncached_step(T: int, n: int, d: int, m: int) -> int:
    """Appendix "Complexity of the Original dLLM Model": T(8nd^2 + 4n^2 d + 6ndm)."""
    return T * (8 * n * d * d + 4 * n * n * d + 6 * n * d * m)


def flops_response_refresh_step(T: int, n: int, r: int, d: int, m: int) -> int:
    """Second term's bracket: T(8rd^2 + 4rnd + 6rdm)."""
    return T * (8 * r * d * d + 4 * r * n * d + 6 * r * d * m)


def flops_adaptive_step(T: int, n: int, r: int, r_hat: int, d: int, m: int) -> int:
    """Third term's bracket as printed: T(2rd^2 + 8 r^ d^2 + 4 r^ n d + 6 r^ d m)."""
    return T * (2 * r * d * d + 8 * r_hat * d * d + 4 * r_hat * n * d + 6 * r_hat * d * m)


def flops_dllm_cache(K: int, K_p: int, K_r: int, T: int, n: int, r: int, r_hat: int,
                     d: int, m: int) -> float:
    """The three-term total of the complexity appendix (K_r | K_p | K assumed there)."""
    return (K / K_p * flops_uncached_step(T, n, d, m)
            + (K / K_r - K / K_p) * flops_response_refresh_step(T, n, r, d, m)
            + K * (1 - 1 / K_r) * flops_adaptive_step(T, n, r, r_hat, d, m))


def cache_elements(layers: int, tokens: int, d: int) -> int:
    """Storage-overhead proof: four tensors of tokens x d per layer."""
    return layers * 4 * tokens * d
