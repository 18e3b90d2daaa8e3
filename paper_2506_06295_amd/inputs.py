"""Seeded synthetic inputs for the cached denoising step.

This module only draws numbers and describes shapes.  It holds none of the
method's arithmetic (no norms, projections, similarity, selection or cache
rules) and imports neither the CPU oracle nor the HIP library, so both can be
fed the very same arrays.

Workload recipe (stands in for the paper's benchmark runs, Sec. 4.1 and the
per-task settings of its appendix "Experimental Details"; none of those
datasets or trained weights are used):

* weights      N(0, 0.02), norm gains 1.0, one seed per (config, layer, tensor);
* embeddings   N(0, 1) rows of a token table plus one fixed [MASK] row;
* prompt       L_p seeded-uniform token ids, constant over the schedule;
* response     starts all-[MASK]; after every step `unmask_per_step`
               seeded-random still-masked positions receive seeded-random ids,
               so the response is fully unmasked when the schedule ends;
* stress mode  additionally perturbs a seeded 30 % of response rows per step
               with N(0, 0.5) noise so the selection boundary is decisive;
* closed loop  (the model's own predictions drive the unmasking): a token table of
               vocab + 1 rows N(0, 1), the last row being [MASK], a final norm gain of 1 and
               a vocabulary projection N(0, 0.02); the prompt ids are the schedule's.

For bf16 configurations all values are rounded to the bf16 grid here (round to
nearest even through torch's conversion) and handed out as float32 arrays.
"""
from __future__ import annotations

import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Optional

import numpy as np
import torch

WEIGHT_NAMES = ("attn_norm_g", "wq", "wk", "wv", "wo", "ffn_norm_g", "w_gate", "w_up", "w_down")


@dataclass(frozen=True)
class Config:
    """Shapes and cache hyper-parameters of one workload.

    Symbols follow the paper: T layers, d width, m FFN width, L_p / L_r prompt
    and response length, rho update ratio, K_p / K_r refresh intervals.
    """

    name: str
    T: int
    d: int
    H_q: int
    H_kv: int
    d_h: int
    m: int
    B: int
    L_p: int
    L_r: int
    steps: int
    rho: float
    K_p: int
    K_r: int
    dtype: str  # "f32" or "bf16": storage type of weights, activations and caches
    vocab: int
    unmask_per_step: int = 4
    block_len: int = 0  # closed loop: positions per semi-autoregressive block (0 = L_r)
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    seed: int = 20250606

    @property
    def n(self) -> int:
        return self.L_p + self.L_r

    @property
    def d_q(self) -> int:
        return self.H_q * self.d_h

    @property
    def d_kv(self) -> int:
        return self.H_kv * self.d_h

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)

    def weight_shapes(self) -> Dict[str, tuple]:
        return {
            "attn_norm_g": (self.d,),
            "wq": (self.d_q, self.d),
            "wk": (self.d_kv, self.d),
            "wv": (self.d_kv, self.d),
            "wo": (self.d, self.d_q),
            "ffn_norm_g": (self.d,),
            "w_gate": (self.m, self.d),
            "w_up": (self.m, self.d),
            "w_down": (self.d, self.m),
        }

    def weight_elements_per_layer(self) -> int:
        return sum(int(np.prod(s)) for s in self.weight_shapes().values())


CONFIGS: Dict[str, Config] = {
    # small fp32 case the oracle finishes in well under a second
    "toy": Config("toy", T=2, d=256, H_q=4, H_kv=4, d_h=64, m=704, B=1, L_p=64, L_r=32,
                  steps=8, rho=0.25, K_p=4, K_r=2, dtype="f32", vocab=1024),
    # the configuration the headline metric is quoted on
    "llada8b": Config("llada8b", T=32, d=4096, H_q=32, H_kv=32, d_h=128, m=12288, B=1,
                      L_p=512, L_r=256, steps=64, rho=0.25, K_p=50, K_r=7, dtype="bf16",
                      vocab=126464),
    "dream7b": Config("dream7b", T=28, d=3584, H_q=28, H_kv=4, d_h=128, m=18944, B=1,
                      L_p=1024, L_r=256, steps=64, rho=0.25, K_p=50, K_r=5, dtype="bf16",
                      vocab=152064),
    "llada8b_long": Config("llada8b_long", T=32, d=4096, H_q=32, H_kv=32, d_h=128, m=12288,
                           B=1, L_p=4096, L_r=512, steps=128, rho=0.1, K_p=100, K_r=8,
                           dtype="bf16", vocab=126464),
    "llada8b_b16": Config("llada8b_b16", T=32, d=4096, H_q=32, H_kv=32, d_h=128, m=12288,
                          B=16, L_p=512, L_r=256, steps=64, rho=0.25, K_p=50, K_r=7,
                          dtype="bf16", vocab=126464),
}


def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """Round a float array to the nearest bf16 value (ties to even); float32 out."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def _rng(cfg: Config, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([cfg.seed, *[int(k) for k in key]]))


def layer_weights(cfg: Config, layer: int) -> Dict[str, np.ndarray]:
    """One layer's weights as float32 arrays, row-major [out, in]."""
    out = {}
    for t, (name, shape) in enumerate(cfg.weight_shapes().items()):
        if name.endswith("_g"):
            w = np.ones(shape, dtype=np.float32)
        else:
            w = (0.02 * _rng(cfg, 1, layer, t).standard_normal(shape, dtype=np.float32))
            if cfg.dtype == "bf16":
                w = to_bf16_grid(w)
        out[name] = w
    return out


def all_weights(cfg: Config) -> List[Dict[str, np.ndarray]]:
    return [layer_weights(cfg, l) for l in range(cfg.T)]


class TokenSchedule:
    """Token ids per step and their embeddings ([B, n, d] float32 arrays)."""

    def __init__(self, cfg: Config, stress: bool = False):
        self.cfg = cfg
        self.stress = stress
        r = _rng(cfg, 2)
        self.mask_id = cfg.vocab  # one extra row beyond the table
        self.prompt_ids = r.integers(0, cfg.vocab, size=(cfg.B, cfg.L_p))
        self._emb_cache: Dict[int, np.ndarray] = {}
        # unmasking order and the ids that appear, fixed up front
        self.order = np.stack([r.permutation(cfg.L_r) for _ in range(cfg.B)])
        self.new_ids = r.integers(0, cfg.vocab, size=(cfg.B, cfg.L_r))

    def _emb(self, tok: int) -> np.ndarray:
        e = self._emb_cache.get(tok)
        if e is None:
            e = _rng(self.cfg, 3, tok).standard_normal(self.cfg.d, dtype=np.float32)
            if self.cfg.dtype == "bf16":
                e = to_bf16_grid(e)
            self._emb_cache[tok] = e
        return e

    def response_ids(self, step: int) -> np.ndarray:
        """Response token ids fed to denoising step `step` (0 = all [MASK])."""
        cfg = self.cfg
        ids = np.full((cfg.B, cfg.L_r), self.mask_id, dtype=np.int64)
        done = min(cfg.L_r, step * cfg.unmask_per_step)
        for b in range(cfg.B):
            pos = self.order[b, :done]
            ids[b, pos] = self.new_ids[b, pos]
        return ids

    def hidden_in(self, step: int) -> np.ndarray:
        cfg = self.cfg
        resp = self.response_ids(step)
        out = np.empty((cfg.B, cfg.n, cfg.d), dtype=np.float32)
        for b in range(cfg.B):
            for t in range(cfg.L_p):
                out[b, t] = self._emb(int(self.prompt_ids[b, t]))
            for j in range(cfg.L_r):
                out[b, cfg.L_p + j] = self._emb(int(resp[b, j]))
        if self.stress:
            r = _rng(cfg, 4, step)
            for b in range(cfg.B):
                rows = r.permutation(cfg.L_r)[: max(1, (3 * cfg.L_r) // 10)]
                noise = 0.5 * r.standard_normal((rows.size, cfg.d), dtype=np.float32)
                out[b, cfg.L_p + rows] += noise
            if cfg.dtype == "bf16":
                out = to_bf16_grid(out)
        return out


def head_weights(cfg: Config) -> Dict[str, np.ndarray]:
    """Token table [vocab + 1, d] (last row: [MASK]), final norm gain [d], vocabulary
    projection [vocab, d]; float32 arrays on the storage type's grid."""
    e = _rng(cfg, 5).standard_normal((cfg.vocab + 1, cfg.d), dtype=np.float32)
    w = 0.02 * _rng(cfg, 6).standard_normal((cfg.vocab, cfg.d), dtype=np.float32)
    if cfg.dtype == "bf16":
        e, w = to_bf16_grid(e), to_bf16_grid(w)
    return {"embed": e, "final_norm_g": np.ones(cfg.d, dtype=np.float32), "lm_head": w}


def initial_tokens(cfg: Config) -> np.ndarray:
    """[B, n] token ids: the schedule's prompt, then an all-[MASK] response (id = vocab)."""
    t = np.full((cfg.B, cfg.n), cfg.vocab, dtype=np.int64)
    t[:, :cfg.L_p] = TokenSchedule(cfg).prompt_ids
    return t


def device_head_weights(cfg: Config, device: str = "cuda") -> Dict[str, torch.Tensor]:
    """Same tensors as head_weights, drawn on `device` (full-size vocabularies)."""
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed + 77)
    e = torch.randn((cfg.vocab + 1, cfg.d), dtype=torch.float32, device=device, generator=gen).to(dt)
    w = (0.02 * torch.randn((cfg.vocab, cfg.d), dtype=torch.float32, device=device,
                            generator=gen)).to(dt)
    return {"embed": e, "final_norm_g": torch.ones(cfg.d, dtype=dt, device=device), "lm_head": w}


def device_weights(cfg: Config, device: str = "cuda", n_layers: Optional[int] = None,
                   seed_offset: int = 0) -> List[Dict[str, torch.Tensor]]:
    """Full-size random-init weights drawn directly on `device` (no host copy).

    Used where 14 GB of host-side draws would dominate the run; values depend on
    the device's generator, so whoever needs them on the host copies them back.
    """
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    gen = torch.Generator(device=device)
    layers = []
    for l in range(cfg.T if n_layers is None else n_layers):
        gen.manual_seed(cfg.seed + 1000 * (l + seed_offset))
        w = {}
        for name, shape in cfg.weight_shapes().items():
            if name.endswith("_g"):
                w[name] = torch.ones(shape, dtype=dt, device=device)
            else:
                w[name] = (0.02 * torch.randn(shape, dtype=torch.float32, device=device,
                                              generator=gen)).to(dt)
        layers.append(w)
    return layers
