"""Shared machinery of the GPU parity tests: run the HIP library and the CPU oracle on the same
seeded inputs and compare them step by step.

Every tolerance comes from an oracle-only quantity, never from the device under test: the
noise floor of the model (tests/noise_floor.py), i.e. how far a float32-accumulating copy of
the oracle lands from the float64 oracle on the same inputs and selected sets, per layer.  It
is measured on the fly for the small models and read from tests/golden/noise_floor_*.json
(written by tests/golden/make_bf16_noise_floor.py) for the full-size ones.

Selection rule (per layer and sequence):
  * always, bit-exact: the GPU's index set is the bottom-k (ties to the lower index) of the
    GPU's own scores -- the integer part of the decision;
  * the GPU's scores agree with the oracle's to max(base, 4 x the layer's score noise);
  * the GPU's set equals the oracle's whenever the oracle's margin at the selection boundary
    (s_(k+1) - s_(k), the Delta of the cross-layer appendix) exceeds the band max(base, 2 x the
    layer's score noise); otherwise any set that is a valid bottom-k up to near-ties of that
    width is accepted.  The oracle always continues with the GPU's set, so that later layers
    are compared on equal terms; a set that breaks the rule fails the step afterwards.
base is 1e-4 for float32 models.  For bf16 models one last-bit difference of a V element moves
a cosine by up to 2^-8 |v_i| / |v| ~ 2^-8 / sqrt(d_kv); base allows two of them:
max(1e-4, 2 * 2^-8 / sqrt(d_kv)), i.e. 1.2e-4 at d_kv = 4096.

Activations (step output, cache tensors), each against bars derived from its own floor
(noise_floor.bars): whole-tensor Frobenius ratio <= 1.5 x floor, worst row <= 2 x floor, worst
element (relative to the tensor's rms) <= 2 x floor, each plus a small epsilon for floors made
of a handful of last-bit differences (noise_floor.EPS); the step output must also meet the workloads' stated tolerance (1e-4 float32, 2e-2
bf16).
"""
from __future__ import annotations

import json
import os
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from oracle import dllm_cache_oracle as O
from paper_2506_06295_amd import binding, inputs as I
from tests import metrics as MT
from tests import noise_floor as NF

GAP_TOL = 1e-4
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def gap_tol(cfg: I.Config) -> float:
    if cfg.dtype == "f32":
        return GAP_TOL
    return max(GAP_TOL, 2.0 * 2.0 ** -8 / np.sqrt(cfg.d_kv))


def stated_tol(cfg: I.Config) -> float:
    """The tolerance the workloads state for the step output."""
    return 1e-4 if cfg.dtype == "f32" else 2e-2


def score_base(cfg: I.Config) -> float:
    return 1e-5 if cfg.dtype == "f32" else gap_tol(cfg)


def load_floor(name: str) -> Dict:
    return json.load(open(os.path.join(GOLDEN, f"noise_floor_{name}.json")))


def oracle_model(cfg: I.Config) -> O.Model:
    return O.Model(cfg.T, cfg.d, cfg.H_q, cfg.H_kv, cfg.d_h, cfg.m, cfg.rms_eps, cfg.rope_theta)


def torch_dtype(cfg: I.Config):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def to_device(cfg: I.Config, a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(torch_dtype(cfg)).contiguous()


def make_pair(cfg: I.Config, weights: List[Dict[str, np.ndarray]], **over):
    """(GPU denoiser, oracle denoiser) on the same weights."""
    rho, K_p, K_r = over.get("rho", cfg.rho), over.get("K_p", cfg.K_p), over.get("K_r", cfg.K_r)
    dev_ws = [{k: to_device(cfg, v) for k, v in w.items()} for w in weights]
    gpu = binding.CachedDenoiser(n_layers=cfg.T, d_model=cfg.d, n_q_heads=cfg.H_q,
                                 n_kv_heads=cfg.H_kv, head_dim=cfg.d_h, d_ffn=cfg.m, batch=cfg.B,
                                 dtype=cfg.dtype, weights=dev_ws, L_p=cfg.L_p, L_r=cfg.L_r, rho=rho,
                                 K_p=K_p, K_r=K_r, rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta,
                                 paging=over.get("paging"))
    policy = {k: over[k] for k in ("metric", "selection", "v_update", "seed", "source") if k in over}
    if policy:
        gpu.set_policy(**policy)
    if over.get("rho_layers") is not None:
        gpu.set_layer_rho(over["rho_layers"])
        policy = dict(policy, rho_layers=over["rho_layers"])
    ora = O.CachedDenoiser(oracle_model(cfg),
                           [{k: np.asarray(v, dtype=np.float64) for k, v in w.items()} for w in weights],
                           cfg.B, cfg.L_p, cfg.L_r, rho, K_p, K_r,
                           storage="bf16" if cfg.dtype == "bf16" else "f64", **policy)
    return gpu, ora


@dataclass
class ParityStats:
    exact: int = 0          # (layer, sequence) pairs with a decisive margin and an identical set
    tied_same: int = 0      # margin inside the band, sets identical anyway
    followed: int = 0       # margin inside the band, GPU chose another admissible set
    failed: int = 0         # decisive margin but different set, inadmissible set, or scores apart
    worst_rel: float = 0.0
    worst_row: float = 0.0
    worst_maxabs: float = 0.0
    worst_score_dev: float = 0.0
    worst_score_dev_over_tol: float = 0.0
    worst_over_bar: float = 0.0     # largest (distance / its bar) seen for any activation tensor
    rel_per_step: List[float] = field(default_factory=list)
    gaps: List[float] = field(default_factory=list)
    failures: List[str] = field(default_factory=list)
    floor: Optional[Dict] = None    # fixture; None: measured on the fly by `shadow`
    shadow: Optional[NF.Shadow] = None

    def current_floor(self) -> Dict:
        return self.floor if self.floor is not None else self.shadow.floor()


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    return MT.frob(got, want)


def check_tensor(stats: ParityStats, cfg, what: str, got: np.ndarray, want: np.ndarray,
                 entry: Dict[str, float], ceiling: Optional[float] = None) -> Dict[str, float]:
    """Three distances of one tensor against the bars of its floor entry; returns the distances."""
    d = MT.all_three(got, want)
    bar = NF.bars(entry, cfg.dtype)
    if ceiling is not None:
        bar["frob"] = min(bar["frob"], ceiling) if entry["frob"] <= ceiling else bar["frob"]
    for k in ("frob", "row", "maxabs"):
        stats.worst_over_bar = max(stats.worst_over_bar, d[k] / bar[k])
        assert d[k] <= bar[k], (f"{what}: {k} distance {d[k]:.3e} above its bar {bar[k]:.3e} "
                                f"(oracle-only floor {entry[k]:.3e}); largest difference at "
                                f"(index, got, want) = {MT.worst_element(got, want)}")
    stats.worst_row = max(stats.worst_row, d["row"])
    stats.worst_maxabs = max(stats.worst_maxabs, d["maxabs"])
    return d


class SelectionCheck:
    """After the GPU ran step i: checks the integer part of its selections at once; `on_layer`
    is the callback for the oracle's step (the oracle follows the GPU's sets); finish() then
    classifies every (layer, sequence) with the layer's oracle-only score noise."""

    def __init__(self, cfg, gpu, ora, i: int, n_sel: int, stats: ParityStats,
                 seqs: Optional[Sequence[int]] = None):
        if stats.floor is None and stats.shadow is None:
            stats.shadow = NF.Shadow(ora)
        self.cfg, self.ora, self.i, self.stats = cfg, ora, i, stats
        self.seqs = seqs = list(range(cfg.B)) if seqs is None else list(seqs)
        T = cfg.T
        self.sel = sel = gpu.sel_idx[:, :, :n_sel].cpu().numpy().astype(np.int64)[:, seqs]
        refresh = i % ora.K_r == 0
        self.ks = ks = [cfg.L_r if refresh else ora.k_layers[l] for l in range(T)]   # valid entries per layer
        self.gpu_scores = None
        if not refresh:
            sc = gpu.read_scores()
            torch.cuda.synchronize()
            self.gpu_scores = sc.cpu().numpy()[:, seqs]
            # integer part of the decision: exact bottom-k of the GPU's own scores
            for l in range(T):
                for b in range(len(seqs)):
                    want = O.bottom_k(self.gpu_scores[l, b].astype(np.float64), ks[l])
                    assert sel[l, b, :ks[l]].tolist() == want.tolist(), \
                        f"step {i} layer {l} seq {seqs[b]}: select kernel"
        self.records = []

    def on_layer(self, l, b, s, own):
        k = self.ks[l]
        got = self.sel[l, b, :k]
        self.records.append((l, b, np.array(s, dtype=np.float64), own.copy(), got))
        # the oracle follows the GPU's set whenever that is a set at all; whether it was an
        # admissible one is decided in finish(), once the layer's score noise is known
        ok = got.size == k and np.unique(got).size == k and (k == 0 or (got.min() >= 0 and got.max() < self.cfg.L_r))
        return got if ok else None

    def finish(self, hidden_in_oracle: np.ndarray, rep: O.StepReport, want: np.ndarray) -> None:
        cfg, stats, i, seqs = self.cfg, self.stats, self.i, self.seqs
        if stats.shadow is not None:
            stats.shadow.follow(hidden_in_oracle, i, rep, want)
        floor = stats.current_floor()
        base, sbase = gap_tol(cfg), score_base(cfg)
        for l, b, s, own, got in self.records:
            k = self.ks[l]
            sd = floor["layers"][l]["score_dev"]
            lbase, lsbase = base, sbase
            if self.ora.metric == "l2" and cfg.dtype == "bf16":
                # the distance score is not normalised: one last-bit difference of an element of
                # the verified row moves it by up to one bf16 ulp of that element; allow two at
                # the largest magnitude the oracle's own tensor holds
                src = self.ora.K[l] if self.ora.source == "k" else self.ora.V[l]
                ulp2 = 2.0 * 2.0 ** -8 * float(np.max(np.abs(src[b])))
                lbase, lsbase = max(base, ulp2), max(sbase, ulp2)
            band = NF.band(sd, lbase)
            gap = O.boundary_gap(s, k)
            stats.gaps.append(gap)
            if self.gpu_scores is not None:
                dev = float(np.max(np.abs(self.gpu_scores[l, b] - s)))
                tol = NF.score_tol(sd, lsbase)
                stats.worst_score_dev = max(stats.worst_score_dev, dev)
                stats.worst_score_dev_over_tol = max(stats.worst_score_dev_over_tol, dev / tol)
                if dev > tol:
                    stats.failed += 1
                    stats.failures.append(f"step {i} layer {l} seq {seqs[b]}: scores {dev:.3e} apart, "
                                          f"tolerance {tol:.3e} (oracle-only score noise {sd:.3e})")
                    continue
            same = got.tolist() == own.tolist()
            if gap > band:
                if same:
                    stats.exact += 1
                else:
                    stats.failed += 1
                    stats.failures.append(f"step {i} layer {l} seq {seqs[b]}: margin {gap:.3e} above the "
                                          f"band {band:.3e} but sets differ")
            elif same:
                stats.tied_same += 1
            elif O.selection_is_admissible(s, k, got, band):
                stats.followed += 1
            else:
                stats.failed += 1
                stats.failures.append(f"step {i} layer {l} seq {seqs[b]}: inadmissible set (margin "
                                      f"{gap:.3e}, band {band:.3e})")
        assert not stats.failed, stats.failures


def run_step_pair(cfg, gpu, ora, hidden_in: np.ndarray, i: int, stats: ParityStats,
                  seqs: Optional[Sequence[int]] = None):
    """One step on both sides; returns (gpu_out float64 ndarray, oracle_out).  `seqs`: the
    sequences of the GPU's batch the oracle runs (default: all); hidden_in is the GPU's input."""
    out_t, n_sel = gpu.step(to_device(cfg, hidden_in), i)
    torch.cuda.synchronize()
    chk = SelectionCheck(cfg, gpu, ora, i, n_sel, stats, seqs)
    h_or = np.asarray(hidden_in, dtype=np.float64)[chk.seqs]
    want, rep = ora.step(h_or, i, on_layer=chk.on_layer)
    chk.finish(h_or, rep, want)
    check_selection_shape(cfg, ora, rep, chk.sel, n_sel)
    got = out_t.float().cpu().numpy().astype(np.float64)[chk.seqs]
    d = check_tensor(stats, cfg, f"step {i} hidden_out", got, want, stats.current_floor()["hidden_out"],
                     ceiling=stated_tol(cfg))
    stats.rel_per_step.append(d["frob"])
    stats.worst_rel = max(stats.worst_rel, d["frob"])
    return got, want


def check_selection_shape(cfg, ora, rep, sel, n_sel: int):
    if rep.response_refresh:
        assert n_sel == cfg.L_r
        assert np.array_equal(sel, np.broadcast_to(np.arange(cfg.L_r), sel.shape))
    else:
        assert n_sel == max(ora.k_layers)
        for l, k in enumerate(ora.k_layers):
            if k:
                assert np.all(np.diff(sel[l, :, :k], axis=-1) > 0), "indices must be ascending"
                assert sel[l, :, :k].min() >= 0 and sel[l, :, :k].max() < cfg.L_r


def compare_caches(cfg, gpu, ora, stats: ParityStats, seqs: Optional[Sequence[int]] = None,
                   verbose: bool = False) -> float:
    """Every layer's four cache tensors against the oracle's, each held to the bars of its own
    floor; returns the worst Frobenius ratio."""
    seqs = list(range(cfg.B)) if seqs is None else list(seqs)
    floor = stats.current_floor()
    worst = 0.0
    for l in range(cfg.T):
        for which, name in enumerate(NF.TENSORS):
            got = gpu.read_cache(l, which)
            torch.cuda.synchronize()
            got = got.float().cpu().numpy()[seqs]
            d = check_tensor(stats, cfg, f"layer {l} cache {name}", got, getattr(ora, name)[l], floor["layers"][l][name])
            worst = max(worst, d["frob"])
            if verbose:
                f = floor["layers"][l][name]
                print(f"[caches] layer {l} {name}: frob {d['frob']:.3e} (floor {f['frob']:.3e})  "
                      f"row {d['row']:.3e} ({f['row']:.3e})  maxabs {d['maxabs']:.3e} ({f['maxabs']:.3e})",
                      flush=True)
    return worst
