"""Oracle-only measurement of the numerical noise floor of a model: how far apart two valid
evaluations are that round the same tensors to the storage type but accumulate in different
precision.  A float32-accumulating copy of the oracle (the shadow) follows the float64 oracle
step by step on the same inputs and the same selected sets; what is recorded per layer:

  * score_dev    max |s_f32 - s_f64| over the verify scores of the layer (adaptive steps);
  * K, V, AttnOut, FFNOut, and hidden_out of the step: the three distances of tests/metrics.py.

Every figure is the maximum over the steps taken.  No implementation that sums in float32 can
be expected to sit closer to the float64 oracle than this, and a margin at the selection
boundary (appendix on cross-layer behaviour) below twice the score noise cannot decide a set.
Nothing here touches the HIP library: the parity tests take their tolerances from these
figures, either measured on the fly (small models) or stored by
tests/golden/make_bf16_noise_floor.py (full-size models).
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

from oracle import dllm_cache_oracle as O
from tests import metrics as MT

TENSORS = ("K", "V", "AttnOut", "FFNOut")


def _merge_max(acc: Dict[str, float], new: Dict[str, float]) -> None:
    for k, v in new.items():
        acc[k] = max(acc.get(k, 0.0), float(v))


class Shadow:
    """Float32-accumulating twin of a float64 CachedDenoiser; follow() is called after every
    step of the twin's original with that step's input and report."""

    def __init__(self, ora: O.CachedDenoiser, seqs: Optional[List[int]] = None):
        self.ora = ora
        self.sh = O.CachedDenoiser(ora.model, ora.weights, ora.B, ora.L_p, ora.L_r, ora.rho, ora.K_p,
                                   ora.K_r, storage=ora.storage, dtype=np.float32, metric=ora.metric,
                                   selection=ora.selection, v_update=ora.v_update, seed=ora.seed,
                                   source=ora.source)
        self.sh.k_layers = list(ora.k_layers)
        T = ora.model.T
        self.layers: List[Dict] = [dict({t: {} for t in TENSORS}, score_dev=0.0) for _ in range(T)]
        self.hidden_out: Dict[str, float] = {}

    def follow(self, hidden_in: np.ndarray, i: int, rep: O.StepReport, out: np.ndarray) -> None:
        out_s, rep_s = self.sh.step(np.asarray(hidden_in, dtype=np.float32), i, forced_sel=rep.selected)
        _merge_max(self.hidden_out, MT.all_three(out_s, out))
        for l in range(self.ora.model.T):
            for b in range(self.ora.B):
                if rep.scores[l][b] is not None:
                    dev = float(np.max(np.abs(rep.scores[l][b] - rep_s.scores[l][b].astype(np.float64))))
                    self.layers[l]["score_dev"] = max(self.layers[l]["score_dev"], dev)
            for t in TENSORS:
                _merge_max(self.layers[l][t], MT.all_three(getattr(self.sh, t)[l], getattr(self.ora, t)[l]))

    def floor(self) -> Dict:
        return {"hidden_out": dict(self.hidden_out), "layers": [
            dict({t: dict(L[t]) for t in TENSORS}, score_dev=L["score_dev"]) for L in self.layers]}


# ---- tolerances derived from a floor -----------------------------------------------------
FROB_FACTOR, ROW_FACTOR, MAXABS_FACTOR = 1.5, 2.0, 2.0
# Added to a bar so that floors made of a handful of last-bit differences stay usable.  bf16: a
# float32 sum taken in another order (matrix-core tiles, split contraction) than the shadow's
# moves up to ~1e-3 of the elements of a tensor across a bf16 rounding boundary, each by one ulp
# (2^-8 relative): a Frobenius ratio of 2^-8 sqrt(1e-3).  float32: summation-order noise itself.
EPS = {"bf16": 2.0 ** -8 * 1e-3 ** 0.5, "f32": 2e-6}


def bars(entry: Dict[str, float], dtype: str = "bf16") -> Dict[str, float]:
    """Largest admissible distances of an implementation from the float64 oracle for a tensor
    whose oracle-only floor is `entry`."""
    eps = EPS[dtype]
    return {"frob": FROB_FACTOR * entry["frob"] + eps,
            "row": ROW_FACTOR * entry["row"] + 2 * eps,
            "maxabs": MAXABS_FACTOR * entry["maxabs"] + 8 * eps}


def band(score_dev: float, base: float = 1e-4) -> float:
    """Width below which a boundary margin does not decide the selected set."""
    return max(base, 2.0 * score_dev)


def score_tol(score_dev: float, base: float) -> float:
    """Largest admissible |s_impl - s_oracle| in a layer whose oracle-only score noise is score_dev."""
    return max(base, 4.0 * score_dev)
