"""Writes tests/golden/bf16_noise_floor.json.  Calls only the oracle (and the input generators).

How far apart are two valid bf16 evaluations of the LLaDA-8B-shaped random-weight model?  The
oracle's uncached step (step 0 of the cached denoiser, a full refresh) is run twice with bf16
storage rounding, once accumulating in float64 and once in float32: same rounding points,
different summation error, hence a few tensor elements that land on the neighbouring bf16
value, amplified through the 32 layers.  The relative Frobenius distance of the step output and
of the last layer's cache tensors is the floor below which no bf16 implementation can be
expected to match another.  Takes several minutes and ~45 GB of host memory.

    python tests/golden/make_bf16_noise_floor.py [config-name]
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import dllm_cache_oracle as O          # noqa: E402
from paper_2506_06295_amd import inputs as I       # noqa: E402


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "llada8b"
    cfg = I.CONFIGS[name]
    t0 = time.time()
    ws = I.all_weights(cfg)
    print(f"weights {time.time() - t0:.0f}s", flush=True)
    h = I.TokenSchedule(cfg, stress=True).hidden_in(0)
    model = O.Model(cfg.T, cfg.d, cfg.H_q, cfg.H_kv, cfg.d_h, cfg.m, cfg.rms_eps, cfg.rope_theta)
    dens = {}
    for tag, dt in (("f32", np.float32), ("f64", np.float64)):
        den = O.CachedDenoiser(model, ws, cfg.B, cfg.L_p, cfg.L_r, cfg.rho, cfg.K_p, cfg.K_r,
                               storage="bf16", dtype=dt)
        out, _ = den.step(h.astype(dt), 0)
        dens[tag] = (out.astype(np.float64), den)
        print(f"{tag} done {time.time() - t0:.0f}s", flush=True)

    def rel(a, b):
        return float(np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b))

    res = {"_about": "relative Frobenius distance between the oracle with float32 and with float64 "
                     "accumulation, bf16 storage rounding in both; written by "
                     "tests/golden/make_bf16_noise_floor.py (oracle only)",
           "config": name, "hidden_out": rel(dens["f32"][0], dens["f64"][0])}
    for l in (0, cfg.T // 2, cfg.T - 1):
        res[f"layer{l}"] = {nm: rel(getattr(dens["f32"][1], nm)[l], getattr(dens["f64"][1], nm)[l].astype(np.float64))
                            for nm in ("K", "V", "AttnOut", "FFNOut")}
    path = os.path.join(ROOT, "tests", "golden", f"bf16_noise_floor_{name}.json")
    json.dump(res, open(path, "w"), indent=1)
    print(json.dumps(res, indent=1))


if __name__ == "__main__":
    main()
