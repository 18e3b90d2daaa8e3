"""Writes tests/golden/noise_floor_<name>.json.  Calls only the oracle, the input generators
and the oracle-only helpers tests/noise_floor.py / tests/metrics.py.

How far apart are two valid bf16 evaluations of a random-weight model of a workload's shape?
The oracle's cached denoiser is run with bf16 storage rounding, accumulating in float64, and a
float32-accumulating twin follows it (same rounding points, different summation error, hence a
few tensor elements that land on the neighbouring bf16 value, amplified from layer to layer).
Per layer the script stores the distances of the four cache tensors (whole-tensor Frobenius
ratio, worst row, worst element), of the step output, and the largest difference of the verify
scores: the parity tests take their per-layer bars and their selection band from these.

    python tests/golden/make_bf16_noise_floor.py llada8b            # full depth, steps 0 and 1
    python tests/golden/make_bf16_noise_floor.py dream7b --layers 2 --kinds
    python tests/golden/make_bf16_noise_floor.py llada8b_b16 --layers 2 --kinds --batch 2

--kinds visits the four step kinds (K_p = 4, K_r = 3: full, adaptive, adaptive, response
refresh, prompt refresh + adaptive).  The full-depth run takes ~15 minutes and ~45 GB of host
memory on 8 cores.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import dllm_cache_oracle as O          # noqa: E402
from paper_2506_06295_amd import inputs as I       # noqa: E402
from tests import noise_floor as NF                # noqa: E402


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("config")
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--kinds", action="store_true")
    ap.add_argument("--steps", type=int, default=2)
    args = ap.parse_args()
    cfg = I.CONFIGS[args.config]
    if args.layers:
        cfg = cfg.replace(T=args.layers)
    if args.batch:
        cfg = cfg.replace(B=args.batch)
    K_p, K_r, steps = (4, 3, 5) if args.kinds else (cfg.K_p, cfg.K_r, args.steps)
    t0 = time.time()
    with ThreadPoolExecutor(max_workers=8) as ex:
        ws = list(ex.map(lambda l: I.layer_weights(cfg, l), range(cfg.T)))
    print(f"weights {time.time() - t0:.0f}s", flush=True)
    sched = I.TokenSchedule(cfg, stress=True)
    model = O.Model(cfg.T, cfg.d, cfg.H_q, cfg.H_kv, cfg.d_h, cfg.m, cfg.rms_eps, cfg.rope_theta)
    ora = O.CachedDenoiser(model, ws, cfg.B, cfg.L_p, cfg.L_r, cfg.rho, K_p, K_r, storage="bf16")
    shadow = NF.Shadow(ora)
    kinds = []
    for i in range(steps):
        h = sched.hidden_in(i)
        out, rep = ora.step(h.astype(np.float64), i)
        shadow.follow(h, i, rep, out)
        kinds.append(("P" if rep.prompt_refresh else "-") + ("R" if rep.response_refresh else "a"))
        print(f"step {i} [{kinds[-1]}] done {time.time() - t0:.0f}s  hidden_out {shadow.hidden_out}", flush=True)
    res = {"_about": "distances between the oracle accumulating in float32 and in float64, bf16 storage "
                     "rounding in both, maxima over the steps taken; written by "
                     "tests/golden/make_bf16_noise_floor.py (oracle only): " + " ".join(sys.argv[1:]),
           "config": cfg.name, "T": cfg.T, "B": cfg.B, "K_p": K_p, "K_r": K_r, "step_kinds": kinds}
    res.update(shadow.floor())
    name = cfg.name + (f"_T{cfg.T}" if args.layers else "")
    path = os.path.join(ROOT, "tests", "golden", f"noise_floor_{name}.json")
    json.dump(res, open(path, "w"), indent=1)
    print("wrote", path, flush=True)


if __name__ == "__main__":
    main()
