"""Writes tests/golden/oracle_small.json from the CPU oracle alone.

Run from the repository root:  python tests/golden/make_golden.py
The file is a drift guard: it stores what the oracle (and nothing else) returned
for the two smallest synthetic workloads when its pins were last green, so an
accidental change to the oracle's arithmetic or to the generators shows up.
It imports only the input generators and the oracle.
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import kvsynth                                   # noqa: E402
from kvsynth.generate import generate           # noqa: E402
from oracle import flashcache_ref as ref         # noqa: E402


def summarise(name, route):
    cfg = kvsynth.get_config(name)
    K, V = generate(cfg, workers=4)
    r = ref.cutoff_r(cfg.n_tokens, cfg.gamma)
    T = ref.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
    out = ref.compress(K, V, cfg.dtype, r, T, route=route)
    return {
        "config": name, "route": route, "r": r, "total_budget": T,
        "input_sha256": hashlib.sha256(K.tobytes() + V.tobytes()).hexdigest(),
        "budgets": out["budgets"].tolist(),
        "ratios": [[float(f"{x:.12e}") for x in row] for row in out["ratios"]],
        "idx_sha256": hashlib.sha256(np.ascontiguousarray(out["idx"]).tobytes()).hexdigest(),
        "idx_head": out["idx"][0, :16].tolist(),
        "score_sum": float(f"{out['score64'].sum():.12e}"),
        "kout_sha256": hashlib.sha256(np.ascontiguousarray(out["K_out"]).tobytes()).hexdigest(),
    }


if __name__ == "__main__":
    data = {"note": "written by tests/golden/make_golden.py from oracle/ only",
            "cases": [summarise("tiny", "definition"), summarise("mid", "fast")]}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_small.json")
    with open(path, "w") as f:
        json.dump(data, f, indent=1)
    print("wrote", path)
