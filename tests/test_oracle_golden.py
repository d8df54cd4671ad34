"""Drift guard: the oracle still returns what tests/golden/oracle_small.json recorded."""
import hashlib
import json
import os

import numpy as np

import kvsynth
from kvsynth.generate import generate
from oracle import flashcache_ref as ref

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "oracle_small.json")


def test_oracle_reproduces_golden_summaries():
    with open(GOLDEN) as f:
        cases = json.load(f)["cases"]
    for case in cases:
        cfg = kvsynth.get_config(case["config"])
        K, V = generate(cfg, workers=4)
        assert hashlib.sha256(K.tobytes() + V.tobytes()).hexdigest() == case["input_sha256"]
        r = ref.cutoff_r(cfg.n_tokens, cfg.gamma)
        T = ref.total_budget(cfg.layers, cfg.n_tokens, cfg.rho)
        assert (r, T) == (case["r"], case["total_budget"])
        out = ref.compress(K, V, cfg.dtype, r, T, route=case["route"])
        assert out["budgets"].tolist() == case["budgets"]
        assert np.allclose(out["ratios"], np.array(case["ratios"]), rtol=1e-9)
        assert out["idx"][0, :16].tolist() == case["idx_head"]
        assert hashlib.sha256(np.ascontiguousarray(out["idx"]).tobytes()).hexdigest() == case["idx_sha256"]
        assert hashlib.sha256(np.ascontiguousarray(out["K_out"]).tobytes()).hexdigest() == case["kout_sha256"]
        assert abs(out["score64"].sum() - case["score_sum"]) <= 1e-9 * case["score_sum"]
