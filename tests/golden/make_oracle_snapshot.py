"""Writes tests/golden/oracle_snapshot.json: what the oracle computes today for one tiny
seeded cache (sketch entries, scores, index sets, adaptive budgets), stored as exact
hexadecimal floats.  It calls only `oracle/` and the seeded input generators.

This is a guard against accidental edits of the oracle, not a pin: the values come from the
oracle itself.  A deliberate change of the oracle's arithmetic re-runs this script and says
so, with the passage of the paper that justifies it, in its commit message.

    python tests/golden/make_oracle_snapshot.py
"""

import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import curdkv_oracle as orc                      # noqa: E402
from paper_2509_15038_amd import workloads as wl             # noqa: E402


def snapshot():
    cfg = wl.scaled(wl.CONFIGS["c2"], layers=2, kv_heads=2, n=96, r=20)
    K, V = wl.host_cache(cfg)
    budgets = np.array([24, 5, 0, 96], dtype=np.int64)
    lt, idx, offsets, Kp, Vp = orc.compress(K, V, "bf16", cfg.sketch_seed, cfg.r, budgets, 4)
    G = orc.sketch(cfg.sketch_seed, 1, 0, 2, 128, cfg.r, "bf16")
    ada = orc.adaptive_budgets(lt[0], 24, 4, 0.2)
    key_only = orc.scores(orc.to_f64(K[0, 1], "bf16"), orc.to_f64(V[0, 1], "bf16"),
                          orc.sketch(cfg.sketch_seed, 0, 1, 2, 128, cfg.r, "bf16"), source="k")
    return {
        "config": {"layers": 2, "kv_heads": 2, "n": 96, "d": 128, "r": 20, "dtype": "bf16",
                   "seed": cfg.sketch_seed, "n_sink": 4, "budgets": budgets.tolist()},
        "sketch_l1_h0_first_row": [float(x).hex() for x in G[0]],
        "scores_l0_h0": [float(x).hex() for x in lt[0, 0]],
        "scores_l1_h1_sum": float(lt[1, 1].sum()).hex(),
        "indices": [s.tolist() for s in idx],
        "offsets": offsets.tolist(),
        "gathered_K_bits_first_row_of_group0": [int(x) for x in Kp[0]],
        "adaptive_budgets_layer0_k24_s4_alpha0.2": ada.tolist(),
        "key_only_scores_l0_h1_first8": [float(x).hex() for x in key_only[:8]],
    }


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_snapshot.json")
    with open(path, "w") as f:
        json.dump(snapshot(), f, indent=1)
        f.write("\n")
    print("wrote", path)
