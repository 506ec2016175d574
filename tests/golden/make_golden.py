"""Writes tests/golden/c1_oracle.json: the oracle's results on the tiny config.

Calls only oracle/ and the seeded generators.  The paper prints no worked
numeric example of tree attention or of the acceptance walk (Section 2.1 gives
the rule, Section 4 only end-to-end ratios), so these stored values are the
oracle's own; they guard against silent drift of the oracle or the generators,
and they are not a pin (the pins are the invariant tests).

    python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import accept_path, tree_verify_attention  # noqa: E402
from workloads import CONFIGS, accept_inputs, attention_inputs, tree_for_config  # noqa: E402


def main():
    cfg = CONFIGS["c1_tiny"]
    par = tree_for_config(cfg)
    x = attention_inputs(cfg)
    out = tree_verify_attention(**x, parent=par, prefix_len=[cfg.prefix_len])
    a = accept_inputs(cfg, par)
    r = accept_path(a["tokens"][0], par[0], a["logits"][0], "greedy")
    doc = {
        "citation": "Section 2.1 steps 2-3 (verification, acceptance); Section 3.1.2 (tree mask)",
        "config": cfg.name,
        "parent": par[0].tolist(),
        "out_sum": float(out.sum()),
        "out_abs_sum": float(np.abs(out).sum()),
        "out_samples": {f"{i},{h},{d}": float(out[0, i, h, d])
                        for (i, h, d) in [(0, 0, 0), (3, 1, 17), (9, 3, 63), (5, 2, 40)]},
        "greedy_path": r.path,
        "greedy_accept_len": r.accept_len,
        "greedy_bonus": r.bonus_token,
    }
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle.json"), "w") as f:
        json.dump(doc, f, indent=1)
        f.write("\n")


if __name__ == "__main__":
    main()
