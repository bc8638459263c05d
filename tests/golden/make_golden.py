"""Writes tests/golden/tiny_sla_oracle.json from the CPU oracle alone.

The paper prints no worked numeric example for this path, so no stored value
here is the paper's: these are the oracle's own outputs on the seeded tiny
config (B=1, H=2, N=1024, d=128, 64x64 blocks, 20 % critical, 40 % marginal,
seed 0), kept so that an unintended change to the oracle's arithmetic shows up
as a diff.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import sla_oracle as so          # noqa: E402
from paper_2512_16093_amd import synth       # noqa: E402  (input generator only)

ROWS = [0, 100, 517, 1023]
COLS = [0, 17, 127]


def build():
    cfg = synth.CONFIGS[0]
    W = synth.as_f64(synth.make_proj(cfg))
    doc = {"config": "tiny seed 0", "rows": ROWS, "cols": COLS, "heads": []}
    for h in range(cfg.H):
        q, k, v = (synth.as_f64(t) for t in synth.make_head(cfg, 0, h))
        entry = {}
        for mode in (so.QUANT_NONE, so.QUANT_QK_INT8, so.QUANT_QK_INT8_PV_FP8):
            r = so.sla_forward_head(q, k, v, cfg.block_q, cfg.block_k, cfg.topk_ratio,
                                    cfg.marginal_ratio, proj_w=W, quant=mode)
            entry[mode] = [[float(r["out"][n, c]) for c in COLS] for n in ROWS]
        entry["mask"] = r["mask"].tolist()
        entry["scores_row0"] = [float(x) for x in r["scores"][0]]
        doc["heads"].append(entry)
    return doc


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_sla_oracle.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1)
    print("wrote", path)
