"""Writes tests/golden/tiny_oracle.json from the CPU oracle alone (never from the HIP path).

Run from the repository root:  python tests/golden/make_tiny_golden.py
"""
import json
import sys
from pathlib import Path

import numpy as np

ROOT = Path(__file__).resolve().parents[2]
sys.path.insert(0, str(ROOT))

import oracle  # noqa: E402
from paper_2406_18139_amd import workloads as W  # noqa: E402

q, k, v, mask = W.generate(W.TINY)
r = oracle.compress(q, k, v, mask.numpy(), W.TINY.budget(), W.TINY.M, "averaged")
out = {
    "kept": r["kept"].tolist(),
    "assign": r["assign"].tolist(),
    "scores": [[repr(float(x)) for x in row] for row in r["scores"]],
    # merged rows are pinned through their per-row sums over the head dimension
    "k_out_rowsum": [[repr(float(x)) for x in row] for row in r["k_out"].sum(-1)],
    "v_out_rowsum": [[repr(float(x)) for x in row] for row in r["v_out"].sum(-1)],
}
(Path(__file__).parent / "tiny_oracle.json").write_text(json.dumps(out, indent=0))
print("wrote tiny_oracle.json")
