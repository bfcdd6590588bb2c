import os
import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for it in items:
        if "gpu" in it.keywords:
            it.add_marker(skip)


def pytest_sessionfinish(session, exitstatus):
    """With LOOKM_PARITY_STATS=<file>: the statistics every GPU parity run recorded (tests/parity.py), as a table."""
    path = os.environ.get("LOOKM_PARITY_STATS")
    if not path:
        return
    try:
        from tests import parity
    except Exception:
        return
    if not parity.STATS:
        return
    cols = ["workload", "layer", "mode", "rule", "H", "L", "B", "M", "heads", "heads_oracle", "kept_diff_heads",
            "min_margin", "nearest_tie_rows", "rows_matched", "score_relerr", "sim_abserr", "merge_abserr"]

    def fmt(v):
        if v is None:
            return "-"
        if isinstance(v, float):
            return f"{v:.3e}"
        return str(v)

    rows = [[fmt(st.get(c)) for c in cols] for st in parity.STATS]
    width = [max(len(c), *(len(r[i]) for r in rows)) for i, c in enumerate(cols)]
    with open(path, "w") as f:
        f.write("GPU path against the CPU oracle, one line per checked call (tests/parity.py):\n"
                "heads = heads run on the GPU, all of them checked stage by stage (selection on the kernel's own scores, the\n"
                "matching against the fp64 oracle's on the call's own lists, merge on the call's own matching); heads_oracle =\n"
                "heads whose scores and kept sets are also compared with the fp64 oracle end to end; kept_diff_heads = of\n"
                "those, heads whose kept set differs from the oracle's; min_margin = smallest relative gap between the last\n"
                "conserved and the first evicted competing score (fp64 oracle); nearest_tie_rows = evicted keys matched to\n"
                "another slot than the oracle's, of rows_matched (all heads); score_relerr, sim_abserr, merge_abserr = largest\n"
                "errors seen (scores relative, cosines absolute, merged rows absolute against unrounded fp64).\n"
                f"pytest exit status {int(exitstatus)}\n\n")
        f.write("  ".join(c.ljust(width[i]) for i, c in enumerate(cols)) + "\n")
        for r in rows:
            f.write("  ".join(x.ljust(width[i]) for i, x in enumerate(r)) + "\n")
