import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _gpu_present():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _gpu_present():
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def read_golden_ctx_lists():
    """Parses tests/golden/ctx_lists.txt into (clip_len, n_clips, w, global, clip, expected)."""
    path = os.path.join(ROOT, "tests", "golden", "ctx_lists.txt")
    cases = []
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, g, clip, exp = [s.strip() for s in line.split(";")]
            clip_len, n_clips, w = [int(x) for x in head.split()]
            cases.append((clip_len, n_clips, w, [int(x) for x in g.split()], int(clip),
                          [int(x) for x in exp.split()]))
    return cases
