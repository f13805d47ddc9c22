"""Model-shape bookkeeping pinned by the parameter counts the paper prints (Table III)."""
import math
import os

import pytest

from synth import model

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table3_param_counts.txt")
DATASETS = {  # F, C, L  (Tables I and II of the paper)
    "Rom.": (300, 18, 3), "Amz.": (300, 5, 4), "Mine.": (7, 2, 7),
    "Tol.": (10, 2, 4), "Ques.": (301, 2, 6), "OGB.": (128, 40, 4),
}
ORDER = ["Rom.", "Amz.", "Mine.", "Tol.", "Ques.", "OGB."]
HIDDEN = 512  # the only width that reproduces every printed count


def _rows():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        out.append((tok[0], int(tok[1]), tok[2:]))
    return out


def _fmt(n: int, like: str) -> str:
    """Render n the way the table does: two decimals with a K or M suffix."""
    if like.endswith("M"):
        return f"{n / 1e6:.2f}M"
    return f"{n / 1e3:.2f}K"


def _count(method: str, p: int, F: int, C: int, L: int) -> int:
    if method == "GCN":
        shapes = model.param_shapes(F, C, L, 1, HIDDEN, first_in=F, slice_hidden=HIDDEN)
        # the single-GPU baseline's classifier input is the plain hidden width
        return model.param_count(shapes)
    h = math.ceil(HIDDEN / p)
    s = F // p + 1  # slice width implied by the printed counts
    shapes = model.param_shapes(F, C, L, p, HIDDEN, first_in=s, slice_hidden=h,
                                slice_encoding=method in ("SE", "FFSE"),
                                feature_fusion=method in ("FF", "FFSE"))
    return model.param_count(shapes)


@pytest.mark.parametrize("method,p,printed", _rows())
def test_table3_counts(method, p, printed):
    assert len(printed) == 6
    for ds, text in zip(ORDER, printed):
        F, C, L = DATASETS[ds]
        n = _count(method, p, F, C, L)
        assert _fmt(n, text) == text, (method, p, ds, n, text)


def test_table_has_54_entries():
    assert sum(len(r[2]) for r in _rows()) == 54
