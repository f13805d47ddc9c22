"""Oracle slice strategy (the paper's Algorithm 1) pinned by its closed form (the start/end
equation of the direct-slicing section) and by the properties both imply."""
import math

import pytest

import oracle


def closed_form(d_in: int, p: int):
    """The paper's start/end equation, 1-based inclusive, turned into 0-based half-open.

    Slice i (1..p) covers [(i-1)*c + 1, i*c] when i*c < d', else [d' - c + 1, d'],
    with c = ceil(d'/p) (the equation's stray 'd' is read as d')."""
    c = math.ceil(d_in / p)
    out = []
    for i in range(1, p + 1):
        if i * c < d_in:
            start, end = (i - 1) * c + 1, i * c
        else:
            start, end = d_in - c + 1, d_in
        out.append((start - 1, end))
    return out, c


def test_hand_examples():
    assert oracle.slice_strategy(7, 2) == ([(0, 4), (3, 7)], 4)
    assert oracle.slice_strategy(128, 4) == ([(0, 32), (32, 64), (64, 96), (96, 128)], 32)
    assert oracle.slice_strategy(301, 3) == ([(0, 101), (101, 202), (200, 301)], 101)
    assert oracle.slice_strategy(5, 5) == ([(i, i + 1) for i in range(5)], 1)
    assert oracle.slice_strategy(9, 1) == ([(0, 9)], 9)


def test_algorithm_equals_closed_form_everywhere():
    checked = 0
    for d in range(1, 161):
        for p in range(1, d + 1):
            c = math.ceil(d / p)
            got, size = oracle.slice_strategy(d, p)
            want, c2 = closed_form(d, p)
            assert size == c2 == c
            assert got == want, (d, p)
            checked += 1
    assert checked == 160 * 161 // 2


@pytest.mark.parametrize("d,p", [(7, 2), (10, 3), (100, 4), (301, 2), (301, 3), (602, 2), (256, 8), (13, 5)])
def test_properties(d, p):
    sl, c = oracle.slice_strategy(d, p)
    assert len(sl) == p
    assert all(e - s == c for s, e in sl)                   # equal widths
    covered = set()
    for s, e in sl:
        assert 0 <= s < e <= d
        covered |= set(range(s, e))
    assert covered == set(range(d))                          # union is the whole feature axis
    overlap = sum(e - s for s, e in sl) - d
    assert overlap == p * c - d                              # only the shifted last slice overlaps
    disjoint = all(sl[i][1] <= sl[i + 1][0] for i in range(p - 1))
    assert disjoint == (d % p == 0)


def test_scale():
    # int(slice_size * scale) truncates toward zero
    sl, c = oracle.slice_strategy(100, 4, 0.5)
    assert c == 25 and sl == [(0, 12), (25, 37), (50, 62), (75, 87)]
    sl, c = oracle.slice_strategy(100, 4, 1.5)   # 37 wide: overlaps, last one shifted to end at 100
    assert sl == [(0, 37), (25, 62), (50, 87), (63, 100)]


@pytest.mark.parametrize("args", [(0, 1, 1.0), (4, 0, 1.0), (4, 5, 1.0), (4, 2, 0.0), (4, 2, -1.0), (4, 2, 0.1), (4, 2, 3.0)])
def test_rejects(args):
    with pytest.raises(ValueError):
        oracle.slice_strategy(*args)
