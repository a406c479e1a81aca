"""Pins of the oracle's TopK-I (Sec. 4.1): brute force on tiny inputs and set properties."""
import json
import os

import numpy as np
import pytest

from oracle import fasa_oracle as O

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "tiny_hand_worked.json")))


def _brute(s, b):
    """Pick the maximum b times; among equal values the lowest index wins.  Pure Python."""
    s = [float(x) for x in s]
    left = list(range(len(s)))
    out = []
    for _ in range(min(b, len(s))):
        best = left[0]
        for i in left[1:]:
            if s[i] > s[best]:
                best = i
        out.append(best)
        left.remove(best)
    return sorted(out)


def test_hand_worked_selection():
    assert O.topk_indices(np.array(GOLD["S_fc1"]), 1).tolist() == GOLD["top1_fc1"]
    assert O.topk_indices(np.array(GOLD["S_fc0"]), 1).tolist() == GOLD["top1_fc0"]
    assert O.topk_indices(np.array(GOLD["S_fc1"]), 2).tolist() == GOLD["top2_fc1"]


@pytest.mark.parametrize("n", [1, 2, 5, 17, 64])
def test_brute_force_all_budgets(n):
    rng = np.random.default_rng(n)
    for trial in range(3):
        s = rng.standard_normal(n).astype(np.float32)
        if trial == 1:
            s = np.round(s * 2) / 2          # many exact duplicates
        if trial == 2:
            s[::3] = 0.0
            s[1::3] = -0.0                   # +0 and -0 compare equal
        for b in range(1, n + 3):
            assert O.topk_indices(s, b).tolist() == _brute(s, b)


def test_properties_on_a_long_row():
    rng = np.random.default_rng(11)
    n, b = 5000, 321
    s = rng.standard_normal(n).astype(np.float32)
    t = O.topk_indices(s, b)
    assert len(t) == b and len(set(t.tolist())) == b and t.min() >= 0 and t.max() < n
    mask = np.zeros(n, bool); mask[t] = True
    assert s[mask].min() >= s[~mask].max()
    assert O.topk_indices(s, 1)[0] == int(np.argmax(s))
    assert O.topk_indices(s, n).tolist() == list(range(n))
    assert O.topk_indices(s, n + 10).tolist() == list(range(n))


def test_ties_go_to_the_lower_index():
    s = np.array([1.0, 3.0, 3.0, 3.0, 0.0, 3.0], dtype=np.float32)
    assert O.topk_indices(s, 2).tolist() == [1, 2]
    assert O.topk_indices(s, 3).tolist() == [1, 2, 3]
    assert O.topk_indices(s, 5).tolist() == [0, 1, 2, 3, 5]


def test_batched_wrapper_shapes():
    rng = np.random.default_rng(12)
    S = rng.standard_normal((2, 3, 50)).astype(np.float32)
    T = O.topk(S, 7, 40)
    assert T.shape == (2, 3, 7) and T.max() < 40
    for b in range(2):
        for h in range(3):
            assert T[b, h].tolist() == _brute(S[b, h, :40], 7)
