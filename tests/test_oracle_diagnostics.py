"""Pins for the oracle's diagnostics: Overlap_n (Eq. 10) and cosine similarity (Eq. 4-5)."""
import math

import numpy as np
import pytest

from conftest import read_table
from oracle import st3_oracle as orc


def test_printed_overlap_values_are_multiples_of_one_over_288():
    """Every printed percentage is m/288 for an integer m: the compared sets hold 288 = 576/2 tokens,
    and they are compared as sets.  The oracle reproduces each value on vectors built to share m ids."""
    rows = read_table("overlap_table.txt")
    assert len(rows) == 10 and rows[0] == ["1", "100.00"]
    n, k = 576, 288
    base = np.arange(n, 0, -1).astype(float)             # token i scores n - i: top-k = ids 0..287
    ids = np.arange(n)
    for step, pct in rows:
        m = round(float(pct) * k / 100.0)
        assert abs(100.0 * m / k - float(pct)) < 0.005, (step, pct)
        other = base.copy()
        # push k - m of the first step's top tokens below everything else
        other[:k - m] = -1.0 - np.arange(k - m)
        assert orc.overlap(base, ids, other, ids, k) == m / k
        assert round(100.0 * orc.overlap(base, ids, other, ids, k), 2) == float(pct)


def test_overlap_definition_against_python_sets():
    rng = np.random.default_rng(0)
    for n_a, n_b, k in [(50, 50, 25), (64, 40, 10), (30, 30, 30), (20, 35, 0 + 7)]:
        ids_a = rng.permutation(100)[:n_a]; ids_b = rng.permutation(100)[:n_b]
        sa = rng.standard_normal(n_a); sb = rng.standard_normal(n_b)
        top_a = set(ids_a[np.argsort(-sa)[:k]].tolist()); top_b = set(ids_b[np.argsort(-sb)[:k]].tolist())
        assert orc.overlap(sa, ids_a, sb, ids_b, k) == len(top_a & top_b) / len(top_a)
    x = rng.standard_normal(40); ids = np.arange(40)
    assert orc.overlap(x, ids, x, ids, 20) == 1.0                          # Overlap_1 = 100 %
    assert orc.overlap(x, ids, x[::-1].copy(), ids[::-1].copy(), 20) == 1.0  # order of storage is irrelevant
    assert orc.overlap(x, ids, -x, ids, 20) == 0.0                         # disjoint halves


def test_cosine_similarity_closed_forms():
    ids = np.arange(6)
    x = np.array([1.0, 2.0, 3.0, 0.5, 0.0, 4.0])
    assert orc.cosine_similarity(x, ids, x, ids) == pytest.approx(1.0, abs=1e-15)
    assert orc.cosine_similarity(x, ids, -x, ids) == pytest.approx(-1.0, abs=1e-15)
    assert orc.cosine_similarity(x, ids, 7.5 * x, ids) == pytest.approx(1.0, abs=1e-15)       # scale invariant
    assert orc.cosine_similarity([1, 0], [0, 1], [0, 1], [0, 1]) == 0.0                        # orthogonal
    assert orc.cosine_similarity([1, 1], [0, 1], [1, 0], [0, 1]) == pytest.approx(math.sqrt(0.5), abs=1e-15)
    perm = np.array([3, 1, 5, 0, 4, 2])
    y = np.array([0.2, 1.0, 2.5, 0.1, 3.0, 0.7])
    want = float(x @ y) / math.sqrt(float(x @ x) * float(y @ y))
    assert orc.cosine_similarity(x[perm], ids[perm], y, ids) == pytest.approx(want, abs=1e-15)   # matched by id
    # a token missing on one side counts as zero there
    assert orc.cosine_similarity([3, 4], [10, 11], [3], [10]) == pytest.approx(9 / (5 * 3), abs=1e-15)
    assert orc.cosine_similarity([0, 0], [0, 1], [1, 2], [0, 1]) == 0.0
    # library cross-check
    rng = np.random.default_rng(1)
    a, b = rng.standard_normal(100), rng.standard_normal(100)
    lib = float(np.dot(a, b) / (np.linalg.norm(a) * np.linalg.norm(b)))
    assert orc.cosine_similarity(a, np.arange(100), b, np.arange(100)) == pytest.approx(lib, abs=1e-14)
