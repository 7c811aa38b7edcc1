"""Pins for the oracle's top-k rule (Eq. 3), retention schedules (Eq. 7-9,
Alg. 1) and KV-memory closed form (Table 2 of the paper)."""
import itertools
import math

import numpy as np
import pytest

from conftest import read_table
from oracle import st3_oracle as orc


# ---------------------------------------------------------------------------
# Eq. 3: top-G
# ---------------------------------------------------------------------------
def _kept_by_rank_count(scores, ids, k):
    """Independent definition: i is kept iff fewer than k entries beat it."""
    n = len(scores)
    keep = []
    for i in range(n):
        beats = sum(1 for j in range(n)
                    if scores[j] > scores[i] or (scores[j] == scores[i] and ids[j] < ids[i]))
        if beats < k:
            keep.append(i)
    return keep


def test_topk_exhaustive_small_with_ties():
    vals = [0.0, 0.5, 1.0]
    for n in range(0, 6):
        for scores in itertools.product(vals, repeat=n):
            for ids in ([*range(n)], [*range(n)][::-1]):
                for k in range(n + 1):
                    got = orc.select_topk(scores, ids, k).tolist()
                    assert got == _kept_by_rank_count(scores, ids, k), (scores, ids, k)


def test_topk_random_against_rank_count_and_argsort():
    rng = np.random.default_rng(0)
    for n in (1, 17, 64, 200):
        s = rng.standard_normal(n)
        s[rng.integers(0, n, n // 3)] = s[0]           # plant ties
        ids = rng.permutation(n)
        for k in (0, 1, n // 2, n - 1, n):
            k = max(0, min(n, k))
            got = orc.select_topk(s, ids, k).tolist()
            assert got == _kept_by_rank_count(s, ids, k)
    # no ties, ids = positions: the library's argsort gives the same set
    s = rng.standard_normal(300)
    got = orc.select_topk(s, np.arange(300), 77)
    assert set(got.tolist()) == set(np.argsort(-s)[:77].tolist())
    assert got.tolist() == sorted(got.tolist())


def test_topk_degenerate_cases_and_nestedness():
    n = 20
    assert orc.select_topk(np.ones(n), np.arange(n), 7).tolist() == list(range(7))
    ids = np.arange(n)[::-1].copy()       # lowest id sits at the highest position
    assert orc.select_topk(np.ones(n), ids, 3).tolist() == [17, 18, 19]
    assert orc.select_topk(np.ones(n), ids, 0).tolist() == []
    assert orc.select_topk(np.ones(n), ids, n).tolist() == list(range(n))
    s = np.random.default_rng(1).integers(0, 5, 40).astype(float)
    prev = set()
    for k in range(41):
        cur = set(orc.select_topk(s, np.arange(40), k).tolist())
        assert prev <= cur and len(cur) == k
        prev = cur
    # prefix of the ranked list == top-k set (Alg. 3's T[l][:m])
    order = orc.ranked_order(s, np.arange(40))
    for k in (0, 5, 23, 40):
        assert set(order[:k].tolist()) == set(orc.select_topk(s, np.arange(40), k).tolist())
    with pytest.raises(ValueError):
        orc.select_topk(s, np.arange(40), 41)


# ---------------------------------------------------------------------------
# Eq. 8 and Sec. 4.4
# ---------------------------------------------------------------------------
def test_beta_closed_form_values():
    fn = {"cos": orc.beta_cos, "linear": orc.beta_linear, "exp": orc.beta_exp}
    rows = read_table("beta_values.txt")
    assert len(rows) >= 15
    for kind, param, n_out, value in rows:
        assert fn[kind](int(n_out), float(param)) == pytest.approx(float(value), abs=1e-15)


def test_beta_cos_shape():
    tau = 50
    b = [orc.beta_cos(t, tau) for t in range(tau + 5)]
    d1 = np.diff(b[:tau + 1]); d2 = np.diff(d1)
    assert np.all(d1 < 0) and np.all(d2 < 0)         # decreasing and concave on [0, tau]
    assert all(x == 0.0 for x in b[tau:])
    lin = [orc.beta_linear(t, tau) for t in range(tau + 1)]
    assert all(c >= l - 1e-15 for c, l in zip(b, lin))   # cosine decays later than linear


# ---------------------------------------------------------------------------
# Eq. 9 / Alg. 1: stride schedule against the paper's printed (S, R, C) rows
# ---------------------------------------------------------------------------
def test_printed_stride_tables_reproduce_C():
    rows = read_table("pvtp_stride_tables.txt")
    assert len(rows) == 60
    for L, S, R, P, C in (tuple(map(int, r)) for r in rows):
        assert orc.conserved_ratio_bp(L, S, P, R) == C, (L, S, R, C)
        keep = orc.keep_pvtp(L, 576, S, P, R)
        assert keep[:3] == [576, 576, 576]
        assert keep[3] == 288                          # 50 % at the 4th layer
        assert keep[-1] == (576 * C) // 10000
        assert all(a >= b for a, b in zip(keep, keep[1:]))
        ev = orc.pvtp_events(L, S)
        assert ev[0] == 3 and all(b - a == S for a, b in zip(ev, ev[1:])) and ev[-1] <= L - 1
        # the token set is shared by the layers between two events
        for l in range(4, L):
            if l not in ev:
                assert keep[l] == keep[l - 1]


def test_linear_schedule_values():
    k13 = orc.keep_linear(40, 576, 2, 1000)
    assert k13[:4] == [576, 576, 576, 561] and k13[-1] == 57 and sum(k13) == 13161
    k7 = orc.keep_linear(32, 576, 2, 1000)
    assert k7[3] == 558 and k7[-1] == 57 and sum(k7) == 10641
    khr = orc.keep_linear(32, 2880, 2, 500)
    assert khr[3] == 2785 and khr[-1] == 144 and sum(khr) == 51106
    for k in (k13, k7, khr):
        assert all(a >= b for a, b in zip(k, k[1:]))
    # exact-rational check of one interior value: ceil(576*0.9*17/37) = 239
    assert k13[19] == 576 - math.ceil(576 * 9 * 17 / 370)


def test_anneal_table_monotone_and_endpoints():
    keep0 = orc.keep_linear(40, 576, 2, 1000)
    tab = orc.keep_anneal(keep0, 512, "cos", 512)
    assert tab.shape == (40, 513)
    assert np.all(tab[:, 0] == keep0)
    assert np.all(np.diff(tab, axis=1) <= 0) and np.all(np.diff(tab, axis=0) <= 0)
    assert np.all(tab[:, 512] == 0)                           # |O| >= tau: nothing left
    assert tab[0, 256] == math.floor(576 * math.sqrt(0.5))    # beta(tau/2) = sqrt(2)/2
    t3 = orc.keep_anneal([600], 90, "cos", 90)
    assert t3[0, 60] == 300 and t3[0, 30] == 519              # beta = 1/2, sqrt(3)/2
    td = orc.keep_anneal([64, 32], 8, "drop", 4)
    assert td[0].tolist() == [64, 60, 56, 52, 48, 44, 40, 36, 32]
    assert td[1].tolist() == [32, 28, 24, 20, 16, 12, 8, 4, 0]
    tl = orc.keep_anneal([100], 50, "linear", 50)
    assert tl[0, 25] == 50 and tl[0, 50] == 0
    te = orc.keep_anneal([1000], 40, "exp", 20)
    assert te[0, 20] == 367 and te[0, 40] == 135


# ---------------------------------------------------------------------------
# KV-cache memory (Table 2, baseline rows; batch 16, bf16)
# ---------------------------------------------------------------------------
def test_kv_bytes_matches_printed_baseline_memory():
    gib = 2.0 ** 30
    # LLaVA-1.5-7B: 32 layers x 32 heads x 128; 4.94 G printed <-> 632 cached tokens
    assert orc.kv_bytes(16, 32, 128, 2, [632] * 32) / gib == pytest.approx(4.94, abs=0.005)
    # LLaVA-1.5-13B: 40 x 40 x 128; 7.70 G printed <-> 631 cached tokens
    assert orc.kv_bytes(16, 40, 128, 2, [631] * 40) / gib == pytest.approx(7.70, abs=0.005)
    # one token, one layer, one head: K and V rows
    assert orc.kv_bytes(1, 1, 128, 2, [1]) == 512
    assert orc.kv_len(35, 576, 128, 0) == 739
    assert orc.kv_len(35, 57, 128, 10) == 230
