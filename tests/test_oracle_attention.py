"""Pins for the oracle's attention and mass (Eq. 2 and Sec. 3.2 of the paper).

Each check compares the oracle with something fixed outside it: a library
routine on the special case it reduces to, a closed form, or an invariant.
"""
import math

import numpy as np
import pytest
import torch

from oracle import st3_oracle as orc


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def test_hand_worked_two_token_case():
    # d = 1, scale = 1.  Row 0 sees key 0 only.  Row 1: logits (0, ln 3) -> (1/4, 3/4).
    Q = np.array([[[[1.0], [1.0]]]])
    K = np.array([[[[0.0], [math.log(3.0)]]]])
    V = np.array([[[[1.0], [5.0]]]])
    O, A = orc.causal_attention(Q, K, V)
    np.testing.assert_allclose(A[0, 0], [[1.0, 0.0], [0.25, 0.75]], atol=1e-15)
    np.testing.assert_allclose(O[0, 0, :, 0], [1.0, 4.0], atol=1e-15)


def test_scale_is_one_over_sqrt_d():
    # d = 4, q = k = (1,1,1,1): q.k = 4, logit = 4/sqrt(4) = 2 against a zero key.
    Q = np.ones((1, 1, 2, 4)); K = np.zeros((1, 1, 2, 4)); K[0, 0, 1] = 1.0
    V = np.zeros((1, 1, 2, 4)); V[0, 0, 1] = 1.0
    O, A = orc.causal_attention(Q, K, V)
    want = math.exp(2.0) / (1.0 + math.exp(2.0))
    assert A[0, 0, 1, 1] == pytest.approx(want, abs=1e-15)
    assert O[0, 0, 1, 0] == pytest.approx(want, abs=1e-15)


@pytest.mark.parametrize("n,d", [(1, 8), (7, 16), (33, 64)])
def test_full_attention_matches_library_sdpa(n, d):
    Q, K, V = (_rand((2, 3, n, d), s) for s in (1, 2, 3))
    O, _ = orc.causal_attention(Q, K, V)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), is_causal=True).numpy()
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)
    O2, _ = orc.prefill_attention(Q, K, V, 2 if n > 4 else 0, min(3, n - 2) if n > 4 else 0)
    np.testing.assert_allclose(O2, ref, rtol=0, atol=1e-12)


def test_softmax_rows_sum_to_one_and_causal_zeros():
    Q, K, V = (_rand((1, 2, 19, 8), s) * 3 for s in (4, 5, 6))
    _, A = orc.causal_attention(Q, K, V)
    np.testing.assert_allclose(A.sum(-1), 1.0, atol=1e-12)
    iu = np.triu_indices(19, 1)
    assert np.all(A[0, 0][iu] == 0.0) and np.all(A[0, 1][iu] == 0.0)
    assert np.all(A >= 0)


def test_all_equal_keys_give_running_mean_of_values():
    n, d = 11, 8
    Q = _rand((1, 1, n, d), 7)
    K = np.tile(_rand((1, 1, 1, d), 8), (1, 1, n, 1))
    V = _rand((1, 1, n, d), 9)
    O, A = orc.causal_attention(Q, K, V)
    for i in range(n):
        np.testing.assert_allclose(O[0, 0, i], V[0, 0, :i + 1].mean(0), atol=1e-12)
    o, mass, p = orc.decode_attention(Q[:, :, -1], K, V, 2, 5)
    np.testing.assert_allclose(o[0, 0], V[0, 0].mean(0), atol=1e-12)
    np.testing.assert_allclose(mass[0], 1.0 / n, atol=1e-15)


def test_one_dominant_key_returns_its_value():
    n, d = 9, 4
    q = np.zeros((1, 1, d)); q[0, 0, 0] = 1.0
    K = np.zeros((1, 1, n, d)); K[0, 0, 6, 0] = 200.0
    V = _rand((1, 1, n, d), 10)
    o, mass, p = orc.decode_attention(q, K, V, 1, 7)
    np.testing.assert_allclose(o[0, 0], V[0, 0, 6], atol=1e-12)
    assert mass[0, 5] == pytest.approx(1.0, abs=1e-12)      # visual index 5 <-> key 6


def test_decode_is_last_row_of_causal_attention():
    B, H, n, d = 2, 3, 13, 16
    Q, K, V = (_rand((B, H, n, d), s) for s in (11, 12, 13))
    O, A = orc.causal_attention(Q, K, V)
    o, mass, p = orc.decode_attention(Q[:, :, -1], K, V, 3, 6)
    np.testing.assert_allclose(o, O[:, :, -1], atol=1e-12)
    np.testing.assert_allclose(p, A[:, :, -1], atol=1e-13)
    np.testing.assert_allclose(mass, A[:, :, -1, 3:9].mean(1), atol=1e-13)


def test_decode_invariant_under_cache_permutation():
    B, H, n, d = 1, 2, 17, 8
    q = _rand((B, H, d), 14); K = _rand((B, H, n, d), 15); V = _rand((B, H, n, d), 16)
    perm = np.random.default_rng(17).permutation(n)
    o1, _, p1 = orc.decode_attention(q, K, V, 0, n)
    o2, _, p2 = orc.decode_attention(q, K[:, :, perm], V[:, :, perm], 0, n)
    np.testing.assert_allclose(o1, o2, atol=1e-12)
    np.testing.assert_allclose(p1[:, :, perm], p2, atol=1e-14)


@pytest.mark.parametrize("window", [1, 2, 5])
def test_prefill_mass_is_window_rows_of_A_and_sums_to_window(window):
    B, H, n, d = 2, 3, 21, 8
    Q, K, V = (_rand((B, H, n, d), s) for s in (18, 19, 20))
    _, A = orc.causal_attention(Q, K, V)
    # every key position declared "visual": total mass = W exactly
    _, mass_all = orc.prefill_attention(Q, K, V, 0, n, window)
    np.testing.assert_allclose(mass_all.sum(-1), float(window), atol=1e-12)
    # a proper visual segment: equals the slice of A, mean over heads, sum over rows
    ns, nv = 4, 9
    _, mass = orc.prefill_attention(Q, K, V, ns, nv, window)
    want = A[:, :, n - window:, ns:ns + nv].sum(2).mean(1)
    np.testing.assert_allclose(mass, want, atol=1e-13)
    assert np.all(mass.sum(-1) <= window) and np.all(mass >= 0)


def test_token_drop_equals_key_mask():
    """Dropping visual rows before a layer equals masking those keys to -inf and
    ignoring those query rows (the two FastV implementations the paper cites)."""
    H, n, d = 2, 15, 8
    Q, K, V = (_rand((1, H, n, d), s) for s in (21, 22, 23))
    kept = np.array([0, 1, 2, 4, 7, 8, 11, 12, 13, 14])
    O_drop, _ = orc.causal_attention(Q[:, :, kept], K[:, :, kept], V[:, :, kept])
    scale = 1 / math.sqrt(d)
    for h in range(H):
        s = Q[0, h] @ K[0, h].T * scale
        bad = np.ones(n, bool); bad[kept] = False
        s[:, bad] = -np.inf
        s[np.triu_indices(n, 1)] = -np.inf
        e = np.exp(s - s.max(-1, keepdims=True)); a = e / e.sum(-1, keepdims=True)
        np.testing.assert_allclose((a @ V[0, h])[kept], O_drop[0, h], atol=1e-12)
