"""Pins for the oracle's end-to-end driver (Alg. 3: PVTP at prefill, VTA at decode)."""
import math

import numpy as np
import pytest

from oracle import st3_oracle as orc
from workloads import decode_qkv, get_workload, prefill_qkv


def _mini(seed, B, H, N0, d, L, T):
    rng = np.random.default_rng(seed)
    pre = [tuple(rng.standard_normal((B, H, N0, d)) for _ in range(3)) for _ in range(L)]
    dec = [[tuple(rng.standard_normal((B, H, d)) for _ in range(3)) for _ in range(L)] for _ in range(T)]
    return pre, dec


def test_keep_everything_equals_plain_attention_over_the_growing_sequence():
    """keep ratio 1.0: prefill is dense causal attention and decode step t is the
    last row of dense causal attention over prompt + t generated tokens."""
    B, H, d, L, T = 2, 2, 8, 3, 4
    ns, nv, nx = 2, 6, 3
    N0 = ns + nv + nx
    pre, dec = _mini(0, B, H, N0, d, L, T)
    keep = np.full((L, T + 1), nv)
    g = orc.Generation(L, H, d, ns, nv, nx, keep)
    r = g.prefill(lambda l: pre[l])
    for l in range(L):
        O, A = orc.causal_attention(*pre[l])
        for b in range(B):
            np.testing.assert_allclose(r["out"][l][b], O[b], atol=1e-12)
            np.testing.assert_allclose(r["mass"][l][b], A[b, :, -1, ns:ns + nv].mean(0), atol=1e-13)
            assert r["selected"][l][b] is None
    for t in range(1, T + 1):
        s = g.decode_step(lambda l: dec[t - 1][l])
        for l in range(L):
            Qf = np.concatenate([pre[l][0]] + [dec[u][l][0][:, :, None] for u in range(t)], axis=2)
            Kf = np.concatenate([pre[l][1]] + [dec[u][l][1][:, :, None] for u in range(t)], axis=2)
            Vf = np.concatenate([pre[l][2]] + [dec[u][l][2][:, :, None] for u in range(t)], axis=2)
            O, A = orc.causal_attention(Qf, Kf, Vf)
            for b in range(B):
                np.testing.assert_allclose(s["out"][l][b], O[b, :, -1], atol=1e-12)
                assert s["kv_len"][l][b] == N0 + t


def test_pruned_run_invariants_and_masked_equivalence():
    B, H, d, L, T = 2, 3, 8, 5, 6
    ns, nv, nx = 3, 16, 4
    N0 = ns + nv + nx
    pre, dec = _mini(1, B, H, N0, d, L, T)
    keep0 = [16, 16, 12, 12, 5]
    keep = orc.keep_anneal(keep0, T, "cos", T + 2)
    g = orc.Generation(L, H, d, ns, nv, nx, keep)
    r = g.prefill(lambda l: pre[l])
    scale = 1 / math.sqrt(d)
    for b in range(B):
        for l in range(L):
            ids = r["ids"][l][b]
            assert len(ids) == keep0[l] and np.all(np.diff(ids) > 0)
            if l:
                assert set(ids) <= set(r["ids"][l - 1][b])            # nested over layers
            # same result from dense attention with the dropped keys masked out
            rows = np.concatenate([np.arange(ns), ns + ids, ns + nv + np.arange(nx)])
            dead = np.ones(N0, bool); dead[rows] = False
            for h in range(H):
                s = pre[l][0][b, h] @ pre[l][1][b, h].T * scale
                s[:, dead] = -np.inf
                s[np.triu_indices(N0, 1)] = -np.inf
                e = np.exp(s - s.max(-1, keepdims=True)); a = e / e.sum(-1, keepdims=True)
                np.testing.assert_allclose((a @ pre[l][2][b, h])[rows], r["out"][l][b][h], atol=1e-12)
        # layer 2 drops the 4 lowest of layer 1's mass; layer 4 the 7 lowest of layer 3's
        m1 = r["mass"][1][b]
        assert set(r["ids"][2][b]) == set(np.argsort(-m1)[:12])
        m3, ids3 = r["mass"][3][b], r["ids"][3][b]
        assert set(r["ids"][4][b]) == set(ids3[np.argsort(-m3)[:5]])
        # ranking columns: layers 0,1 own mass; layers 2,3 <- mass_1 cut; layer 4 <- mass_3 cut
        np.testing.assert_array_equal(g.rho[0][b], r["mass"][0][b])
        np.testing.assert_array_equal(g.rho[1][b], r["mass"][1][b])
        np.testing.assert_array_equal(g.rho[2][b], m1[r["ids"][2][b]])
        np.testing.assert_array_equal(g.rho[3][b], g.rho[2][b])
        np.testing.assert_array_equal(g.rho[4][b], m3[np.searchsorted(ids3, r["ids"][4][b])])
    prev_ids = [[x.copy() for x in g.ids[l]] for l in range(L)]
    rho0 = [[x.copy() for x in g.rho[l]] for l in range(L)]
    ids0 = [[x.copy() for x in g.ids[l]] for l in range(L)]
    for t in range(1, T + 1):
        s = g.decode_step(lambda l: dec[t - 1][l])
        for l in range(L):
            for b in range(B):
                ids = s["ids"][l][b]
                assert len(ids) == keep[l, t]
                assert set(ids) <= set(prev_ids[l][b])                 # nested over steps
                assert s["kv_len"][l][b] == orc.kv_len(ns, keep[l, t], nx, t)
                # static mode: survivors are a prefix of the prefill ranking (Eq. 7)
                order = ids0[l][b][np.argsort(-rho0[l][b], kind="stable")]
                assert set(ids) == set(order[:keep[l, t]])
                m = s["mass"][l][b]
                assert m.shape == (keep[l, t],) and np.all(m >= 0) and m.sum() <= 1
        prev_ids = s["ids"]
    # closed-form KV bytes equal the bytes actually held
    lens = g.cache_lens()
    held = sum(g.K[l][b].nbytes + g.V[l][b].nbytes for l in range(L) for b in range(B)) // 8 * 2
    assert held == orc.kv_bytes(B, H, d, 2, lens)


def test_current_mode_reranks_by_latest_mass():
    B, H, d, L, T = 1, 2, 8, 1, 3
    ns, nv, nx = 1, 10, 2
    pre, dec = _mini(2, B, H, ns + nv + nx, d, L, T)
    keep = np.array([[10, 8, 6, 4]])
    g = orc.Generation(L, H, d, ns, nv, nx, keep, mode="current")
    g.prefill(lambda l: pre[l])
    last_mass, last_ids = g.rho[0][0].copy(), g.ids[0][0].copy()
    for t in range(1, T + 1):
        s = g.decode_step(lambda l: dec[t - 1][l])
        want = set(last_ids[np.argsort(-last_mass)[:keep[0, t]]])
        assert set(s["ids"][0][0]) == want
        last_mass, last_ids = s["mass"][0][0], s["ids"][0][0]


def test_tiny_workload_counts_and_visual_segment_emptying():
    w = get_workload("tiny")
    keep = orc.schedule_for(w)
    g = orc.Generation(w.layers, w.heads, w.head_dim, w.n_sys, w.n_vis, w.n_txt, keep)
    r = g.prefill(lambda l: prefill_qkv(w, l, 1))
    assert [len(x[0]) for x in r["ids"]] == [64, 32]
    for t in range(1, w.steps + 1):
        s = g.decode_step(lambda l: decode_qkv(w, l, t, 1))
    assert [len(x[0]) for x in s["ids"]] == [32, 0]
    assert s["mass"][1][0].shape == (0,)
    assert g.cache_lens() == [8 + 32 + 16 + 8, 8 + 0 + 16 + 8]


def test_workload_inputs_are_reproducible_and_bf16_exact():
    from workloads import bf16_round_bits
    from workloads.synth import bf16_bits_to_f32
    w = get_workload("llava15_7b")
    q1, k1, v1 = decode_qkv(w, 3, 5, 2)
    q2, k2, v2 = decode_qkv(w, 3, 5, 2)
    assert np.array_equal(q1, q2) and np.array_equal(k1, k2) and np.array_equal(v1, v2)
    assert not np.array_equal(q1, decode_qkv(w, 3, 6, 2)[0])
    assert np.array_equal(bf16_bits_to_f32(bf16_round_bits(k1)), k1)     # already bf16 values
    assert abs(float(k1.std()) - w.sigma) < 0.05 * w.sigma
    # round-to-nearest-even at the half-way point
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8)], np.float32)
    assert bf16_bits_to_f32(bf16_round_bits(x)).tolist() == [1.0, 1.0 + 2.0 ** -6, -1.0]


def test_planted_workload_structure():
    from workloads.synth import planted_layout
    w = get_workload("skewed_13b")
    import dataclasses
    ws = dataclasses.replace(w, heads=2, layers=1)
    hot, exact, near, u = planted_layout(ws)
    assert len(hot) == 58 and exact.shape == (32, 8) and near.shape == (16, 8)
    q, k, v = prefill_qkv(ws, 0, 1)
    s0 = ws.n_sys
    for grp in exact[:3]:
        for m in grp[1:]:
            assert np.array_equal(k[0, :, s0 + m], k[0, :, s0 + grp[0]])
    grp = near[0]
    diff = k[0, :, s0 + grp[1]] != k[0, :, s0 + grp[0]]
    assert diff.sum() == 1 and diff[0, 1]
    # hot keys take roughly 90 % of the last row's visual mass
    _, mass = orc.prefill_attention(q, k, v, ws.n_sys, ws.n_vis)
    frac = mass[0, hot].sum() / mass[0].sum()
    assert 0.75 < frac < 0.98
    # exact-tie groups tie in fp64 mass as well (identical keys in every head)
    assert mass[0, exact[0][0]] == mass[0, exact[0][5]]
