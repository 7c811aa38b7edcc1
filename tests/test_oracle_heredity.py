"""Pins for the oracle's QK heredity (Eq. 6, Alg. 2): a lazy layer applies the source layer's
attention probabilities to its own values."""
import numpy as np
import pytest
import torch

from oracle import st3_oracle as orc


def _mini(seed, B, H, N0, d, L, T):
    rng = np.random.default_rng(seed)
    pre = [tuple(rng.standard_normal((B, H, N0, d)) for _ in range(3)) for _ in range(L)]
    dec = [[tuple(rng.standard_normal((B, H, d)) for _ in range(3)) for _ in range(L)] for _ in range(T)]
    return pre, dec


def test_heredity_attention_against_library_sdpa_with_foreign_values():
    """Eq. 6 is ordinary causal attention whose values come from another layer: a library SDPA in
    float64 fed (Q_src, K_src, V_l) must agree."""
    rng = np.random.default_rng(3)
    Qs, Ks, Vl = (rng.standard_normal((2, 3, 17, 8)) for _ in range(3))
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Qs), torch.from_numpy(Ks), torch.from_numpy(Vl), is_causal=True).numpy()
    np.testing.assert_allclose(orc.heredity_attention(Qs, Ks, Vl), want, atol=1e-12)


def test_heredity_attention_closed_forms():
    rng = np.random.default_rng(4)
    B, H, n, d = 1, 2, 9, 9
    Qs, Ks = rng.standard_normal((B, H, n, d)), rng.standard_normal((B, H, n, d))
    # one-hot values: the output IS the probability matrix of the source layer
    eye = np.broadcast_to(np.eye(n), (B, H, n, n)).copy()
    P = orc.heredity_attention(Qs, Ks, eye)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-13)
    assert np.all(np.triu(P[0, 0], 1) == 0)
    Vl = rng.standard_normal((B, H, n, d))
    np.testing.assert_allclose(orc.heredity_attention(Qs, Ks, Vl), P @ Vl, atol=1e-12)
    # all source keys equal: uniform probabilities over the prefix, whatever the queries are
    Kc = np.broadcast_to(rng.standard_normal((B, H, 1, d)), (B, H, n, d))
    out = orc.heredity_attention(Qs, Kc, Vl)
    want = np.cumsum(Vl, axis=2) / np.arange(1, n + 1)[None, None, :, None]
    np.testing.assert_allclose(out, want, atol=1e-12)
    # linear in the values
    V2 = rng.standard_normal((B, H, n, d))
    np.testing.assert_allclose(orc.heredity_attention(Qs, Ks, 2 * Vl - V2),
                               2 * orc.heredity_attention(Qs, Ks, Vl) - orc.heredity_attention(Qs, Ks, V2), atol=1e-12)


@pytest.mark.parametrize("mode", ["static", "current"])
def test_lazy_layers_with_the_sources_values_repeat_the_sources_output(mode):
    """Feed the lazy layers the SAME value inputs as their source: Self-attn(Q^src, K^src, V^src)
    is the source's own attention, at prefill and at every decode step, through evictions."""
    B, H, d, L, T = 2, 2, 8, 5, 5
    ns, nv, nx = 2, 12, 3
    pre, dec = _mini(11, B, H, ns + nv + nx, d, L, T)
    lazy = {3: 2, 4: 2}
    for l in lazy:                                   # same values; Q and K inputs stay foreign and must be ignored
        pre[l] = (pre[l][0], pre[l][1], pre[2][2])
        for t in range(T):
            dec[t][l] = (dec[t][l][0], dec[t][l][1], dec[t][2][2])
    keep = np.array([[12] * 6, [12, 11, 10, 9, 8, 7], [8, 7, 6, 4, 2, 0], [8, 7, 6, 4, 2, 0], [8, 7, 6, 4, 2, 0]])
    g = orc.Generation(L, H, d, ns, nv, nx, keep, mode=mode, lazy=lazy)
    plain = orc.Generation(L, H, d, ns, nv, nx, keep, mode=mode)       # the same run without heredity
    r, rp = g.prefill(lambda l: pre[l]), plain.prefill(lambda l: pre[l])
    for l in lazy:
        for b in range(B):
            np.testing.assert_allclose(r["out"][l][b], r["out"][2][b], atol=1e-13)
            np.testing.assert_allclose(r["mass"][l][b], r["mass"][2][b], atol=1e-15)
            assert np.array_equal(r["ids"][l][b], r["ids"][2][b])
            assert g.K[l][b] is None
    for l in range(3):                               # layers up to the source do not notice
        for b in range(B):
            np.testing.assert_array_equal(r["out"][l][b], rp["out"][l][b])
    for t in range(1, T + 1):
        s, sp = g.decode_step(lambda l: dec[t - 1][l]), plain.decode_step(lambda l: dec[t - 1][l])
        for b in range(B):
            for l in lazy:
                np.testing.assert_allclose(s["out"][l][b], s["out"][2][b], atol=1e-13)
                np.testing.assert_allclose(s["mass"][l][b], s["mass"][2][b], atol=1e-15)
                assert np.array_equal(s["ids"][l][b], s["ids"][2][b])
                assert s["kv_len"][l][b] == s["kv_len"][2][b] == ns + keep[2][t] + nx + t
            for l in range(3):
                np.testing.assert_array_equal(s["out"][l][b], sp["out"][l][b])
    lens = g.cache_lens()
    assert orc.kv_bytes(B, H, d, 2, lens, value_only=lazy) == B * H * d * 2 * (2 * sum(lens[:3]) + lens[3] + lens[4])


def test_lazy_layer_with_uniform_source_attention_averages_its_own_cache():
    """All source keys equal: the source's probabilities are uniform and every visual score ties,
    so the lowest ids survive (Eq. 3 tie rule) and the lazy layer's output is the plain mean of the
    value rows ITS cache must hold: system, surviving visual, text, generated."""
    B, H, d, L, T = 1, 2, 4, 3, 4
    ns, nv, nx = 1, 8, 2
    N0 = ns + nv + nx
    rng = np.random.default_rng(5)
    pre, dec = _mini(6, B, H, N0, d, L, T)
    kc = rng.standard_normal((B, H, 1, d))
    pre[1] = (pre[1][0], np.broadcast_to(kc, (B, H, N0, d)).copy(), pre[1][2])
    for t in range(T):
        dec[t][1] = (dec[t][1][0], kc[:, :, 0].copy(), dec[t][1][2])
    keep = np.array([[8] * 5, [8, 6, 5, 3, 0], [8, 6, 5, 3, 0]])
    g = orc.Generation(L, H, d, ns, nv, nx, keep, lazy={2: 1})
    r = g.prefill(lambda l: pre[l])
    Vp = pre[2][2][0]
    want = np.cumsum(Vp, axis=1) / np.arange(1, N0 + 1)[None, :, None]
    np.testing.assert_allclose(r["out"][2][0], want, atol=1e-12)
    for t in range(1, T + 1):
        s = g.decode_step(lambda l: dec[t - 1][l])
        k = keep[2][t]
        assert s["ids"][2][0].tolist() == list(range(k))
        rows = np.concatenate([Vp[:, :ns], Vp[:, ns:ns + k], Vp[:, ns + nv:]] +
                              [dec[u][2][2][0][:, None] for u in range(t)], axis=1)
        np.testing.assert_allclose(s["out"][2][0], rows.mean(axis=1), atol=1e-12)
        np.testing.assert_allclose(s["mass"][2][0], np.full(k, 1.0 / rows.shape[1]), atol=1e-15)


def test_lazy_configuration_errors():
    keep = np.array([[4, 4], [4, 3], [4, 3], [4, 3]])
    args = (4, 1, 4, 0, 4, 1)
    orc.Generation(*args, keep, lazy={2: 1, 3: 1})
    with pytest.raises(ValueError):
        orc.Generation(*args, keep, lazy={1: 0})             # keeps differ from the source's
    with pytest.raises(ValueError):
        orc.Generation(*args, keep, lazy={3: 1})             # layer 2 in between is not lazy
    with pytest.raises(ValueError):
        orc.Generation(*args, keep, lazy={2: 1, 3: 2})       # the source is itself lazy
    with pytest.raises(ValueError):
        orc.Generation(*args, keep, lazy={1: 1})
