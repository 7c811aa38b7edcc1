"""Pins for the oracle's FP8 E4M3 KV-cache variant (an implementation variant of the cache, not part
of the paper): code values and rounding against a library float8_e4m3fn conversion and closed forms."""
import numpy as np
import pytest
import torch

from oracle import st3_oracle as orc


def test_all_256_codes_decode_like_the_library_type():
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = orc.e4m3_decode(codes)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))
    # closed forms from the format definition
    assert got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6 and got[0x38] == 1.0
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and got[0xFE] == -448.0


@pytest.mark.parametrize("scale", [1.0, 0.019152, 3.0, 2.0 ** -7])
def test_in_range_rounding_matches_the_library_conversion(scale):
    rng = np.random.default_rng(int(scale * 1e6) % 1000)
    x = np.concatenate([rng.standard_normal(20000) * 100 * scale, rng.standard_normal(20000) * scale,
                        rng.standard_normal(5000) * 0.01 * scale]).astype(np.float32)
    t = x / np.float32(scale)                                  # float32 division, as the quantiser defines
    keep = np.abs(t) <= 448.0                                  # beyond that the library type does not saturate
    want = torch.from_numpy(t[keep]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = orc.e4m3_quantize(x[keep], scale)
    assert np.array_equal(got, want)


def test_midpoints_go_to_the_even_code_and_the_ends_saturate():
    table = orc.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    assert np.all(np.diff(table) > 0)
    mids = ((table[:-1] + table[1:]) / 2).astype(np.float32)   # exactly representable in float32
    assert np.array_equal(mids.astype(np.float64), (table[:-1] + table[1:]) / 2)
    got = orc.e4m3_quantize(mids, 1.0)
    want = np.array([c if c % 2 == 0 else c + 1 for c in range(0x7E)], dtype=np.uint8)
    assert np.array_equal(got, want)
    assert np.array_equal(orc.e4m3_quantize(-mids, 1.0), want | 0x80)
    just_above = np.nextafter(mids, np.float32(np.inf))
    assert np.array_equal(orc.e4m3_quantize(just_above, 1.0), np.arange(1, 0x7F, dtype=np.uint8))
    special = np.array([1e9, -np.inf, np.nan, -0.0, 0.0, 2.0 ** -10, 2.0 ** -11, 449.0, 465.0], np.float32)
    assert orc.e4m3_quantize(special, 1.0).tolist() == [0x7E, 0xFE, 0x7F, 0x80, 0x00, 0x00, 0x00, 0x7E, 0x7E]


@pytest.mark.parametrize("scale", [1.0, 0.25, 0.019152, 7.3])
def test_quantising_a_decoded_code_gives_the_code_back(scale):
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    x = (orc.e4m3_decode(codes) * float(np.float32(scale))).astype(np.float32)
    assert np.array_equal(orc.e4m3_quantize(x, scale), codes)
    np.testing.assert_array_equal(orc.e4m3_roundtrip(x, scale), orc.e4m3_decode(codes) * float(np.float32(scale)))


def test_generation_with_an_e4m3_cache():
    """Inputs already on the E4M3 grid make the E4M3 run equal to the plain one; with ordinary inputs the
    prefill outputs do not change (the prompt is attended unquantised), the decode outputs do, and every
    cached value is a code value times its strip's scale."""
    B, H, d, L, T = 2, 2, 8, 2, 3
    ns, nv, nx = 1, 6, 2
    N0 = ns + nv + nx
    rng = np.random.default_rng(12)
    ks = (0.01 + rng.random((B, H)) * 0.02).astype(np.float32)
    vs = (0.01 + rng.random((B, H)) * 0.02).astype(np.float32)
    keep = np.array([[6, 6, 5, 4], [4, 4, 3, 2]])
    pre = [tuple(rng.standard_normal((B, H, N0, d)) for _ in range(3)) for _ in range(L)]
    dec = [[tuple(rng.standard_normal((B, H, d)) for _ in range(3)) for _ in range(L)] for _ in range(T)]
    plain = orc.Generation(L, H, d, ns, nv, nx, keep)
    fp8 = orc.Generation(L, H, d, ns, nv, nx, keep, kv_format="e4m3", k_scale=ks, v_scale=vs)
    rp, rf = plain.prefill(lambda l: pre[l]), fp8.prefill(lambda l: pre[l])
    for l in range(L):
        for b in range(B):
            np.testing.assert_array_equal(rp["out"][l][b], rf["out"][l][b])
            np.testing.assert_array_equal(rp["mass"][l][b], rf["mass"][l][b])
    differs = False
    for t in range(T):
        sp, sf = plain.decode_step(lambda l: dec[t][l]), fp8.decode_step(lambda l: dec[t][l])
        differs |= any(np.abs(sp["out"][l][b] - sf["out"][l][b]).max() > 1e-6 for l in range(L) for b in range(B))
    assert differs
    table = set(orc.e4m3_decode(np.arange(256, dtype=np.uint8))[~np.isnan(orc.e4m3_decode(np.arange(256, dtype=np.uint8)))])
    for l in range(L):
        for b in range(B):
            for h in range(H):
                assert set(np.round(fp8.K[l][b][h].ravel() / float(ks[b, h]), 9)) <= {round(v, 9) for v in table}
                assert set(np.round(fp8.V[l][b][h].ravel() / float(vs[b, h]), 9)) <= {round(v, 9) for v in table}
    # inputs on the grid: nothing changes
    grid = orc.e4m3_decode(np.arange(0x08, 0x60, dtype=np.uint8))
    def on_grid(shape, sc):
        return rng.choice(grid, shape) * rng.choice([-1.0, 1.0], shape) * sc.astype(np.float64)
    pre_g = [(rng.standard_normal((B, H, N0, d)), on_grid((B, H, N0, d), ks[:, :, None, None]),
              on_grid((B, H, N0, d), vs[:, :, None, None])) for _ in range(L)]
    dec_g = [[(rng.standard_normal((B, H, d)), on_grid((B, H, d), ks[:, :, None]), on_grid((B, H, d), vs[:, :, None]))
              for _ in range(L)] for _ in range(T)]
    a = orc.Generation(L, H, d, ns, nv, nx, keep)
    c = orc.Generation(L, H, d, ns, nv, nx, keep, kv_format="e4m3", k_scale=ks, v_scale=vs)
    a.prefill(lambda l: pre_g[l]); c.prefill(lambda l: pre_g[l])
    for t in range(T):
        sa, sc_ = a.decode_step(lambda l: dec_g[t][l]), c.decode_step(lambda l: dec_g[t][l])
        for l in range(L):
            for b in range(B):
                np.testing.assert_allclose(sc_["out"][l][b], sa["out"][l][b], rtol=0, atol=1e-6)
