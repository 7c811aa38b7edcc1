"""The documented size limits of the C-ABI calls: the largest supported sizes against the oracle,
one past them refused on the host with nothing enqueued."""
import zlib

import numpy as np
import pytest
import torch

from gpu_util import DEV, TORCH_DTYPE, assert_attention_close, assert_mass_close, rand_values, to_dev, to_np64
from oracle import st3_oracle as orc
from paper_2412_20105_amd import binding as st3

pytestmark = pytest.mark.gpu


def _i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


def _ws(shape, cap, nv, window=1):
    ws = torch.empty((st3.st3_workspace_bytes(shape, cap, nv, window),), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)
    st3.st3_workspace_init(shape, cap, ws)
    return ws


def test_select_topk_at_its_largest_n():
    n, k, B = 16384, 8191, 2
    rng = np.random.default_rng(31)
    s = rng.standard_normal((B, n)).astype(np.float32)
    s[1] = np.round(s[1] * 4) / 4                               # long runs of ties, decided by id
    ids = np.stack([rng.permutation(n) for _ in range(B)]).astype(np.int32)
    d_s, d_i = torch.from_numpy(s).to(DEV), torch.from_numpy(ids).to(DEV)
    mask = torch.zeros((B, n), dtype=torch.uint8, device=DEV)
    idx = torch.zeros((B, k), dtype=torch.int32, device=DEV)
    st3.st3_select_topk(d_s, d_i, None, n, k, mask, idx)
    torch.cuda.synchronize()
    for b in range(B):
        order = np.lexsort((ids[b], -s[b].astype(np.float64)))  # score descending, then id ascending
        want = np.sort(order[:k])
        assert np.array_equal(idx[b].cpu().numpy(), want)
        assert int(mask[b].sum()) == k
    with pytest.raises(st3.St3Error) as e:
        st3.st3_select_topk(torch.zeros((1, n + 1), device=DEV), None, None, n + 1, 1, None,
                            torch.zeros((1, 1), dtype=torch.int32, device=DEV))
    assert e.value.status == st3.ST3_ERR_UNSUPPORTED


@pytest.mark.parametrize("mode", [st3.ST3_STABLE, st3.ST3_HOLE_FILL])
def test_select_compact_layer_at_its_largest_visual_segment(mode):
    nv, keep, ns, tail, B, H, D = 8192, 3000, 2, 40, 2, 1, 64
    cap = ns + nv + tail + 1
    rng = np.random.default_rng(32 + mode)
    K = rand_values(rng, (B, H, cap, D), "f32"); V = rand_values(rng, (B, H, cap, D), "f32")
    score = rng.standard_normal((B, nv)).astype(np.float32)
    score[1] = np.round(score[1] * 8) / 8
    ids = np.stack([rng.permutation(nv) for _ in range(B)]).astype(np.int32)
    shape = st3.make_shape(B, H, D, st3.ST3_F32)
    dK, dV = to_dev(K, "f32"), to_dev(V, "f32")
    d_score, d_ids = torch.from_numpy(score.copy()).to(DEV), torch.from_numpy(ids.copy()).to(DEV)
    vis_len, kv_len = _i32([nv, nv - 7]), _i32([ns + nv + tail, ns + nv - 7 + tail])
    seg = st3.segments(ns, nv, ns + nv + tail, vis_len, kv_len)
    st3.st3_select_compact_layer(shape, st3.kv_layer(dK, dV), seg, d_score, d_ids, keep, mode, _ws(shape, cap, nv))
    torch.cuda.synchronize()
    gK, gV = dK.cpu().numpy(), dV.cpu().numpy()
    for b, nb in enumerate([nv, nv - 7]):
        pos = orc.select_topk(score[b, :nb].astype(np.float64), ids[b, :nb], keep)
        assert vis_len[b].item() == keep and kv_len[b].item() == ns + keep + tail
        got_ids = d_ids[b, :keep].cpu().numpy()
        if mode == st3.ST3_STABLE:
            assert np.array_equal(got_ids, ids[b, pos])
        else:
            assert np.array_equal(np.sort(got_ids), np.sort(ids[b, pos]))
        where = np.empty(nv, np.int64); where[ids[b, :nb]] = np.arange(nb)
        order = where[got_ids]
        assert np.array_equal(gK[b][:, ns:ns + keep], K[b][:, ns + order])
        assert np.array_equal(gV[b][:, ns:ns + keep], V[b][:, ns + order])
        tail_rows = gK[b][0, ns + keep:ns + keep + tail]
        want_tail = K[b][0, ns + nb:ns + nb + tail]
        assert sorted(map(bytes, tail_rows)) == sorted(map(bytes, want_tail))
    seg_big = st3.segments(0, nv + 1, nv + 1, vis_len, kv_len)
    big = torch.zeros((B, H, nv + 2, D), device=DEV)
    with pytest.raises(st3.St3Error) as e:
        st3.st3_select_compact_layer(shape, st3.kv_layer(big, big.clone()), seg_big,
                                     torch.zeros((B, nv + 1), device=DEV),
                                     torch.zeros((B, nv + 1), dtype=torch.int32, device=DEV), 5, mode,
                                     _ws(shape, nv + 2, nv + 1))
    assert e.value.status == st3.ST3_ERR_UNSUPPORTED


def test_decode_attention_over_a_long_cache_cut_into_the_maximum_number_of_chunks():
    B, H, D, ns, nv = 1, 2, 128, 3, 8000
    L = 32768 + 5
    rng = np.random.default_rng(33)
    K = rand_values(rng, (B, H, L, D), "bf16", 1.43); V = rand_values(rng, (B, H, L, D), "bf16", 1.43)
    q = rand_values(rng, (B, H, D), "bf16", 1.43)
    shape = st3.make_shape(B, H, D, st3.ST3_BF16)
    out = torch.zeros((B, H, D), dtype=torch.bfloat16, device=DEV)
    mass = torch.zeros((B, nv), dtype=torch.float32, device=DEV)
    seg = st3.segments(ns, nv, L, _i32([nv]), _i32([L]))
    st3.st3_decode_attention(shape, to_dev(q, "bf16"), st3.kv_layer(to_dev(K, "bf16"), to_dev(V, "bf16")), seg, out, mass,
                             _ws(shape, L, nv))
    torch.cuda.synchronize()
    o, m, _ = orc.decode_attention(q, K, V, ns, nv)
    assert_attention_close(to_np64(out)[0], o[0], "bf16", "long cache")
    assert_mass_close(to_np64(mass)[0], m[0], "long cache")


def test_decode_attention_with_strips_longer_than_the_logit_staging_holds():
    """A workgroup collects the logits it keeps for the mass in LDS, 4096 rows at most, so a strip longer than that is
    cut even where the batch alone fills the chip: 256 strips with 4150 visual keys each, ragged lengths."""
    B, H, D, ns, nv, tail = 8, 32, 64, 4, 4150, 46
    L = ns + nv + tail
    rng = np.random.default_rng(35)
    K = rand_values(rng, (B, H, L, D), "bf16", 1.2); V = rand_values(rng, (B, H, L, D), "bf16", 1.2)
    q = rand_values(rng, (B, H, D), "bf16", 1.2)
    vis = [nv, nv - 1, 4097, 4096, 4095, 2000, 1, 0]
    lens = [ns + v + tail - (b % 3) for b, v in enumerate(vis)]
    shape = st3.make_shape(B, H, D, st3.ST3_BF16)
    out = torch.zeros((B, H, D), dtype=torch.bfloat16, device=DEV)
    mass = torch.full((B, nv), -2.0, dtype=torch.float32, device=DEV)
    seg = st3.segments(ns, nv, L, _i32(vis), _i32(lens))
    st3.st3_decode_attention(shape, to_dev(q, "bf16"), st3.kv_layer(to_dev(K, "bf16"), to_dev(V, "bf16")), seg, out, mass,
                             _ws(shape, L, nv))
    torch.cuda.synchronize()
    for b in range(B):
        o, m, _ = orc.decode_attention(q[b:b + 1], K[b:b + 1, :, :lens[b]], V[b:b + 1, :, :lens[b]], ns, vis[b])
        assert_attention_close(to_np64(out)[b], o[0], "bf16", f"b={b}")
        assert_mass_close(to_np64(mass)[b, :vis[b]], m[0], f"b={b}")


def test_prefill_attention_at_a_long_prompt():
    B, H, D, n, ns, nv, W = 1, 2, 64, 4100, 10, 3000, 2
    rng = np.random.default_rng(34)
    Q, K, V = (rand_values(rng, (B, H, n, D), "bf16", 1.2) for _ in range(3))
    shape = st3.make_shape(B, H, D, st3.ST3_BF16)
    out = torch.zeros((B, H, n, D), dtype=torch.bfloat16, device=DEV)
    mass = torch.zeros((B, nv), dtype=torch.float32, device=DEV)
    st3.st3_prefill_attention(shape, to_dev(Q, "bf16"), to_dev(K, "bf16"), to_dev(V, "bf16"), n, ns, nv, W, out, mass,
                              _ws(shape, n, nv, W))
    torch.cuda.synchronize()
    o, m = orc.prefill_attention(Q, K, V, ns, nv, W)
    assert_attention_close(to_np64(out)[0], o[0], "bf16", "long prompt")
    assert_mass_close(to_np64(mass)[0], m[0], "long prompt")
    with pytest.raises(st3.St3Error) as e:
        st3.st3_prefill_attention(shape, out, out, out, 32769, 0, 0, 1, out, None, _ws(shape, n, nv, W))
    assert e.value.status in (st3.ST3_ERR_UNSUPPORTED, st3.ST3_ERR_INVALID_ARG)


def test_workspace_and_alignment_errors_enqueue_nothing():
    B, H, D, L = 1, 2, 128, 64
    shape = st3.make_shape(B, H, D, st3.ST3_BF16)
    K = torch.zeros((B, H, L, D), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((B, H, D), dtype=torch.bfloat16, device=DEV)
    out = torch.full((B, H, D), 3.0, dtype=torch.bfloat16, device=DEV)
    seg = st3.segments(0, 8, L, _i32([8]), _i32([L]))
    ws = _ws(shape, L, 8)
    with pytest.raises(st3.St3Error) as e:
        st3.st3_decode_attention(shape, q, st3.kv_layer(K, K.clone()), seg, out, None, ws[:64])
    assert e.value.status == st3.ST3_ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(st3.St3Error) as e:                       # a query that is not 16-byte aligned
        qq = torch.zeros((B * H * D + 8,), dtype=torch.bfloat16, device=DEV)[1:1 + B * H * D].view(B, H, D)
        st3.st3_decode_attention(shape, qq, st3.kv_layer(K, K.clone()), seg, out, None, ws)
    assert e.value.status == st3.ST3_ERR_INVALID_ARG
    with pytest.raises(st3.St3Error) as e:                       # lengths bound beyond the cache capacity
        st3.st3_decode_attention(shape, q, st3.kv_layer(K, K.clone()), st3.segments(0, 8, L + 1, _i32([8]), _i32([L])),
                                 out, None, ws)
    assert e.value.status == st3.ST3_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert torch.all(out == 3.0)                                 # nothing ran
