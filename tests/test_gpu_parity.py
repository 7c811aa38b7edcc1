"""Element-by-element parity of every C-ABI compute call against the CPU oracle."""
import zlib

import numpy as np
import pytest
import torch

from gpu_util import (DEV, TORCH_DTYPE, assert_attention_close, assert_mass_close, rand_values, to_dev, to_np64)
from oracle import st3_oracle as orc
from paper_2412_20105_amd import binding as st3

pytestmark = pytest.mark.gpu

CODE = {"f32": st3.ST3_F32, "bf16": st3.ST3_BF16}


def _ws(shape, capacity, max_vis, window=1):
    n = st3.st3_workspace_bytes(shape, capacity, max_vis, window)
    assert n > 0
    ws = torch.empty((n,), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)                                   # all NaN bit patterns: nothing stale may be read unmasked
    st3.st3_workspace_init(shape, capacity, ws)
    return ws


def _i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


# ---------------------------------------------------------------------------
# decode attention + mass
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,D,B,H,lens,ns,nv", [
    ("f32", 64, 1, 4, [88], 8, 64),
    ("f32", 128, 2, 3, [300, 1], 0, 1),
    ("bf16", 128, 3, 5, [739, 257, 256], 35, 200),     # several splits, ragged batch, chunk edge
    ("bf16", 64, 2, 2, [1000, 31], 3, 20),
    ("bf16", 128, 2, 2, [33, 0], 1, 7),                # an empty sequence
    ("bf16", 128, 1, 40, [1251], 35, 576),             # 13B head count, cache at full length
    ("bf16", 128, 1, 22, [1000], 35, 200),             # 12 chunks wanted, 11 needed once the chunk is rounded to 32 rows
    ("f32", 64, 3, 7, [2000, 1999, 5], 0, 0),          # no visual segment at all
])
def test_decode_attention_matches_oracle(dtype, D, B, H, lens, ns, nv):
    print(f"decode dtype={dtype} D={D} B={B} H={H} lens={lens}", flush=True)
    rng = np.random.default_rng(zlib.crc32(repr((dtype, D, B, H, lens)).encode()))
    cap = max(lens) + 5
    sigma = 1.0 if dtype == "f32" else 1.43
    K = rand_values(rng, (B, H, cap, D), dtype, sigma)
    V = rand_values(rng, (B, H, cap, D), dtype, sigma)
    q = rand_values(rng, (B, H, D), dtype, sigma)
    vis = [max(0, min(nv, L - ns)) for L in lens]
    shape = st3.make_shape(B, H, D, CODE[dtype])
    dK, dV, dq = to_dev(K, dtype), to_dev(V, dtype), to_dev(q, dtype)
    for b in range(B):                                 # rows beyond a sequence hold NaN: they must never count
        dK[b, :, lens[b]:] = float("nan"); dV[b, :, lens[b]:] = float("nan")
    out = torch.zeros((B, H, D), dtype=TORCH_DTYPE[dtype], device=DEV)
    mass = torch.full((B, nv + 3), -7.0, dtype=torch.float32, device=DEV)
    kv_len, vis_len = _i32(lens), _i32(vis)
    seg = st3.segments(ns, nv, max(lens), vis_len, kv_len)
    st3.st3_decode_attention(shape, dq, st3.kv_layer(dK, dV), seg, out, mass, _ws(shape, cap, nv))
    torch.cuda.synchronize()
    got_o, got_m = to_np64(out), to_np64(mass)
    for b in range(B):
        if lens[b] == 0:
            assert np.all(got_o[b] == 0)
            continue
        o, m, _ = orc.decode_attention(q[b:b + 1], K[b:b + 1, :, :lens[b]], V[b:b + 1, :, :lens[b]], ns, vis[b])
        assert_attention_close(got_o[b], o[0], dtype, f"b={b}")
        assert_mass_close(got_m[b, :vis[b]], m[0], f"b={b}")
        assert np.all(got_m[b, vis[b]:] == -7.0)           # untouched beyond vis_len


def test_decode_without_mass_and_custom_scale():
    rng = np.random.default_rng(5)
    B, H, D, L = 1, 2, 64, 70
    K = rand_values(rng, (B, H, L, D), "f32"); V = rand_values(rng, (B, H, L, D), "f32")
    q = rand_values(rng, (B, H, D), "f32")
    shape = st3.make_shape(B, H, D, st3.ST3_F32, 0.05)
    out = torch.zeros((B, H, D), dtype=torch.float32, device=DEV)
    seg = st3.segments(0, 0, L, _i32([0]), _i32([L]))
    st3.st3_decode_attention(shape, to_dev(q, "f32"), st3.kv_layer(to_dev(K, "f32"), to_dev(V, "f32")), seg, out, None,
                             _ws(shape, L, 0))
    o, _, _ = orc.decode_attention(q, K, V, 0, 0, scale=0.05)
    assert_attention_close(to_np64(out), o, "f32")


# ---------------------------------------------------------------------------
# append
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128)])
def test_kv_append(dtype, D):
    rng = np.random.default_rng(6)
    B, H, cap = 3, 4, 20
    K = rand_values(rng, (B, H, cap, D), dtype); V = rand_values(rng, (B, H, cap, D), dtype)
    kn = rand_values(rng, (B, H, D), dtype); vn = rand_values(rng, (B, H, D), dtype)
    lens = [5, 0, 19]
    dK, dV = to_dev(K, dtype), to_dev(V, dtype)
    kv_len = _i32(lens)
    shape = st3.make_shape(B, H, D, CODE[dtype])
    st3.st3_kv_append(shape, st3.kv_layer(dK, dV), st3.segments(0, 0, 19, _i32([0, 0, 0]), kv_len),
                      to_dev(kn, dtype), to_dev(vn, dtype))
    torch.cuda.synchronize()
    wantK, wantV = K.copy(), V.copy()
    for b in range(B):
        wantK[b, :, lens[b]] = kn[b]; wantV[b, :, lens[b]] = vn[b]
    assert np.array_equal(dK.float().cpu().numpy(), wantK) and np.array_equal(dV.float().cpu().numpy(), wantV)
    assert kv_len.cpu().tolist() == [6, 1, 20]


# ---------------------------------------------------------------------------
# top-k selection
# ---------------------------------------------------------------------------
def _check_topk(scores, ids, n_list, n, k):
    B = scores.shape[0]
    d_scores = torch.from_numpy(scores).to(DEV)
    d_ids = None if ids is None else torch.from_numpy(ids.astype(np.int32)).to(DEV)
    mask = torch.full((B, n), 9, dtype=torch.uint8, device=DEV)
    idx = torch.full((B, k + 2), -5, dtype=torch.int32, device=DEV)
    n_dev = None if n_list is None else _i32(n_list)
    st3.st3_select_topk(d_scores, d_ids, n_dev, n, k, mask, idx)
    torch.cuda.synchronize()
    mask, idx = mask.cpu().numpy(), idx.cpu().numpy()
    for b in range(B):
        nb = n if n_list is None else n_list[b]
        kb = min(k, nb)
        tie = np.arange(nb) if ids is None else ids[b, :nb]
        want = orc.select_topk(scores[b, :nb].astype(np.float64), tie, kb)
        assert idx[b, :kb].tolist() == want.tolist(), (b, nb, kb)
        assert np.all(idx[b, kb:k] == -1) and np.all(idx[b, k:] == -5)
        wm = np.zeros(n, np.uint8); wm[want] = 1
        assert np.array_equal(mask[b], wm)


def test_select_topk_random_ties_and_ragged():
    rng = np.random.default_rng(7)
    for n, k in [(1, 1), (5, 0), (64, 32), (576, 288), (577, 561), (2880, 144), (1000, 1000), (8192, 100),
                 (9000, 4500)]:
        print(f"topk n={n} k={k}", flush=True)
        B = 3
        s = rng.standard_normal((B, n)).astype(np.float32)
        s[1] = np.round(s[1] * 2) / 2                     # heavy ties
        s[2, : n // 2] = 0.25                             # half the row equal
        ids = np.stack([rng.permutation(n) for _ in range(B)])
        _check_topk(s, ids, None, n, k)
        _check_topk(s, None, None, n, k)
    s = rng.standard_normal((4, 300)).astype(np.float32)
    ids = np.stack([rng.permutation(300) + 1000 for _ in range(4)])
    _check_topk(s, ids, [300, 17, 0, 128], 300, 100)


def test_select_topk_special_values():
    n = 200
    s = np.zeros((3, n), np.float32)
    s[0, ::2] = -0.0                                      # -0.0 ties with +0.0
    s[1] = np.linspace(-1e-30, 1e-30, n, dtype=np.float32)
    s[1, 5] = np.inf; s[1, 6] = -np.inf
    s[2] = -np.abs(np.random.default_rng(8).standard_normal(n)).astype(np.float32)
    ids = np.stack([np.arange(n)[::-1].copy() for _ in range(3)])
    _check_topk(s, ids, None, n, 37)
    _check_topk(s, ids, None, n, 199)


def test_select_topk_exhaustive_tiny():
    import itertools
    vals = [0.0, 0.5, 1.0]
    rows, idsl = [], []
    n = 5
    for sc in itertools.product(vals, repeat=n):
        rows.append(sc); idsl.append(list(range(n))[::-1])
    s = np.array(rows, np.float32); ids = np.array(idsl)
    for k in range(n + 1):
        _check_topk(s, ids, None, n, k)


# ---------------------------------------------------------------------------
# stable row compaction
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("row_bytes,inner,stride_pad", [(256, 3, 0), (4, 1, 0), (10240, 1, 0), (24, 2, 8), (512, 2, 16)])
def test_compact_rows_stable(row_bytes, inner, stride_pad):
    rng = np.random.default_rng(9)
    B, n, tail, lead = 2, 77, 9, 3
    rows_total = lead + n + tail
    stride_row = row_bytes + stride_pad
    buf = rng.integers(0, 255, (B, inner, rows_total, stride_row), dtype=np.uint8)
    d = torch.from_numpy(buf.copy()).to(DEV)
    for pattern in ("random", "every_other", "last_k", "first_k", "none", "all"):
        src = buf.copy()
        d.copy_(torch.from_numpy(src))
        keeps = []
        for b in range(B):
            if pattern == "random":
                kp = np.sort(rng.choice(n, 40, replace=False))
            elif pattern == "every_other":
                kp = np.arange(0, n, 2)[:39]
            elif pattern == "last_k":
                kp = np.arange(n - 40, n)
            elif pattern == "first_k":
                kp = np.arange(40)
            elif pattern == "none":
                kp = np.arange(0)
            else:
                kp = np.arange(n)
            keeps.append(kp)
        k = max(len(x) for x in keeps)
        idx = np.full((B, k + 1), -1, np.int32)
        for b in range(B):
            idx[b, :len(keeps[b])] = keeps[b]
        d_idx = torch.from_numpy(idx).to(DEV)
        base = d.data_ptr() + lead * stride_row
        st3.st3_compact_rows(base, B, inner, inner * rows_total * stride_row, rows_total * stride_row, stride_row,
                             row_bytes, d_idx, k, n, tail)
        torch.cuda.synchronize()
        got = d.cpu().numpy()
        for b in range(B):
            kb = len(keeps[b])
            for i in range(inner):
                want = src[b, i].copy()
                seg = src[b, i, lead:lead + n + tail]
                new = np.concatenate([seg[keeps[b]], seg[n:n + tail]])
                want[lead:lead + kb + tail, :row_bytes] = new[:, :row_bytes]
                # rows past the compacted region and the padding bytes keep whatever they held
                assert np.array_equal(got[b, i, :lead + kb + tail, :row_bytes], want[:lead + kb + tail, :row_bytes]), \
                    (pattern, b, i)
                assert np.array_equal(got[b, i, :, row_bytes:], src[b, i, :, row_bytes:])
                assert np.array_equal(got[b, i, :lead], src[b, i, :lead])


def test_compact_rows_takes_the_leading_run_of_valid_indices():
    """An index list is its valid entries followed by padding: whatever follows the first entry
    outside [0, n) is ignored, and the tail lands right behind the leading run."""
    rng = np.random.default_rng(10)
    n, tail, row_bytes = 12, 3, 32
    lists = [[3, -1, 5, 7], [1, 4, 12, 6], [0, 2, 9, 11], [-1, 1, 2, 3]]      # valid prefixes of 1, 2, 4, 0 entries
    B = len(lists)
    buf = rng.integers(0, 255, (B, 1, n + tail, row_bytes), dtype=np.uint8)
    d = torch.from_numpy(buf.copy()).to(DEV)
    d_idx = torch.tensor(lists, dtype=torch.int32, device=DEV)
    st3.st3_compact_rows(d.data_ptr(), B, 1, (n + tail) * row_bytes, 0, row_bytes, row_bytes, d_idx, 4, n, tail)
    torch.cuda.synchronize()
    got = d.cpu().numpy()
    for b, lst in enumerate(lists):
        run = 0
        while run < len(lst) and 0 <= lst[run] < n:
            run += 1
        want = np.concatenate([buf[b, 0, lst[:run]], buf[b, 0, n:]])
        assert np.array_equal(got[b, 0, :run + tail], want), (b, lst)


# ---------------------------------------------------------------------------
# select-and-compact of a layer's cache
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("B,inner,width,dtype,head,n,k,tail,n_pairs", [
    (3, 5, 128, torch.bfloat16, 35, 200, 77, 40, 3),        # Q, K, V rows of a layer in one launch
    (2, 1, 5120, torch.bfloat16, 8, 64, 33, 16, 1),         # hidden rows at full width (10 KB)
    (2, 3, 64, torch.float32, 0, 50, 50, 0, 2),             # identity list = strided copy, no head, no tail
    (1, 2, 8, torch.bfloat16, 4, 30, 0, 3, 4),              # nothing kept; 16-byte rows; four tensors
    (2, 2, 128, torch.bfloat16, 3, 2880, 1500, 256, 2),     # high-resolution segment
])
def test_gather_rows(B, inner, width, dtype, head, n, k, tail, n_pairs):
    """Alg. 1/3: X = [S, V[T], I] rebuilt out of place for several tensors with one index list."""
    print(f"gather B={B} inner={inner} width={width} n={n} k={k} pairs={n_pairs}", flush=True)
    g = torch.Generator(device="cpu"); g.manual_seed(n * 7 + k)
    rows_src, rows_dst = head + n + tail, head + k + tail
    idx = torch.stack([torch.sort(torch.randperm(n, generator=g)[:k]).values for _ in range(B)]).to(torch.int32)
    if k == n:
        idx_dev = None
    else:
        idx_dev = torch.full((B, k + 5), -3, dtype=torch.int32)
        idx_dev[:, :k] = idx
        idx_dev = idx_dev.to(DEV)[:, :max(k, 1)] if k > 0 else idx_dev.to(DEV)
    pairs, refs = [], []
    for p in range(n_pairs):
        src = torch.randn((B, inner, rows_src + p, width), generator=g).to(dtype)      # own strides per tensor
        dst = torch.full((B, inner, rows_dst + 2 * p + 1, width), 9.0, dtype=dtype)
        ref = dst.clone()
        for b in range(B):
            take = torch.cat([torch.arange(head), head + idx[b].long(), head + n + torch.arange(tail)])
            ref[b, :, :rows_dst] = src[b][:, take]
        d_src, d_dst = src.to(DEV), dst.to(DEV)
        pairs.append((d_src, d_dst)); refs.append(ref)
    st3.st3_gather_rows(pairs, head, idx_dev, k, n, tail)
    torch.cuda.synchronize()
    for (d_src, d_dst), ref in zip(pairs, refs):
        assert torch.equal(d_dst.cpu().view(torch.uint8), ref.view(torch.uint8))      # bit exact, rows beyond untouched


def test_gather_rows_argument_errors():
    a = torch.zeros((1, 1, 8, 8), dtype=torch.bfloat16, device=DEV)
    b = torch.zeros((1, 1, 8, 8), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(st3.St3Error):
        st3.st3_gather_rows([(a, a)], 0, None, 8, 8, 0)                      # destination overlaps source
    with pytest.raises(st3.St3Error):
        st3.st3_gather_rows([(a, b)], 0, None, 4, 8, 0)                      # no list, but k != n
    with pytest.raises(st3.St3Error):
        st3.st3_gather_rows([(a, b)] * 5, 0, None, 8, 8, 0)                  # too many tensors
    with pytest.raises(st3.St3Error):
        st3.st3_gather_rows([(a[..., :4], b[..., :4])], 0, None, 8, 8, 0)    # 8-byte rows


@pytest.mark.parametrize("mode", [st3.ST3_STABLE, st3.ST3_HOLE_FILL])
@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_select_compact_layer(mode, dtype, D):
    rng = np.random.default_rng(10 + mode)
    B, H, ns = 4, 3, 5
    cap, cap_v = 400, 300
    vis = [300, 120, 37, 10]
    tails = [60, 0, 2, 33]                     # rows behind the visual segment (text + generated)
    lens = [ns + v + t for v, t in zip(vis, tails)]
    shape = st3.make_shape(B, H, D, CODE[dtype])
    for keep_count in (300, 150, 36, 10, 3, 0):
        print(f"select_compact mode={mode} dtype={dtype} keep={keep_count}", flush=True)
        K = rand_values(rng, (B, H, cap, D), dtype); V = rand_values(rng, (B, H, cap, D), dtype)
        score = rng.standard_normal((B, cap_v)).astype(np.float32)
        score[1] = np.round(score[1] * 3) / 3              # ties decided by id
        ids = np.stack([rng.permutation(1000)[:cap_v] for _ in range(B)]).astype(np.int32)
        dK, dV = to_dev(K, dtype), to_dev(V, dtype)
        d_score = torch.from_numpy(score.copy()).to(DEV); d_ids = torch.from_numpy(ids.copy()).to(DEV)
        vis_len, kv_len = _i32(vis), _i32(lens)
        seg = st3.segments(ns, max(vis), max(lens), vis_len, kv_len)
        st3.st3_select_compact_layer(shape, st3.kv_layer(dK, dV), seg, d_score, d_ids, keep_count, mode,
                                     _ws(shape, cap, max(vis)))
        torch.cuda.synchronize()
        gK, gV = dK.float().cpu().numpy(), dV.float().cpu().numpy()
        g_score, g_ids = d_score.cpu().numpy(), d_ids.cpu().numpy()
        g_vis, g_len = vis_len.cpu().tolist(), kv_len.cpu().tolist()
        for b in range(B):
            nb = vis[b]; kb = min(keep_count, nb)
            pos = orc.select_topk(score[b, :nb].astype(np.float64), ids[b, :nb], kb)
            assert g_vis[b] == kb and g_len[b] == lens[b] - (nb - kb), (b, g_vis[b], g_len[b])
            # system rows untouched
            assert np.array_equal(gK[b][:, :ns], K[b][:, :ns]) and np.array_equal(gV[b][:, :ns], V[b][:, :ns])
            tail_src = np.arange(ns + nb, lens[b])
            if mode == st3.ST3_STABLE or kb == nb:
                order = pos
                tail_order = tail_src
            else:
                # any order is valid: recover it from the id column, then check it is a permutation
                got_ids = g_ids[b, :kb]
                assert sorted(got_ids.tolist()) == sorted(ids[b, pos].tolist()), b
                where = {int(t): p for p, t in enumerate(ids[b, :nb])}
                order = np.array([where[int(t)] for t in got_ids], dtype=np.int64)
                # rows behind the segment: a permutation of the old tail, matched by content
                tail_order = None
            assert np.array_equal(g_ids[b, :kb], ids[b, order])
            assert np.array_equal(g_score[b, :kb], score[b, order])
            assert np.array_equal(gK[b][:, ns:ns + kb], K[b][:, ns + order])
            assert np.array_equal(gV[b][:, ns:ns + kb], V[b][:, ns + order])
            got_tail_K = gK[b][:, ns + kb:g_len[b]]; got_tail_V = gV[b][:, ns + kb:g_len[b]]
            if tail_order is not None:
                assert np.array_equal(got_tail_K, K[b][:, tail_order]) and np.array_equal(got_tail_V, V[b][:, tail_order])
            else:
                # match each surviving tail row to its source by head-0 K content; K and V must move together
                key = {K[b, 0, r].tobytes(): int(r) for r in tail_src}
                srcs = [key[got_tail_K[0, j].tobytes()] for j in range(got_tail_K.shape[1])]
                assert sorted(srcs) == tail_src.tolist()
                assert np.array_equal(got_tail_K, K[b][:, srcs]) and np.array_equal(got_tail_V, V[b][:, srcs])
                moved = sum(1 for j, r in enumerate(srcs) if r != ns + kb + j)
                assert moved <= nb - kb                    # at most one move per evicted row


# ---------------------------------------------------------------------------
# QK heredity at decode (Eq. 6, Alg. 2): a lazy layer applies its source's probabilities to its own V
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,D,B,H,lens,ns,nv,cap_extra", [
    ("bf16", 128, 3, 5, [739, 257, 256], 35, 200, 0),      # split strips, ragged batch
    ("bf16", 128, 2, 2, [33, 0], 1, 7, 9),                 # an empty sequence; caches of different capacity
    ("f32", 64, 2, 3, [300, 1], 0, 1, 0),
    ("bf16", 128, 26, 40, [200] * 25 + [77], 35, 100, 3),  # enough strips that none is split
])
def test_decode_attention_inherit(dtype, D, B, H, lens, ns, nv, cap_extra):
    print(f"inherit dtype={dtype} D={D} B={B} H={H} lens={lens[:4]}", flush=True)
    rng = np.random.default_rng(zlib.crc32(repr(("inh", dtype, D, B, H, lens)).encode()))
    cap_s = max(lens) + 5
    cap_l = cap_s + cap_extra
    sigma = 1.0 if dtype == "f32" else 1.43
    K = rand_values(rng, (B, H, cap_s, D), dtype, sigma)
    Vs = rand_values(rng, (B, H, cap_s, D), dtype, sigma)
    Vl = rand_values(rng, (B, H, cap_l, D), dtype, sigma)       # the lazy layer's own values
    q = rand_values(rng, (B, H, D), dtype, sigma)
    vn = rand_values(rng, (B, H, D), dtype, sigma)
    vis = [max(0, min(nv, L - ns)) for L in lens]
    shape = st3.make_shape(B, H, D, CODE[dtype])
    dK, dVs, dVl, dq = to_dev(K, dtype), to_dev(Vs, dtype), to_dev(Vl, dtype), to_dev(q, dtype)
    out_s = torch.zeros((B, H, D), dtype=TORCH_DTYPE[dtype], device=DEV)
    out_l = torch.full((B, H, D), 5.0, dtype=TORCH_DTYPE[dtype], device=DEV)
    ws_s, ws_l = _ws(shape, cap_s, nv), _ws(shape, cap_l, nv)
    # the lazy layer appends first (V only), the source's cache already holds its rows
    lens_before = [max(L - 1, 0) for L in lens]
    kv_len_l, vis_len = _i32(lens_before), _i32(vis)
    lazy_kv = st3.kv_layer(None, dVl)
    st3.st3_kv_append(shape, lazy_kv, st3.segments(ns, nv, max(lens_before), vis_len, kv_len_l), None, to_dev(vn, dtype))
    torch.cuda.synchronize()
    got_len = kv_len_l.cpu().tolist()
    Vl_ref = Vl.copy()
    for b in range(B):
        assert got_len[b] == lens_before[b] + 1
        Vl_ref[b, :, lens_before[b]] = vn[b]
    assert np.array_equal(dVl.float().cpu().numpy(), Vl_ref.astype(np.float32))
    lens_l = got_len                                         # = lens, except an empty sequence now holds one row
    for b in range(B):                                       # rows beyond a sequence hold NaN: they must never count
        dVl[b, :, lens_l[b]:] = float("nan"); dK[b, :, lens_l[b]:] = float("nan"); dVs[b, :, lens_l[b]:] = float("nan")
    kv_len_s = _i32(lens_l)
    # source layer attends (no mass asked for: the probabilities are kept all the same) ...
    st3.st3_decode_attention(shape, dq, st3.kv_layer(dK, dVs), st3.segments(ns, nv, max(lens_l), vis_len, kv_len_s),
                             out_s, None, ws_s)
    # ... and the lazy layer inherits them
    st3.st3_decode_attention_inherit(shape, lazy_kv, st3.segments(ns, nv, max(lens_l), vis_len, kv_len_l), ws_s, cap_s,
                                     out_l, ws_l)
    torch.cuda.synchronize()
    got = to_np64(out_l)
    for b in range(B):
        n = lens_l[b]
        o, _, p = orc.decode_attention(q[b:b + 1], K[b:b + 1, :, :n], Vl_ref[b:b + 1, :, :n], ns, min(vis[b], n))
        assert_attention_close(got[b], o[0], dtype, f"b={b}")
        np.testing.assert_allclose(o[0], np.einsum("hj,hjd->hd", p[0], Vl_ref[b, :, :n].astype(np.float64)), atol=1e-12)


# ---------------------------------------------------------------------------
# FP8 E4M3 KV cache (implementation variant of the cache, not from the paper)
# ---------------------------------------------------------------------------
def _e4m3_adversarial(rng, shape, scale):
    """bf16-exact inputs that land on E4M3 values, on the midpoints between them (ties), just beside
    the midpoints, in the subnormal range, beyond +-448, plus ordinary random values."""
    table = orc.e4m3_decode(np.arange(0x7F, dtype=np.uint8))
    mids = (table[:-1] + table[1:]) / 2                       # 4 significant bits: exact in bf16
    pool = np.concatenate([table, mids, mids * (1 + 2.0 ** -7), mids * (1 - 2.0 ** -7), [0.0, 500.0, 1e6, 2.0 ** -10,
                           2.0 ** -11, 3 * 2.0 ** -11]])
    x = rng.choice(pool, shape) * rng.choice([-1.0, 1.0], shape) * scale
    r = rng.random(shape) < 0.5
    x = np.where(r, rng.standard_normal(shape) * 100 * scale, x)
    return to_np64(torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16)).astype(np.float32)   # round to bf16 once


@pytest.mark.parametrize("D", [128, 64])
def test_quantize_rows_and_append_give_the_oracles_codes(D):
    rng = np.random.default_rng(50 + D)
    B, H, n, cap = 2, 3, 70, 75
    ks = np.array([[1.0, 0.25, 0.0191], [3.0, 0.013, 1.0]], np.float32)
    vs = np.array([[0.5, 1.0, 0.02], [0.0107, 2.0, 0.3]], np.float32)
    K = _e4m3_adversarial(rng, (B, H, n, D), ks[:, :, None, None].astype(np.float64))
    V = _e4m3_adversarial(rng, (B, H, n, D), vs[:, :, None, None].astype(np.float64))
    shape = st3.make_shape(B, H, D, st3.ST3_BF16)
    dKc = torch.full((B, H, cap, D), 0x55, dtype=torch.uint8, device=DEV); dVc = dKc.clone()
    kv = st3.kv_layer(dKc, dVc, torch.from_numpy(ks).to(DEV), torch.from_numpy(vs).to(DEV))
    st3.st3_quantize_rows(shape, to_dev(K, "bf16"), kv, 0, n)
    st3.st3_quantize_rows(shape, to_dev(V, "bf16"), kv, 1, n)
    # one more row through the append call
    kn = _e4m3_adversarial(rng, (B, H, D), ks[:, :, None].astype(np.float64))
    vn = _e4m3_adversarial(rng, (B, H, D), vs[:, :, None].astype(np.float64))
    kv_len = _i32([n, n - 3])
    st3.st3_kv_append(shape, kv, st3.segments(0, 0, n, _i32([0, 0]), kv_len), to_dev(kn, "bf16"), to_dev(vn, "bf16"))
    torch.cuda.synchronize()
    want_K = orc.e4m3_quantize(K, ks[:, :, None, None]); want_V = orc.e4m3_quantize(V, vs[:, :, None, None])
    got_K, got_V = dKc.cpu().numpy(), dVc.cpu().numpy()
    for b, row in enumerate([n, n - 3]):               # the appended row lands at the old kv_len[b]
        wk = np.concatenate([want_K[b], np.full((H, cap - n, D), 0x55, np.uint8)], axis=1)
        wv = np.concatenate([want_V[b], np.full((H, cap - n, D), 0x55, np.uint8)], axis=1)
        wk[:, row] = orc.e4m3_quantize(kn[b], ks[b][:, None])
        wv[:, row] = orc.e4m3_quantize(vn[b], vs[b][:, None])
        assert np.array_equal(got_K[b], wk), b
        assert np.array_equal(got_V[b], wv), b
    assert kv_len.cpu().tolist() == [n + 1, n - 2]


@pytest.mark.parametrize("D,B,H,lens,ns,nv", [
    (128, 3, 5, [739, 257, 256], 35, 200),
    (64, 2, 3, [1000, 31], 3, 20),
    (128, 26, 40, [200] * 25 + [77], 35, 100),
])
@pytest.mark.parametrize("tile", [0, 1, 3, 4])            # 0: the launcher's own choice; else that build of the attend kernel
def test_decode_attention_and_heredity_over_an_e4m3_cache(D, B, H, lens, ns, nv, tile):
    print(f"e4m3 decode D={D} B={B} H={H} lens={lens[:4]} tile={tile}", flush=True)
    st3.st3_debug_set_attend_tile(tile)
    try:
        _e4m3_decode_case(D, B, H, lens, ns, nv)
    finally:
        st3.st3_debug_set_attend_tile(0)


def _e4m3_decode_case(D, B, H, lens, ns, nv):
    rng = np.random.default_rng(zlib.crc32(repr(("e4m3", D, B, H, lens)).encode()))
    cap = max(lens) + 5
    def codes(shape):
        c = rng.integers(0, 256, shape, dtype=np.uint8)
        return np.where(c & 0x7F == 0x7F, np.uint8(0x30), c).astype(np.uint8)      # no NaN codes in valid rows
    Kc, Vc, Vl = codes((B, H, cap, D)), codes((B, H, cap, D)), codes((B, H, cap, D))
    # scales that put the logits in a sane range: code values are up to 448
    ks = (0.002 + rng.random((B, H)) * 0.004).astype(np.float32)
    vs = (0.005 + rng.random((B, H)) * 0.01).astype(np.float32)
    q = rand_values(rng, (B, H, D), "bf16", 1.43)
    vis = [max(0, min(nv, L - ns)) for L in lens]
    shape = st3.make_shape(B, H, D, st3.ST3_BF16)
    dK, dV, dVl = (torch.from_numpy(x.copy()).to(DEV) for x in (Kc, Vc, Vl))
    for b in range(B):                                 # NaN codes beyond every sequence
        dK[b, :, lens[b]:] = 0x7F; dV[b, :, lens[b]:] = 0xFF; dVl[b, :, lens[b]:] = 0x7F
    d_ks, d_vs = torch.from_numpy(ks).to(DEV), torch.from_numpy(vs).to(DEV)
    out = torch.zeros((B, H, D), dtype=torch.bfloat16, device=DEV)
    out_l = torch.zeros((B, H, D), dtype=torch.bfloat16, device=DEV)
    mass = torch.full((B, nv + 3), -7.0, dtype=torch.float32, device=DEV)
    kv_len, vis_len = _i32(lens), _i32(vis)
    seg = st3.segments(ns, nv, max(lens), vis_len, kv_len)
    ws_s, ws_l = _ws(shape, cap, nv), _ws(shape, cap, nv)
    st3.st3_decode_attention(shape, to_dev(q, "bf16"), st3.kv_layer(dK, dV, d_ks, d_vs), seg, out, mass, ws_s)
    st3.st3_decode_attention_inherit(shape, st3.kv_layer(None, dVl, None, d_vs), seg, ws_s, cap, out_l, ws_l)
    torch.cuda.synchronize()
    got_o, got_l, got_m = to_np64(out), to_np64(out_l), to_np64(mass)
    for b in range(B):
        n = lens[b]
        Kd = orc.e4m3_decode(Kc[b:b + 1, :, :n]) * ks[b].astype(np.float64)[None, :, None, None]
        Vd = orc.e4m3_decode(Vc[b:b + 1, :, :n]) * vs[b].astype(np.float64)[None, :, None, None]
        Vld = orc.e4m3_decode(Vl[b:b + 1, :, :n]) * vs[b].astype(np.float64)[None, :, None, None]
        o, m, _ = orc.decode_attention(q[b:b + 1], Kd, Vd, ns, vis[b])
        ol, _, _ = orc.decode_attention(q[b:b + 1], Kd, Vld, ns, vis[b])
        assert_attention_close(got_o[b], o[0], "bf16", f"b={b}")
        assert_attention_close(got_l[b], ol[0], "bf16", f"lazy b={b}")
        assert_mass_close(got_m[b, :vis[b]], m[0], f"b={b}")


# ---------------------------------------------------------------------------
# fused layer step: append + attention + mass, then the eviction for the next step (Alg. 3)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("mode", [st3.ST3_STABLE, st3.ST3_HOLE_FILL])
@pytest.mark.parametrize("dtype,D,H,lens,keep_after", [
    ("bf16", 128, 4, [192, 191, 193, 64], 20),     # the appended row opens a chunk of its own / closes one
    ("bf16", 128, 4, [256, 255, 128, 97], -1),     # no eviction: lengths only grow
    ("f32", 64, 3, [300, 33, 128, 257], 0),        # everything visual goes
    ("bf16", 128, 2, [420, 419, 300, 389], 7),     # more than the in-kernel row-move limit is evicted
])
def test_decode_layer_step(mode, dtype, D, H, lens, keep_after):
    print(f"layer_step mode={mode} dtype={dtype} lens={lens} keep_after={keep_after}", flush=True)
    rng = np.random.default_rng(zlib.crc32(repr((dtype, D, H, lens, keep_after)).encode()))
    B, ns = len(lens), 6
    cap = max(lens) + 3
    vis = [min(L - ns - 2, 100 + 40 * b) for b, L in enumerate(lens)]
    nv = max(vis)
    sigma = 1.0 if dtype == "f32" else 1.43
    K = rand_values(rng, (B, H, cap, D), dtype, sigma); V = rand_values(rng, (B, H, cap, D), dtype, sigma)
    q, kn, vn = (rand_values(rng, (B, H, D), dtype, sigma) for _ in range(3))
    score = rng.standard_normal((B, nv)).astype(np.float32)
    ids = np.stack([rng.permutation(2000)[:nv] for _ in range(B)]).astype(np.int32)
    shape = st3.make_shape(B, H, D, CODE[dtype])
    dK, dV = to_dev(K, dtype), to_dev(V, dtype)
    for b in range(B):                                 # rows beyond a sequence hold NaN: they must never count
        dK[b, :, lens[b]:] = float("nan"); dV[b, :, lens[b]:] = float("nan")
    d_score, d_ids = torch.from_numpy(score.copy()).to(DEV), torch.from_numpy(ids.copy()).to(DEV)
    out = torch.zeros((B, H, D), dtype=TORCH_DTYPE[dtype], device=DEV)
    mass = torch.full((B, nv + 2), -7.0, dtype=torch.float32, device=DEV)
    vis_len, kv_len = _i32(vis), _i32(lens)
    seg = st3.segments(ns, nv, max(lens), vis_len, kv_len)
    st3.st3_decode_layer_step(shape, st3.kv_layer(dK, dV), seg, d_score, d_ids, keep_after, mode, to_dev(q, dtype),
                              to_dev(kn, dtype), to_dev(vn, dtype), out, mass, _ws(shape, cap, nv))
    torch.cuda.synchronize()
    got_o, got_m = to_np64(out), to_np64(mass)
    gK, gV = dK.float().cpu().numpy(), dV.float().cpu().numpy()
    g_ids, g_score = d_ids.cpu().numpy(), d_score.cpu().numpy()
    for b in range(B):
        L, nb = lens[b], vis[b]
        Kb = np.concatenate([K[b, :, :L], kn[b][:, None]], axis=1)      # what the attention must see
        Vb = np.concatenate([V[b, :, :L], vn[b][:, None]], axis=1)
        o, m, _ = orc.decode_attention(q[b:b + 1], Kb[None], Vb[None], ns, nb)
        assert_attention_close(got_o[b], o[0], dtype, f"b={b}")
        assert_mass_close(got_m[b, :nb], m[0], f"b={b}")
        assert np.all(got_m[b, nb:] == -7.0)
        kb = nb if keep_after < 0 else min(keep_after, nb)
        assert vis_len[b].item() == kb and kv_len[b].item() == L + 1 - (nb - kb), b
        pos = orc.select_topk(score[b, :nb].astype(np.float64), ids[b, :nb], kb)
        got_ids = g_ids[b, :kb]
        if mode == st3.ST3_STABLE or kb == nb:
            assert np.array_equal(got_ids, ids[b, pos])
        else:
            assert sorted(got_ids.tolist()) == sorted(ids[b, pos].tolist())
        where = {int(t): p for p, t in enumerate(ids[b, :nb])}
        order = np.array([where[int(t)] for t in got_ids], dtype=np.int64)
        assert np.array_equal(g_score[b, :kb], score[b, order])
        assert np.array_equal(gK[b][:, :ns], K[b][:, :ns])
        assert np.array_equal(gK[b][:, ns:ns + kb], Kb[:, ns + order]) and np.array_equal(gV[b][:, ns:ns + kb], Vb[:, ns + order])
        # rows behind the segment (text, generated, the new token): the same rows, K and V moved together
        tail_src = np.arange(ns + nb, L + 1)
        got_tail_K, got_tail_V = gK[b][:, ns + kb:kv_len[b].item()], gV[b][:, ns + kb:kv_len[b].item()]
        key = {Kb[0, r].tobytes(): int(r) for r in tail_src}
        srcs = [key[got_tail_K[0, j].tobytes()] for j in range(got_tail_K.shape[1])]
        assert sorted(srcs) == tail_src.tolist()
        if mode == st3.ST3_STABLE:
            assert srcs == tail_src.tolist()
        assert np.array_equal(got_tail_K, Kb[:, srcs]) and np.array_equal(got_tail_V, Vb[:, srcs])


@pytest.mark.parametrize("mode,hint", [(st3.ST3_STABLE, "none"), (st3.ST3_HOLE_FILL, "none"), (st3.ST3_STABLE, "first"),
                                       (st3.ST3_HOLE_FILL, "last"), (st3.ST3_STABLE, "far")])
@pytest.mark.parametrize("dtype,D,H,tails,keep_after,B_extra", [
    ("bf16", 128, 4, [60, 1, 129, 0], 20, 0),      # a sequence without any tail row yet: the new row is its first
    ("bf16", 128, 40, [128, 300, 7, 64], 90, 24),  # enough strips that none is split; rows past the segment in the first tiles
    ("f32", 64, 3, [40, 41, 42, 43], 0, 0),        # the whole visual segment goes, the tail stays where it is
    ("bf16", 128, 2, [33, 200, 90, 5], 7, 0),      # more than the in-kernel row-move limit is evicted
])
def test_decode_layer_step_with_a_fixed_tail(mode, hint, dtype, D, H, tails, keep_after, B_extra):
    """The rows behind the visual segment start at tail_start[b] and never move; between the segment
    and them the cache holds NaN.  Attention must see system + visual + tail + the new token; the
    eviction may only touch the visual segment.  The host's guess at the layout (right for one
    sequence and wrong for the others, or wrong for all) must not show in any result."""
    print(f"fixed tail mode={mode} hint={hint} dtype={dtype} H={H} tails={tails} keep_after={keep_after}", flush=True)
    tails = tails + [50] * B_extra
    rng = np.random.default_rng(zlib.crc32(repr(("ft", dtype, D, H, tails, keep_after)).encode()))
    B, ns = len(tails), 6
    vis = [100 + (37 * b) % 120 for b in range(B)]
    nv = max(vis)
    ts = [ns + v + (13 * b) % 70 for b, v in enumerate(vis)]          # some sequences have no gap yet (b = 0)
    lens = [t + r for t, r in zip(ts, tails)]                         # physical end of each tail
    cap = max(lens) + 3
    sigma = 1.0 if dtype == "f32" else 1.43
    K = rand_values(rng, (B, H, cap, D), dtype, sigma); V = rand_values(rng, (B, H, cap, D), dtype, sigma)
    q, kn, vn = (rand_values(rng, (B, H, D), dtype, sigma) for _ in range(3))
    score = rng.standard_normal((B, nv)).astype(np.float32)
    ids = np.stack([rng.permutation(2000)[:nv] for _ in range(B)]).astype(np.int32)
    shape = st3.make_shape(B, H, D, CODE[dtype])
    dK, dV = to_dev(K, dtype), to_dev(V, dtype)
    for b in range(B):                                 # dead rows and everything past the end: NaN
        for t in (dK, dV):
            t[b, :, ns + vis[b]:ts[b]] = float("nan"); t[b, :, lens[b]:] = float("nan")
    K0, V0 = dK.float().cpu().numpy(), dV.float().cpu().numpy()
    d_score, d_ids = torch.from_numpy(score.copy()).to(DEV), torch.from_numpy(ids.copy()).to(DEV)
    out = torch.zeros((B, H, D), dtype=TORCH_DTYPE[dtype], device=DEV)
    mass = torch.full((B, nv + 2), -7.0, dtype=torch.float32, device=DEV)
    vis_len, kv_len, tail_start = _i32(vis), _i32(lens), _i32(ts)
    guess = {"none": (0, 0), "first": (vis[0], ts[0]), "last": (vis[-1], ts[-1]), "far": (3, 2 ** 31 - 1)}[hint]
    seg = st3.segments(ns, nv, max(lens), vis_len, kv_len, tail_start, *guess)
    st3.st3_decode_layer_step(shape, st3.kv_layer(dK, dV), seg, d_score, d_ids, keep_after, mode, to_dev(q, dtype),
                              to_dev(kn, dtype), to_dev(vn, dtype), out, mass, _ws(shape, cap, nv))
    torch.cuda.synchronize()
    got_o, got_m = to_np64(out), to_np64(mass)
    gK, gV = dK.float().cpu().numpy(), dV.float().cpu().numpy()
    g_ids, g_score = d_ids.cpu().numpy(), d_score.cpu().numpy()
    assert tail_start.cpu().tolist() == ts
    for b in range(B):
        nb, L = vis[b], lens[b]
        live = np.concatenate([np.arange(ns + nb), np.arange(ts[b], L)])
        Kb = np.concatenate([K[b][:, live], kn[b][:, None]], axis=1)
        Vb = np.concatenate([V[b][:, live], vn[b][:, None]], axis=1)
        o, m, _ = orc.decode_attention(q[b:b + 1], Kb[None], Vb[None], ns, nb)
        assert_attention_close(got_o[b], o[0], dtype, f"b={b}")
        assert_mass_close(got_m[b, :nb], m[0], f"b={b}")
        kb = nb if keep_after < 0 else min(keep_after, nb)
        assert vis_len[b].item() == kb and kv_len[b].item() == L + 1, b        # the end of the tail only grows
        pos = orc.select_topk(score[b, :nb].astype(np.float64), ids[b, :nb], kb)
        got_ids = g_ids[b, :kb]
        if mode == st3.ST3_STABLE or kb == nb:
            assert np.array_equal(got_ids, ids[b, pos])
        else:
            assert sorted(got_ids.tolist()) == sorted(ids[b, pos].tolist())
        where = {int(t): p for p, t in enumerate(ids[b, :nb])}
        order = np.array([where[int(t)] for t in got_ids], dtype=np.int64)
        assert np.array_equal(g_score[b, :kb], score[b, order])
        assert np.array_equal(gK[b][:, :ns], K[b][:, :ns])
        assert np.array_equal(gK[b][:, ns:ns + kb], K[b][:, ns + order]) and np.array_equal(gV[b][:, ns:ns + kb], V[b][:, ns + order])
        # the tail: bit for bit where it was, the new row right behind it, nothing else touched from there on
        assert np.array_equal(gK[b][:, ts[b]:L], K[b][:, ts[b]:L]) and np.array_equal(gV[b][:, ts[b]:L], V[b][:, ts[b]:L])
        assert np.array_equal(gK[b][:, L], kn[b]) and np.array_equal(gV[b][:, L], vn[b])
        assert np.array_equal(gK[b][:, L + 1:], K0[b][:, L + 1:], equal_nan=True)


# ---------------------------------------------------------------------------
# prefill attention + mass
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,D,B,H,n,ns,nv,W", [
    ("f32", 64, 1, 4, 88, 8, 64, 1),
    ("f32", 64, 2, 2, 131, 0, 131, 4),          # everything visual, window reaches into the segment
    ("f32", 128, 1, 2, 65, 3, 40, 2),
    ("bf16", 128, 2, 3, 200, 35, 100, 1),
    ("bf16", 64, 1, 2, 300, 10, 250, 3),
    ("bf16", 128, 1, 2, 739, 35, 576, 1),
    ("bf16", 128, 1, 1, 1, 0, 1, 1),
])
def test_prefill_attention_matches_oracle(dtype, D, B, H, n, ns, nv, W):
    print(f"prefill dtype={dtype} D={D} B={B} H={H} n={n} W={W}", flush=True)
    rng = np.random.default_rng(zlib.crc32(repr((dtype, D, n, W)).encode()))
    sigma = 1.0 if dtype == "f32" else 1.43
    Q, K, V = (rand_values(rng, (B, H, n, D), dtype, sigma) for _ in range(3))
    shape = st3.make_shape(B, H, D, CODE[dtype])
    cap = n + 7                                             # K/V live inside a larger cache
    dK = torch.zeros((B, H, cap, D), dtype=TORCH_DTYPE[dtype], device=DEV); dK[:, :, :n] = to_dev(K, dtype)
    dV = torch.zeros((B, H, cap, D), dtype=TORCH_DTYPE[dtype], device=DEV); dV[:, :, :n] = to_dev(V, dtype)
    out = torch.zeros((B, H, n, D), dtype=TORCH_DTYPE[dtype], device=DEV)
    mass = torch.full((B, nv + 2), -3.0, dtype=torch.float32, device=DEV)
    st3.st3_prefill_attention(shape, to_dev(Q, dtype), dK[:, :, :n], dV[:, :, :n], n, ns, nv, W, out, mass,
                              _ws(shape, cap, nv, W))
    torch.cuda.synchronize()
    O, m = orc.prefill_attention(Q, K, V, ns, nv, W)
    assert_attention_close(to_np64(out), O, dtype)
    assert_mass_close(to_np64(mass)[:, :nv], m)
    assert np.all(to_np64(mass)[:, nv:] == -3.0)


@pytest.mark.parametrize("n", [129, 160, 161, 224, 257, 289, 321, 353, 385, 416, 449, 512, 513])
def test_prefill_query_tiles_cut_from_the_end(n):
    """The MFMA kernel cuts its 128-row query tiles from the end of the prompt in 32-row blocks, so a strip's
    first tile starts 0, 32, 64 or 96 rows before row 0: every such offset, with one to four tiles behind it."""
    print(f"prefill end-aligned tiles n={n}", flush=True)
    rng = np.random.default_rng(7700 + n)
    B, H, D, ns, W = 1, 2, 128, 5, 2
    nv = n - ns - 3
    Q, K, V = (rand_values(rng, (B, H, n, D), "bf16", 1.43) for _ in range(3))
    shape = st3.make_shape(B, H, D, CODE["bf16"])
    out = torch.full((B, H, n + 1, D), 7.0, dtype=torch.bfloat16, device=DEV)     # one guard row behind the prompt
    mass = torch.zeros((B, nv), dtype=torch.float32, device=DEV)
    st3.st3_prefill_attention(shape, to_dev(Q, "bf16"), to_dev(K, "bf16"), to_dev(V, "bf16"), n, ns, nv, W,
                              out[:, :, :n], mass, _ws(shape, n, nv, W))
    torch.cuda.synchronize()
    O, m = orc.prefill_attention(Q, K, V, ns, nv, W)
    assert_attention_close(to_np64(out[:, :, :n]), O, "bf16")
    assert_mass_close(to_np64(mass), m)
    assert np.all(to_np64(out[:, :, n]) == 7.0)


def test_prefill_rows_two_gib_apart_take_the_row_kernel():
    """The MFMA kernel addresses a strip as a scalar base plus 32 bits of offset; K and V whose rows lie so far
    apart that a strip spans 2 GiB or more must still come out right (the row kernel serves them)."""
    n, B, H, D, ns, nv, W = 3, 1, 2, 128, 0, 3, 1
    stride_t = 1 << 29                                              # elements: 1 GiB between consecutive rows
    print(f"prefill with stride_t={stride_t} elements", flush=True)
    rng = np.random.default_rng(4242)
    Q, K, V = (rand_values(rng, (B, H, n, D), "bf16", 1.43) for _ in range(3))
    shape = st3.make_shape(B, H, D, CODE["bf16"])
    big = [torch.zeros(((n - 1) * stride_t + H * D,), dtype=torch.bfloat16, device=DEV) for _ in range(2)]
    views = [b.as_strided((B, H, n, D), (0, D, stride_t, 1)) for b in big]
    views[0].copy_(to_dev(K, "bf16")); views[1].copy_(to_dev(V, "bf16"))
    out = torch.zeros((B, H, n, D), dtype=torch.bfloat16, device=DEV)
    mass = torch.zeros((B, nv), dtype=torch.float32, device=DEV)
    st3.st3_prefill_attention(shape, to_dev(Q, "bf16"), views[0], views[1], n, ns, nv, W, out, mass, _ws(shape, n, nv, W))
    torch.cuda.synchronize()
    O, m = orc.prefill_attention(Q, K, V, ns, nv, W)
    assert_attention_close(to_np64(out), O, "bf16")
    assert_mass_close(to_np64(mass), m)


# ---------------------------------------------------------------------------
# diagnostics: Overlap_n (Eq. 10), cosine similarity (Eq. 4-5)
# ---------------------------------------------------------------------------
def test_overlap_topk_matches_oracle():
    rng = np.random.default_rng(11)
    B = 5
    for n_a, n_b, k, id_space in [(576, 576, 288, 576), (300, 200, 100, 1000), (64, 64, 64, 64), (40, 90, 0, 128),
                                  (2880, 2000, 1440, 4096)]:
        print(f"overlap n_a={n_a} n_b={n_b} k={k}", flush=True)
        sa = rng.standard_normal((B, n_a)).astype(np.float32); sb = rng.standard_normal((B, n_b)).astype(np.float32)
        sa[1] = np.round(sa[1] * 2) / 2; sb[1] = np.round(sb[1] * 2) / 2          # ties decided by id
        ia = np.stack([rng.permutation(id_space)[:n_a] for _ in range(B)]).astype(np.int32)
        ib = np.stack([rng.permutation(id_space)[:n_b] for _ in range(B)]).astype(np.int32)
        na = [n_a, n_a // 2, n_a, 1, n_a]; nb = [n_b, n_b, n_b // 3, n_b, 1]
        ov = torch.full((B,), -1, dtype=torch.int32, device=DEV); ta = torch.full((B,), -1, dtype=torch.int32, device=DEV)
        st3.st3_overlap_topk(torch.from_numpy(sa).to(DEV), torch.from_numpy(ia).to(DEV), n_a,
                             torch.from_numpy(sb).to(DEV), torch.from_numpy(ib).to(DEV), n_b, k, id_space, ov, ta,
                             n_a_dev=_i32(na), n_b_dev=_i32(nb))
        torch.cuda.synchronize()
        for b in range(B):
            A = orc.topk_id_set(sa[b, :na[b]].astype(np.float64), ia[b, :na[b]], k)
            Bs = orc.topk_id_set(sb[b, :nb[b]].astype(np.float64), ib[b, :nb[b]], k)
            assert int(ta[b]) == len(A) and int(ov[b]) == len(A & Bs), (b, n_a, n_b, k)
            if len(A):
                assert int(ov[b]) / int(ta[b]) == orc.overlap(sa[b, :na[b]].astype(np.float64), ia[b, :na[b]],
                                                               sb[b, :nb[b]].astype(np.float64), ib[b, :nb[b]], k)


def test_cosine_similarity_matches_oracle():
    rng = np.random.default_rng(12)
    B = 4
    for n_a, n_b, id_space, with_ids in [(576, 576, 576, True), (300, 450, 1024, True), (739, 739, 739, False), (1, 5, 8, True)]:
        va = np.abs(rng.standard_normal((B, n_a))).astype(np.float32); vb = np.abs(rng.standard_normal((B, n_b))).astype(np.float32)
        va[2] = 0.0
        ia = np.stack([rng.permutation(id_space)[:n_a] for _ in range(B)]).astype(np.int32)
        ib = np.stack([rng.permutation(id_space)[:n_b] for _ in range(B)]).astype(np.int32)
        cs = torch.full((B,), 9.0, dtype=torch.float32, device=DEV)
        st3.st3_cosine_similarity(torch.from_numpy(va).to(DEV), torch.from_numpy(ia).to(DEV) if with_ids else None, n_a,
                                  torch.from_numpy(vb).to(DEV), torch.from_numpy(ib).to(DEV) if with_ids else None, n_b,
                                  id_space, cs)
        torch.cuda.synchronize()
        for b in range(B):
            want = orc.cosine_similarity(va[b].astype(np.float64), ia[b] if with_ids else np.arange(n_a),
                                         vb[b].astype(np.float64), ib[b] if with_ids else np.arange(n_b))
            assert abs(float(cs[b]) - want) <= 2e-6, (b, float(cs[b]), want)


def test_overlap_of_decode_mass_across_steps_current_mode():
    """The paper's use of Eq. 10: top-50 % sets of the same layer's visual mass at step 1 and step n."""
    import dataclasses
    from paper_2412_20105_amd import pipeline
    from workloads import decode_qkv, get_workload, prefill_qkv
    w = dataclasses.replace(get_workload("llava15_7b"), layers=1, heads=4, steps=4, n_vis=96, n_txt=8,
                            layer_schedule={"kind": "full"}, step_schedule={"kind": "none"})
    keep = pipeline.keep_table_for(w)
    gen = pipeline.Generation(1, w.heads, w.head_dim, torch.bfloat16, 2, w.n_sys, w.n_vis, w.n_txt, w.steps, keep, device=DEV)
    ref = orc.Generation(1, w.heads, w.head_dim, w.n_sys, w.n_vis, w.n_txt, np.array(keep))
    pre = prefill_qkv(w, 0, 2)
    ref.prefill(lambda l: pre)
    gen.prefill_layer(0, *(to_dev(x, "bf16") for x in pre))
    masses, ref_masses = [], []
    for t in range(1, w.steps + 1):
        d = decode_qkv(w, 0, t, 2)
        s = ref.decode_step(lambda l: d)
        out, mass = gen.decode_layer(0, t, *(to_dev(x, "bf16") for x in d))
        masses.append(mass.clone()); ref_masses.append(s["mass"][0])
    ids = gen.layers[0].ids
    ov = torch.zeros((2,), dtype=torch.int32, device=DEV); ta = torch.zeros((2,), dtype=torch.int32, device=DEV)
    k = w.n_vis // 2
    for n in range(w.steps):
        st3.st3_overlap_topk(masses[0], ids, w.n_vis, masses[n], ids, w.n_vis, k, w.n_vis, ov, ta)
        torch.cuda.synchronize()
        for b in range(2):
            want = orc.overlap(ref_masses[0][b], np.arange(w.n_vis), ref_masses[n][b], np.arange(w.n_vis), k)
            # the GPU ranks its own fp32 mass: allow one token to flip on a near-tie
            assert abs(int(ov[b]) / int(ta[b]) - want) <= 1.0 / k + 1e-12
        if n == 0:
            assert ov.cpu().tolist() == [k, k]
