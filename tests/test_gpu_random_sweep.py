"""Randomised sweep of the fused decode call over its whole argument space: both cache layouts,
right / wrong / absent layout hints, one to many chunks per strip, ragged batches with tail-less
sequences, both compaction modes, with and without a mass output.  Every case is checked
against the oracle like the hand-picked cases of test_gpu_parity.py; the seeds are fixed."""
import numpy as np
import pytest
import torch

from gpu_util import DEV, TORCH_DTYPE, assert_attention_close, assert_mass_close, rand_values, to_dev, to_np64
from oracle import st3_oracle as orc
from paper_2412_20105_amd import binding as st3

pytestmark = pytest.mark.gpu

CODE = {"f32": st3.ST3_F32, "bf16": st3.ST3_BF16}


def _i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


def _case(seed):
    rng = np.random.default_rng(1000 + seed)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    D = int(rng.choice([64, 128]))
    B = int(rng.integers(1, 5))
    H = int(rng.choice([1, 2, 3, 5, 8]))
    ns = int(rng.choice([0, 1, 6, 35]))
    long_cache = rng.random() < 0.35                  # few strips and many rows: the strip is cut into chunks
    vmax = int(rng.integers(1, 700 if long_cache else 150))
    vis = [int(rng.integers(0, vmax + 1)) for _ in range(B)]
    vis[int(rng.integers(0, B))] = vmax
    fixed = rng.random() < 0.6
    gaps = [int(rng.choice([0, 1, 31, 32, 33, int(rng.integers(0, 200))])) if fixed else 0 for _ in range(B)]
    tmax = 2500 if long_cache else 120
    tails = [int(rng.choice([0, 1, int(rng.integers(0, tmax))])) for _ in range(B)]
    ts = [ns + v + g for v, g in zip(vis, gaps)]
    lens = [t + r for t, r in zip(ts, tails)]
    keep_after = int(rng.choice([-1, 0, max(0, vmax - 1), int(rng.integers(0, vmax + 1))]))
    mode = int(rng.choice([st3.ST3_STABLE, st3.ST3_HOLE_FILL]))
    hint = str(rng.choice(["none", "first", "last", "far"])) if fixed else "none"
    want_mass = rng.random() < 0.8
    return dict(seed=seed, dtype=dtype, D=D, B=B, H=H, ns=ns, vis=vis, fixed=fixed, ts=ts, tails=tails, lens=lens,
                keep_after=keep_after, mode=mode, hint=hint, want_mass=want_mass)


@pytest.mark.parametrize("block", range(12))
def test_decode_layer_step_random_cases(block):
    _run_cases(range(block * 10, block * 10 + 10))


@pytest.mark.parametrize("tile", [1, 4, 6, 8])
def test_decode_layer_step_random_cases_with_every_tile_size(tile):
    """The attend kernel picks one of its builds (loads per lane and tile) from the size of the launch;
    small launches like these would only ever reach one of them, so each build is forced in turn."""
    st3.st3_debug_set_attend_tile(tile)
    try:
        _run_cases(range(200, 216))
    finally:
        st3.st3_debug_set_attend_tile(0)


def _run_cases(seeds):
    for seed in seeds:
        c = _case(seed)
        print("sweep case", {k: c[k] for k in ("seed", "dtype", "D", "B", "H", "ns", "vis", "fixed", "ts", "lens",
                                               "keep_after", "mode", "hint", "want_mass")}, flush=True)
        rng = np.random.default_rng(5000 + seed)
        dtype, D, B, H, ns, vis, lens, ts = c["dtype"], c["D"], c["B"], c["H"], c["ns"], c["vis"], c["lens"], c["ts"]
        nv = max(vis)
        cap = max(lens) + 1 + int(rng.integers(0, 4))
        sigma = 1.0 if dtype == "f32" else 1.43
        K = rand_values(rng, (B, H, cap, D), dtype, sigma); V = rand_values(rng, (B, H, cap, D), dtype, sigma)
        q, kn, vn = (rand_values(rng, (B, H, D), dtype, sigma) for _ in range(3))
        score = rng.standard_normal((B, max(nv, 1))).astype(np.float32)
        ids = np.stack([rng.permutation(4000)[:max(nv, 1)] for _ in range(B)]).astype(np.int32)
        shape = st3.make_shape(B, H, D, CODE[dtype])
        dK, dV = to_dev(K, dtype), to_dev(V, dtype)
        for b in range(B):                                 # dead rows and everything past the end: NaN
            for t in (dK, dV):
                t[b, :, ns + vis[b]:ts[b]] = float("nan"); t[b, :, lens[b]:] = float("nan")
        d_score, d_ids = torch.from_numpy(score.copy()).to(DEV), torch.from_numpy(ids.copy()).to(DEV)
        out = torch.zeros((B, H, D), dtype=TORCH_DTYPE[dtype], device=DEV)
        mass = torch.full((B, nv + 2), -7.0, dtype=torch.float32, device=DEV) if c["want_mass"] else None
        vis_len, kv_len = _i32(vis), _i32(lens)
        tail_start = _i32(ts) if c["fixed"] else None
        guess = {"none": (0, 0), "first": (vis[0], ts[0]), "last": (vis[-1], ts[-1]), "far": (3, 2 ** 31 - 1)}[c["hint"]]
        seg = st3.segments(ns, nv, max(lens), vis_len, kv_len, tail_start, *guess)
        n_ws = st3.st3_workspace_bytes(shape, cap, nv, 1)
        ws = torch.empty((n_ws,), dtype=torch.uint8, device=DEV); ws.fill_(0xFF)
        st3.st3_workspace_init(shape, cap, ws)
        keep_after = c["keep_after"]
        st3.st3_decode_layer_step(shape, st3.kv_layer(dK, dV), seg, d_score, d_ids, keep_after, c["mode"], to_dev(q, dtype),
                                  to_dev(kn, dtype), to_dev(vn, dtype), out, mass, ws)
        torch.cuda.synchronize()
        got_o = to_np64(out)
        got_m = to_np64(mass) if mass is not None else None
        gK, gV = dK.float().cpu().numpy(), dV.float().cpu().numpy()
        g_ids = d_ids.cpu().numpy()
        for b in range(B):
            nb, L = vis[b], lens[b]
            live = np.concatenate([np.arange(ns + nb), np.arange(ts[b], L)]).astype(np.int64)
            Kb = np.concatenate([K[b][:, live], kn[b][:, None]], axis=1)
            Vb = np.concatenate([V[b][:, live], vn[b][:, None]], axis=1)
            o, m, _ = orc.decode_attention(q[b:b + 1], Kb[None], Vb[None], ns, nb)
            assert_attention_close(got_o[b], o[0], dtype, f"seed={seed} b={b}")
            if got_m is not None:
                assert_mass_close(got_m[b, :nb], m[0], f"seed={seed} b={b}")
                assert np.all(got_m[b, nb:] == -7.0)
            kb = nb if keep_after < 0 else min(keep_after, nb)
            want_len = L + 1 if c["fixed"] else L + 1 - (nb - kb)
            assert vis_len[b].item() == kb and kv_len[b].item() == want_len, (seed, b)
            pos = orc.select_topk(score[b, :nb].astype(np.float64), ids[b, :nb], kb)
            got_ids = g_ids[b, :kb]
            if c["mode"] == st3.ST3_STABLE or kb == nb:
                assert np.array_equal(got_ids, ids[b, pos]), (seed, b)
            else:
                assert sorted(got_ids.tolist()) == sorted(ids[b, pos].tolist()), (seed, b)
            where = {int(t): p for p, t in enumerate(ids[b, :nb])}
            order = np.array([where[int(t)] for t in got_ids], dtype=np.int64)
            assert np.array_equal(gK[b][:, ns:ns + kb], K[b][:, ns + order]), (seed, b)
            assert np.array_equal(gV[b][:, ns:ns + kb], V[b][:, ns + order]), (seed, b)
            # the rows behind the segment plus the new one: the same multiset, K and V moved together
            lo = ts[b] if c["fixed"] else ns + kb
            got_tail_K, got_tail_V = gK[b][:, lo:want_len], gV[b][:, lo:want_len]
            src = np.concatenate([np.arange(ts[b], L), [-1]]).astype(np.int64)       # -1: the appended row
            rowK = lambda r: kn[b] if r < 0 else K[b][:, r]
            rowV = lambda r: vn[b] if r < 0 else V[b][:, r]
            key = {rowK(r)[0].tobytes(): int(r) for r in src}
            assert got_tail_K.shape[1] == len(src), (seed, b)
            srcs = [key[got_tail_K[0, j].tobytes()] for j in range(got_tail_K.shape[1])]
            assert sorted(srcs) == sorted(src.tolist()), (seed, b)
            if c["fixed"] or c["mode"] == st3.ST3_STABLE:
                assert srcs == src.tolist(), (seed, b)
            for j, r in enumerate(srcs):
                assert np.array_equal(got_tail_K[:, j], rowK(r)) and np.array_equal(got_tail_V[:, j], rowV(r)), (seed, b, j)


@pytest.mark.parametrize("block", range(6))
def test_prefill_attention_random_cases(block):
    """Prompt lengths around the tile edges of both prefill kernels (128 queries, 64 keys), every
    window, visual segments anywhere in the prompt, K and V as strided views of a larger cache."""
    for seed in range(block * 6, block * 6 + 6):
        rng = np.random.default_rng(9000 + seed)
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        D = int(rng.choice([64, 128]))
        B, H = int(rng.integers(1, 3)), int(rng.choice([1, 2, 5]))
        n = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257,
                            int(rng.integers(1, 600))]))
        ns = int(rng.integers(0, n + 1))
        nv = int(rng.integers(0, n - ns + 1))
        W = int(rng.integers(1, min(n, 16) + 1))
        print(f"prefill sweep seed={seed} dtype={dtype} D={D} B={B} H={H} n={n} ns={ns} nv={nv} W={W}", flush=True)
        sigma = 1.0 if dtype == "f32" else 1.43
        Q, K, V = (rand_values(rng, (B, H, n, D), dtype, sigma) for _ in range(3))
        shape = st3.make_shape(B, H, D, CODE[dtype])
        cap = n + int(rng.integers(0, 9))
        dK = torch.full((B, H, cap, D), float("nan"), dtype=TORCH_DTYPE[dtype], device=DEV); dK[:, :, :n] = to_dev(K, dtype)
        dV = torch.full((B, H, cap, D), float("nan"), dtype=TORCH_DTYPE[dtype], device=DEV); dV[:, :, :n] = to_dev(V, dtype)
        out = torch.zeros((B, H, n, D), dtype=TORCH_DTYPE[dtype], device=DEV)
        mass = torch.full((B, nv + 2), -3.0, dtype=torch.float32, device=DEV)
        n_ws = st3.st3_workspace_bytes(shape, cap, nv, W)
        ws = torch.empty((n_ws,), dtype=torch.uint8, device=DEV); ws.fill_(0xFF)
        st3.st3_workspace_init(shape, cap, ws)
        st3.st3_prefill_attention(shape, to_dev(Q, dtype), dK[:, :, :n], dV[:, :, :n], n, ns, nv, W, out, mass, ws)
        torch.cuda.synchronize()
        O, m = orc.prefill_attention(Q, K, V, ns, nv, W)
        assert_attention_close(to_np64(out), O, dtype, f"seed={seed}")
        assert_mass_close(to_np64(mass)[:, :nv], m, f"seed={seed}")
        assert np.all(to_np64(mass)[:, nv:] == -3.0)
