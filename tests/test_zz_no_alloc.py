"""st3_decode_attention_noalloc (scratch in a device array of the library itself) against
st3_decode_attention (workspace passed in by the caller): same kernels, so outputs and masses
must agree to the bit, and both must match the oracle.  Two calls in a row share the array, the
second on a smaller input, which must not see anything the first one left behind."""
import ctypes as C

import numpy as np
import pytest
import torch

from gpu_util import DEV, TORCH_DTYPE, assert_attention_close, assert_mass_close, rand_values, to_dev, to_np64
from oracle import st3_oracle as orc
from paper_2412_20105_amd import binding as st3

pytestmark = pytest.mark.gpu

CODE = {"f32": st3.ST3_F32, "bf16": st3.ST3_BF16}


def _case(rng, dtype, D, B, H, lens, ns, nv):
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
    kv_len = torch.tensor(lens, dtype=torch.int32, device=DEV)
    vis_len = torch.tensor(vis, dtype=torch.int32, device=DEV)
    seg = st3.segments(ns, nv, max(lens), vis_len, kv_len)
    kv = st3.kv_layer(dK, dV)
    outs, masses = [], []
    for which in ("noalloc", "workspace"):
        out = torch.zeros((B, H, D), dtype=TORCH_DTYPE[dtype], device=DEV)
        mass = torch.full((B, nv + 3), -7.0, dtype=torch.float32, device=DEV)
        if which == "noalloc":
            st3.st3_decode_attention_noalloc(shape, dq, kv, seg, out, mass)
        else:
            ws = torch.empty((st3.st3_workspace_bytes(shape, cap, nv, 1),), dtype=torch.uint8, device=DEV)
            st3.st3_decode_attention(shape, dq, kv, seg, out, mass, ws)
        torch.cuda.synchronize()
        outs.append(out); masses.append(mass)
    assert torch.equal(outs[0].view(torch.uint8), outs[1].view(torch.uint8)), "outputs differ between the two entry points"
    assert torch.equal(masses[0], masses[1]), "masses differ between the two entry points"
    got_o, got_m = to_np64(outs[0]), to_np64(masses[0])
    for b in range(B):
        if lens[b] == 0:
            assert np.all(got_o[b] == 0)
            continue
        o, m, _ = orc.decode_attention(q[b:b + 1], K[b:b + 1, :, :lens[b]], V[b:b + 1, :, :lens[b]], ns, vis[b])
        assert_attention_close(got_o[b], o[0], dtype, f"b={b}")
        assert_mass_close(got_m[b, :vis[b]], m[0], f"b={b}")
        assert np.all(got_m[b, vis[b]:] == -7.0)


def test_noalloc_entry_point_matches_the_workspace_entry_point_on_two_calls_in_a_row():
    rng = np.random.default_rng(77)
    # first a larger input (strips cut into several chunks, ragged batch, an empty sequence) ...
    _case(rng, "bf16", 128, 4, 5, [739, 257, 0, 256], 35, 200)
    # ... then a smaller one on the same GPU: it finds the first call's partials and logits in the array
    _case(rng, "bf16", 128, 2, 3, [90, 33], 8, 40)
    # other element type and head size, enough strips that no strip is cut (no merge launch)
    _case(rng, "f32", 64, 8, 40, [300, 299, 5, 64, 1, 128, 200, 77], 4, 50)
    _case(rng, "f32", 64, 1, 2, [40], 0, 0)


def test_noalloc_entry_point_refuses_what_does_not_fit_its_array():
    lib = st3.lib()
    fake = 0x1000
    sh = st3.make_shape(64, 40, 128, st3.ST3_BF16)
    cap = 4096                                          # 64 * 40 * 4096 logits alone are 42 MB
    assert st3.st3_workspace_bytes(sh, cap, 0, 1) > st3.ST3_NOALLOC_SCRATCH_BYTES
    kv = st3.KvLayer(fake, fake, 40 * cap * 128, cap * 128, 128, cap)
    seg = st3.Segments(8, 64, 100, fake, fake)
    assert lib.st3_decode_attention_noalloc(C.byref(sh), fake, C.byref(kv), C.byref(seg), fake, None, 0,
                                            None) == st3.ST3_ERR_WORKSPACE_TOO_SMALL
    assert lib.st3_decode_attention_noalloc(C.byref(sh), None, C.byref(kv), C.byref(seg), fake, None, 0,
                                            None) == st3.ST3_ERR_INVALID_ARG
