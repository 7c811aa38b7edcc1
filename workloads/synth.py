"""Seeded synthetic Q/K/V tensors.

Every tensor is a pure function of (workload seed, tensor tag, layer, step):
a Philox counter-based stream is keyed by those four integers and standard
normals are drawn from it in C order.  Values are returned as float32; for
bf16 workloads they are first rounded to the nearest bf16 (ties to even), so
the float32 array holds exactly the numbers the device stores and the oracle
can widen them to float64 without loss.

Nothing here depends on attention, ranking or retention counts.
"""
from __future__ import annotations

import numpy as np

from .configs import Workload

_TAGS = {"q": 1, "k": 2, "v": 3, "dq": 4, "dk": 5, "dv": 6, "dir": 7, "perm": 8}


def _stream(seed: int, tag: str, layer: int, step: int) -> np.random.Generator:
    key = [np.uint64(seed), np.uint64((_TAGS[tag] << 40) | (layer << 20) | step)]
    return np.random.Generator(np.random.Philox(key=np.array(key, dtype=np.uint64)))


def bf16_round_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bf16 bit pattern, round to nearest, ties to even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(bits).astype(np.float64)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x = x.astype(np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(bf16_round_bits(x))
    if dtype == "f32":
        return x
    raise ValueError(dtype)


def normal_block(seed: int, tag: str, layer: int, step: int, shape, sigma: float) -> np.ndarray:
    """N(0, sigma^2) block of the given shape, float64, before storage rounding."""
    return _stream(seed, tag, layer, step).standard_normal(shape) * sigma


# ---------------------------------------------------------------------------
# planted structure of the skewed workload
# ---------------------------------------------------------------------------
N_HOT = 58          # ~10 % of 576 visual tokens
TIE_GROUP = 8
N_EXACT_GROUPS = 32  # 256 cold tokens whose K rows repeat bit for bit in groups of 8
N_NEAR_GROUPS = 16   # 128 cold tokens whose K rows differ by one bf16 ulp


def planted_layout(w: Workload):
    """Which visual token ids are hot / exact-tie / near-tie / free.

    Returns (hot_ids, exact_groups [G,8], near_groups [G,8], direction u [d]).
    """
    g = _stream(w.seed, "perm", 0, 0)
    perm = g.permutation(w.n_vis)
    hot = np.sort(perm[:N_HOT])
    cold = np.sort(perm[N_HOT:])
    ne = N_EXACT_GROUPS * TIE_GROUP
    nn = N_NEAR_GROUPS * TIE_GROUP
    exact = cold[:ne].reshape(N_EXACT_GROUPS, TIE_GROUP)
    near = cold[ne:ne + nn].reshape(N_NEAR_GROUPS, TIE_GROUP)
    u = _stream(w.seed, "dir", 0, 0).standard_normal(w.head_dim)
    u /= np.linalg.norm(u)
    return hot, exact, near, u


def _plant_amplitude(w: Workload) -> float:
    # a = b with a*b/sqrt(d) = ln 81: a hot key's logit is lifted by ln 81, so
    # 58 hot keys out of 576 take about 58*81/(58*81+518) = 90 % of the mass.
    return float(np.sqrt(np.log(81.0) * np.sqrt(w.head_dim)))


def _plant_keys(w: Workload, k: np.ndarray) -> np.ndarray:
    """k: [B,H,N0,d] float64 before rounding -> float32 stored values."""
    hot, exact, near, u = planted_layout(w)
    a = _plant_amplitude(w)
    s0 = w.n_sys
    k = k.copy()
    k[:, :, s0 + hot, :] += a * u
    for grp in exact:
        k[:, :, s0 + grp, :] = k[:, :, s0 + grp[:1], :]
    for grp in near:
        k[:, :, s0 + grp, :] = k[:, :, s0 + grp[:1], :]
    ks = _store(k, w.dtype)
    if w.dtype == "bf16":
        bits = bf16_round_bits(ks)
        for grp in near:
            for m in range(1, TIE_GROUP):
                # member m: one ulp up in magnitude, coordinate m of head 0
                bits[:, 0, s0 + grp[m], m] += np.uint16(1)
        ks = bf16_bits_to_f32(bits)
    else:
        for grp in near:
            for m in range(1, TIE_GROUP):
                col = ks[:, 0, s0 + grp[m], m].view(np.uint32)
                col += np.uint32(1)
    return ks


# ---------------------------------------------------------------------------
# public generators
# ---------------------------------------------------------------------------
def prefill_qkv(w: Workload, layer: int, batch: int):
    """Layer `layer`'s prompt tensors Q, K, V: float32 [B, H, N0, d]."""
    shape = (batch, w.heads, w.n_prompt, w.head_dim)
    q = normal_block(w.seed, "q", layer, 0, shape, w.sigma)
    k = normal_block(w.seed, "k", layer, 0, shape, w.sigma)
    v = normal_block(w.seed, "v", layer, 0, shape, w.sigma)
    if w.planted:
        _, _, _, u = planted_layout(w)
        q = q + _plant_amplitude(w) * u
        ks = _plant_keys(w, k)
    else:
        ks = _store(k, w.dtype)
    return _store(q, w.dtype), ks, _store(v, w.dtype)


def decode_qkv(w: Workload, layer: int, step: int, batch: int):
    """Layer `layer`'s tensors for the token consumed at decode step `step`>=1:
    q, k, v float32 [B, H, d] (decoder outputs taken as random vectors)."""
    shape = (batch, w.heads, w.head_dim)
    q = normal_block(w.seed, "dq", layer, step, shape, w.sigma)
    k = normal_block(w.seed, "dk", layer, step, shape, w.sigma)
    v = normal_block(w.seed, "dv", layer, step, shape, w.sigma)
    if w.planted:
        _, _, _, u = planted_layout(w)
        q = q + _plant_amplitude(w) * u
    return _store(q, w.dtype), _store(k, w.dtype), _store(v, w.dtype)
