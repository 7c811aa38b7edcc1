"""CPU oracle for the ST3 attention / pruning path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 NumPy statement of what the hot path computes, written
from the paper (ST3: Spatial-Temporal Visual Token Trimming) and sharing no
code with the HIP library.  Only tests, the smoke check and the benchmark's
`cpu_baseline` leg may import this module; the product path never does.

What is defined here, and the passage each part follows:

* `causal_attention`, `decode_attention`  - Eq. 2 (softmax((QK^T + M)/sqrt d) V,
  M = -inf above the diagonal), the latter being Eq. 2 with a single query row
  placed after every cached key.
* the `mass` outputs of `prefill_attention` / `decode_attention` - Sec. 3.2:
  the last row(s) of A, restricted to the visual key positions; reduced over
  heads by a mean (the paper treats the row as one vector and is silent on
  heads) and over the last W query rows by a sum (W = 1 is the paper's choice).
* `select_topk`                           - Eq. 3: indices of the G largest
  scores.  Ties: lower original token id wins.
* `beta_cos`, `beta_linear`, `beta_exp`   - Eq. 8 and Sec. 4.4.
* `keep_pvtp`                             - Sec. 3.2/4.2, Eq. 9, Alg. 1: no
  pruning in layers 0..2, first event at layer 3 removes P, each later event
  (every S layers) removes R of the ORIGINAL count.
* `keep_linear`, `keep_anneal`            - the benchmark's linear-over-layers
  schedule and Eq. 7 (count = |V^{l,0}| * beta^t, floored).
* `kv_bytes`                              - closed-form KV-cache size.
* `overlap`, `cosine_similarity`          - Eq. 10 and Eq. 4-5 (diagnostics).
* `Generation`                            - Alg. 3 end to end on given Q/K/V:
  prefill with progressive pruning, then decode steps with annealing.
* `e4m3_decode`, `e4m3_quantize`, `Generation(kv_format="e4m3")` - NOT from the
  paper: the KV cache held in OCP FP8 E4M3 with one float32 scale per (b, h)
  strip for K and one for V, as an implementation variant of the cache of
  Sec. 4.3.  Codes follow the OCP 8-bit floating point specification (bias 7,
  no infinities, S.1111.111 = NaN, largest finite 448); the quantiser divides
  by the scale in float32, saturates at +-448 and rounds to nearest, ties to
  the even code.  Attention then reads code value x scale.
* `heredity_attention` and `Generation(lazy=...)` - Eq. 6 / Alg. 2 (QK
  heredity): a lazy layer l computes Self-attn(Q^{l-n}, K^{l-n}, V^l), i.e. the
  source layer's probabilities applied to its own values.

Pins (tests/test_oracle_*.py): full attention at keep ratio 1 against a
library SDPA in float64; softmax rows sum to 1; all-equal keys; permutation
invariance; mass sums; brute-force top-k on all small cases; nestedness; the
60 printed (L,S,R,P)->C rows of the paper's stride tables; beta closed forms;
KV bytes against the paper's Table 2 baseline rows; QK heredity: equal values
give back the source layer's output, the result is linear in V, one-hot values
return the probabilities themselves; E4M3: all 256 codes and in-range
rounding against a library float8_e4m3fn conversion, midpoints, saturation,
idempotence.  Accuracy/CIDEr/A100
latency figures of the paper are parity unpinned (they need datasets, trained
weights and other systems).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np

F64 = np.float64


# ---------------------------------------------------------------------------
# Eq. 2: attention
# ---------------------------------------------------------------------------
def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Row-wise softmax of a float64 matrix; -inf entries get probability 0."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_probs_causal(q: np.ndarray, k: np.ndarray, scale: Optional[float] = None) -> np.ndarray:
    """A = Softmax((Q K^T + M)/sqrt(d)) for one head.  q, k: [n, d] -> [n, n]."""
    q = np.asarray(q, F64)
    k = np.asarray(k, F64)
    n, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    s = q @ k.T
    mask = np.triu(np.ones((n, n), dtype=bool), 1)    # strictly above the diagonal
    s = np.where(mask, -np.inf, s)
    return softmax_rows(s * scale)


def causal_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: Optional[float] = None):
    """Eq. 2 for every (b, h).  Q, K, V: [B, H, n, d].

    Returns (O [B,H,n,d], A [B,H,n,n]).  A is returned whole so that callers can
    read any row of it; use small n.
    """
    Q = np.asarray(Q, F64); K = np.asarray(K, F64); V = np.asarray(V, F64)
    B, H, n, d = Q.shape
    O = np.empty((B, H, n, d), F64)
    A = np.empty((B, H, n, n), F64)
    for b in range(B):
        for h in range(H):
            a = attention_probs_causal(Q[b, h], K[b, h], scale)
            A[b, h] = a
            O[b, h] = a @ V[b, h]
    return O, A


def prefill_attention(Q, K, V, n_sys: int, n_vis: int, window: int = 1, scale: Optional[float] = None):
    """Causal attention over a prompt laid out [S, V, I] plus the visual mass.

    mass[b, j] = (1/H) sum_h sum_{r in last `window` rows} A_h[r, n_sys + j].
    Does not materialise A for all heads at once, so it is usable at n ~ 3000.
    Returns (O [B,H,n,d], mass [B,n_vis]).
    """
    Q = np.asarray(Q, F64); K = np.asarray(K, F64); V = np.asarray(V, F64)
    B, H, n, d = Q.shape
    if not (0 <= n_sys and 0 <= n_vis and n_sys + n_vis <= n and 1 <= window <= n):
        raise ValueError("bad segment layout")
    O = np.empty((B, H, n, d), F64)
    mass = np.zeros((B, n_vis), F64)
    for b in range(B):
        for h in range(H):
            a = attention_probs_causal(Q[b, h], K[b, h], scale)
            O[b, h] = a @ V[b, h]
            mass[b] += a[n - window:, n_sys:n_sys + n_vis].sum(axis=0)
    return O, mass / H


def decode_attention(q, K, V, n_sys: int, n_vis: int, scale: Optional[float] = None):
    """One new query per (b, h) over a cache of `Lkv` keys, all of which precede it.

    q: [B,H,d]; K, V: [B,H,Lkv,d] (visual keys at [n_sys, n_sys+n_vis)).
    Returns (o [B,H,d], mass [B,n_vis], p [B,H,Lkv]).
    """
    q = np.asarray(q, F64); K = np.asarray(K, F64); V = np.asarray(V, F64)
    B, H, Lkv, d = K.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    o = np.empty((B, H, d), F64)
    p = np.empty((B, H, Lkv), F64)
    for b in range(B):
        for h in range(H):
            s = (K[b, h] @ q[b, h]) * scale
            ph = softmax_rows(s[None, :])[0]
            p[b, h] = ph
            o[b, h] = ph @ V[b, h]
    mass = p[:, :, n_sys:n_sys + n_vis].mean(axis=1)
    return o, mass, p


def heredity_attention(Q_src, K_src, V, scale: Optional[float] = None) -> np.ndarray:
    """Eq. 6: the attention of a lazy layer, Self-attn(Q^{l-n}, K^{l-n}, V^l): the causal
    probabilities of the source layer's queries and keys, applied to this layer's values.
    Q_src, K_src, V: [B, H, n, d] -> [B, H, n, d]."""
    return causal_attention(Q_src, K_src, V, scale)[0]


# ---------------------------------------------------------------------------
# Eq. 3: top-G selection
# ---------------------------------------------------------------------------
def select_topk(scores: Sequence[float], ids: Sequence[int], k: int) -> np.ndarray:
    """Positions (ascending) of the k best entries under (score desc, id asc)."""
    scores = np.asarray(scores, F64)
    ids = np.asarray(ids)
    n = scores.shape[0]
    if not 0 <= k <= n:
        raise ValueError("k out of range")
    order = sorted(range(n), key=lambda i: (-scores[i], int(ids[i])))
    return np.array(sorted(order[:k]), dtype=np.int64)


def ranked_order(scores, ids) -> np.ndarray:
    """All positions, best first, under the same total order (Alg. 3's T[l])."""
    scores = np.asarray(scores, F64)
    n = scores.shape[0]
    return np.array(sorted(range(n), key=lambda i: (-scores[i], int(ids[i]))), dtype=np.int64)


# ---------------------------------------------------------------------------
# Eq. 10 and Eq. 4-5: diagnostics on score vectors
# ---------------------------------------------------------------------------
def topk_id_set(scores, ids, k: int) -> set:
    """Token ids of the k best entries (same total order as select_topk)."""
    ids = np.asarray(ids)
    return set(int(ids[p]) for p in select_topk(scores, ids, min(k, len(ids))))


def overlap(scores_1, ids_1, scores_n, ids_n, k: int) -> float:
    """Eq. 10: |TopK(T_1) & TopK(T_n)| / |TopK(T_1)|."""
    a = topk_id_set(scores_1, ids_1, k)
    b = topk_id_set(scores_n, ids_n, k)
    return len(a & b) / len(a)


def cosine_similarity(sa, ids_a, sb, ids_b) -> float:
    """Eq. 4-5: cosine similarity of two score vectors, entries matched by token id; a token
    present on one side only counts as zero on the other."""
    sa = np.asarray(sa, F64); sb = np.asarray(sb, F64)
    where_b = {int(t): j for j, t in enumerate(ids_b)}
    dot = 0.0
    for i, t in enumerate(ids_a):
        j = where_b.get(int(t))
        if j is not None:
            dot += sa[i] * sb[j]
    na, nb = math.sqrt(float(sa @ sa)), math.sqrt(float(sb @ sb))
    return dot / (na * nb) if na > 0 and nb > 0 else 0.0


# ---------------------------------------------------------------------------
# Eq. 8 / Sec. 4.4: attenuation functions, argument = number of generated tokens
# ---------------------------------------------------------------------------
def beta_cos(n_out: int, tau: float) -> float:
    return math.cos(n_out * math.pi / (2.0 * tau)) if n_out < tau else 0.0


def beta_linear(n_out: int, tau: float) -> float:
    return 1.0 - n_out / tau if n_out < tau else 0.0


def beta_exp(n_out: int, sigma: float) -> float:
    return math.exp(-n_out / sigma)


# ---------------------------------------------------------------------------
# retention schedules (host-side integers; the device only ever sees counts)
# ---------------------------------------------------------------------------
def pvtp_events(L: int, S: int, first_layer: int = 3) -> List[int]:
    """0-indexed layers at which Alg. 1 prunes: l >= 3 and (l-3) % S == 0."""
    return [l for l in range(L) if l >= first_layer and (l - first_layer) % S == 0]


def keep_pvtp(L: int, n_vis: int, S: int, P_bp: int, R_bp: int, first_layer: int = 3) -> List[int]:
    """Visual tokens held by each layer at prefill under stride S.

    The first event removes P of the original count, every later event a
    further R of the ORIGINAL count (Eq. 9 is additive in R); ratios are in
    basis points so the arithmetic is exact; counts are floored, never < 0.
    """
    keep = []
    removed_bp = 0
    for l in range(L):
        if l >= first_layer and (l - first_layer) % S == 0:
            removed_bp += P_bp if l == first_layer else R_bp
        ratio_bp = max(0, 10000 - removed_bp)
        keep.append((n_vis * ratio_bp) // 10000)
    return keep


def conserved_ratio_bp(L: int, S: int, P_bp: int, R_bp: int, first_layer: int = 3) -> int:
    """Last-layer conserved ratio C in basis points: 1 - P - E*R, E = later events."""
    events = pvtp_events(L, S, first_layer)
    return 10000 - P_bp - (len(events) - 1) * R_bp


def keep_linear(L: int, n_vis: int, last_full_layer: int, end_ratio_bp: int) -> List[int]:
    """Keep ratio falling linearly from 1 at `last_full_layer` to `end_ratio` at L-1."""
    den = (L - 1) - last_full_layer
    keep = []
    for l in range(L):
        if l <= last_full_layer:
            keep.append(n_vis)
        else:
            num = n_vis * (10000 - end_ratio_bp) * (l - last_full_layer)
            dropped = -((-num) // (10000 * den))       # ceil
            keep.append(n_vis - dropped)
    return keep


def keep_anneal(keep_l0: Sequence[int], T: int, kind: str, param: float) -> np.ndarray:
    """Eq. 7: keep[l][t] = floor(keep[l][0] * beta^t) for t = 0..T, [L, T+1] int.

    kind "drop" is the tiny workload's rule: `param` tokens fewer per step.
    """
    L = len(keep_l0)
    out = np.zeros((L, T + 1), dtype=np.int64)
    for l in range(L):
        for t in range(T + 1):
            if kind == "cos":
                c = math.floor(keep_l0[l] * beta_cos(t, param) + 1e-9)
            elif kind == "linear":
                c = math.floor(keep_l0[l] * beta_linear(t, param) + 1e-9)
            elif kind == "exp":
                c = math.floor(keep_l0[l] * beta_exp(t, param) + 1e-9)
            elif kind == "drop":
                c = max(0, keep_l0[l] - int(param) * t)
            elif kind == "none":
                c = keep_l0[l]
            else:
                raise ValueError(kind)
            out[l, t] = min(c, keep_l0[l])
    return out


def schedule_for(workload) -> np.ndarray:
    """keep[l][t] table for a `workloads.Workload` from its schedule parameters."""
    ls = workload.layer_schedule
    if ls["kind"] == "table":
        keep0 = list(ls["keep"])
    elif ls["kind"] == "linear":
        keep0 = keep_linear(workload.layers, workload.n_vis, ls["last_full_layer"], ls["end_ratio_bp"])
    elif ls["kind"] == "pvtp":
        keep0 = keep_pvtp(workload.layers, workload.n_vis, ls["S"], ls["P_bp"], ls["R_bp"])
    elif ls["kind"] == "full":
        keep0 = [workload.n_vis] * workload.layers
    else:
        raise ValueError(ls["kind"])
    ss = workload.step_schedule
    if ss["kind"] == "drop":
        return keep_anneal(keep0, workload.steps, "drop", ss["per_step"])
    if ss["kind"] in ("cos", "linear"):
        return keep_anneal(keep0, workload.steps, ss["kind"], ss["tau"])
    if ss["kind"] == "exp":
        return keep_anneal(keep0, workload.steps, "exp", ss["sigma"])
    if ss["kind"] == "none":
        return keep_anneal(keep0, workload.steps, "none", 0)
    raise ValueError(ss["kind"])


def kv_len(n_sys: int, keep_lt: int, n_txt: int, t: int) -> int:
    """Keys held by a layer while decoding step t (t = 0: right after prefill)."""
    return n_sys + keep_lt + n_txt + t


def kv_bytes(B: int, H: int, d: int, elem_bytes: int, lens: Sequence[int],
             value_only: Sequence[int] = ()) -> int:
    """KV-cache bytes: K and V, every layer, `lens[l]` keys each.  Layers listed in
    `value_only` (lazy layers of Alg. 2, which never form K) hold V alone."""
    vo = set(int(l) for l in value_only)
    return B * sum((1 if l in vo else 2) * H * d * elem_bytes * int(n) for l, n in enumerate(lens))


# ---------------------------------------------------------------------------
# FP8 E4M3 KV-cache variant (implementation choice, not in the paper)
# ---------------------------------------------------------------------------
E4M3_MAX = 448.0


def e4m3_decode(codes) -> np.ndarray:
    """Value of OCP FP8 E4M3 codes (uint8): sign bit, 4 exponent bits (bias 7), 3 mantissa bits;
    exponent 0 is subnormal (m/8 * 2^-6); S.1111.111 is NaN; there are no infinities."""
    c = np.asarray(codes, np.uint8).astype(np.int64)
    sign = np.where(c >> 7 == 1, -1.0, 1.0)
    e = (c >> 3) & 15
    m = c & 7
    normal = (1.0 + m / 8.0) * np.exp2((e - 7).astype(F64))
    sub = (m / 8.0) * 2.0 ** -6
    v = sign * np.where(e == 0, sub, normal)
    return np.where((e == 15) & (m == 7), np.nan, v)


def e4m3_quantize(x, scale) -> np.ndarray:
    """Codes of x / scale: the division is done in float32 (x and scale as float32), the quotient
    saturates at +-448 and is rounded to the nearest E4M3 value, ties to the even code; the sign is
    kept (also of zero); NaN gives 0x7F."""
    t = np.asarray(x, np.float32) / np.asarray(scale, np.float32)
    table = e4m3_decode(np.arange(0x7F, dtype=np.uint8))       # the 127 non-negative finite values, ascending
    a = np.minimum(np.abs(t).astype(F64), E4M3_MAX)
    hi = np.clip(np.searchsorted(table, a, side="left"), 0, 0x7E)      # first value >= a
    lo = np.maximum(hi - 1, 0)
    d_hi, d_lo = table[hi] - a, a - table[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    code = np.where(np.signbit(t), code | 0x80, code).astype(np.uint8)
    return np.where(np.isnan(t), np.uint8(0x7F), code).astype(np.uint8)


def e4m3_roundtrip(x, scale) -> np.ndarray:
    """What a cache in E4M3 returns for x: decode(quantize(x, scale)) * scale (scale as float32)."""
    sc = np.asarray(scale, np.float32).astype(F64)
    return e4m3_decode(e4m3_quantize(x, scale)) * sc


# ---------------------------------------------------------------------------
# Alg. 3 end to end
# ---------------------------------------------------------------------------
class Generation:
    """Prefill with progressive pruning, then decode steps with annealing.

    State per layer l and sequence b (sequences are independent):
      ids[l][b]   original visual token ids alive at layer l, ascending
      rho[l][b]   the score that ranks them (aligned with ids)
      K[l], V[l]  cache as lists per b of arrays [H, len, d] in the order
                  system | alive visual (ascending id) | text | generated
    mode "static": rho is fixed at prefill (Alg. 3's top-index cache T[l]).
    mode "current": rho is replaced by the layer's own mass after every step.
    lazy (Eq. 6, Alg. 2): {l: src} makes layer l a lazy layer of source layer src < l.  Its
      Q and K inputs are ignored; its attention is Self-attn(Q^src, K^src, V^l), at prefill
      and at every decode step, so its probabilities, mass, kept set and ranking are the
      source's.  Lazy layers follow their source directly (src+1 .. src+n, the paper's
      "28 -> 29~31") and share its row of the keep table; K[l] stays None for them.
    """

    def __init__(self, L: int, H: int, d: int, n_sys: int, n_vis: int, n_txt: int,
                 keep: np.ndarray, window: int = 1, mode: str = "static",
                 scale: Optional[float] = None, lazy: Optional[Dict[int, int]] = None,
                 kv_format: str = "same", k_scale=None, v_scale=None):
        self.L, self.H, self.d = L, H, d
        self.n_sys, self.n_vis, self.n_txt = n_sys, n_vis, n_txt
        self.keep = np.asarray(keep)
        assert self.keep.shape[0] == L
        self.window, self.mode, self.scale = window, mode, scale
        # kv_format "e4m3": what enters a cache (prefill rows, appended rows) is replaced by its
        # E4M3 round trip with scales k_scale[b, h], v_scale[b, h]; the prefill attention itself
        # still sees the unquantised prompt
        if kv_format not in ("same", "e4m3"):
            raise ValueError(kv_format)
        self.kv_format = kv_format
        self.k_scale = None if k_scale is None else np.asarray(k_scale, np.float32)
        self.v_scale = None if v_scale is None else np.asarray(v_scale, np.float32)
        self.lazy = dict(lazy or {})
        for l, src in self.lazy.items():
            if not (0 <= src < l < L) or src in self.lazy:
                raise ValueError("a lazy layer needs a non-lazy source layer before it")
            if any(m not in self.lazy or self.lazy[m] != src for m in range(src + 1, l)):
                raise ValueError("lazy layers must follow their source directly")
            if not np.array_equal(self.keep[l], self.keep[src]):
                raise ValueError("a lazy layer keeps what its source keeps")
        self.ids: List[List[np.ndarray]] = []
        self.rho: List[List[np.ndarray]] = []
        self.K: List[List[np.ndarray]] = []
        self.V: List[List[np.ndarray]] = []
        self.t = 0

    def _into_cache(self, rows: np.ndarray, scales, b: int) -> np.ndarray:
        """rows [H, n, d] as the cache of sequence b will return them."""
        if self.kv_format == "same":
            return np.array(rows, F64)
        return e4m3_roundtrip(rows, scales[b][:, None, None])

    # -- prefill ------------------------------------------------------------
    def prefill(self, qkv_of_layer) -> Dict[str, list]:
        """qkv_of_layer(l) -> (Q, K, V) each [B, H, N0, d] over the UNPRUNED prompt.

        Returns per-layer lists: "out" (O_l per b, [H, n_l, d]), "mass" (per b),
        "ids" (per b), "selected" (positions kept within the previous layer's
        alive list at a prune event, else None).
        """
        L, ns, nv, nx = self.L, self.n_sys, self.n_vis, self.n_txt
        res = {"out": [], "mass": [], "ids": [], "selected": []}
        prev_ids = prev_mass = None
        inherited = None      # per b: scores of the most recent prune event, cut to the alive set
        src_QK = {}           # source layer -> its (Q, K) inputs, for the lazy layers behind it
        for l in range(L):
            Q, K, V = (np.asarray(x, F64) for x in qkv_of_layer(l))
            if l in self.lazy:
                Q, K = src_QK[self.lazy[l]]           # Eq. 6: Q^{l-n}, K^{l-n}
            elif l in self.lazy.values():
                src_QK[l] = (Q, K)
            B = Q.shape[0]
            if l == 0:
                prev_ids = [np.arange(nv, dtype=np.int64) for _ in range(B)]
                inherited = [None] * B
            k_l = int(self.keep[l, 0])
            ids_l, sel_l = [], []
            for b in range(B):
                if k_l < len(prev_ids[b]):
                    # Eq. 3: rank by the PREVIOUS layer's scores
                    pos = select_topk(prev_mass[b], prev_ids[b], k_l)
                    ids_l.append(prev_ids[b][pos])
                    inherited[b] = prev_mass[b][pos]
                    sel_l.append(pos)
                else:
                    ids_l.append(prev_ids[b])
                    sel_l.append(None)
            out_l, mass_l, rho_l, Kc, Vc = [], [], [], [], []
            for b in range(B):
                rows = np.concatenate([np.arange(ns), ns + ids_l[b], ns + nv + np.arange(nx)])
                o, m = prefill_attention(Q[b:b + 1][:, :, rows], K[b:b + 1][:, :, rows],
                                         V[b:b + 1][:, :, rows], ns, len(ids_l[b]),
                                         self.window, self.scale)
                out_l.append(o[0]); mass_l.append(m[0])
                Kc.append(None if l in self.lazy else self._into_cache(K[b][:, rows], self.k_scale, b))
                Vc.append(self._into_cache(V[b][:, rows], self.v_scale, b))
                # ranking column: the scores that last decided membership; a
                # layer that precedes every prune event ranks by its own mass
                rho_l.append(m[0].copy() if inherited[b] is None else inherited[b].copy())
            self.ids.append(ids_l); self.rho.append(rho_l)
            self.K.append(Kc); self.V.append(Vc)
            res["out"].append(out_l); res["mass"].append(mass_l)
            res["ids"].append([x.copy() for x in ids_l]); res["selected"].append(sel_l)
            prev_ids, prev_mass = ids_l, mass_l
        return res

    # -- one decode step ----------------------------------------------------
    def decode_step(self, qkv_of_layer) -> Dict[str, list]:
        """qkv_of_layer(l) -> (q, k, v) each [B, H, d] for the token of step t+1."""
        self.t += 1
        t = self.t
        ns = self.n_sys
        res = {"out": [], "mass": [], "ids": [], "kv_len": []}
        src_q = {}
        for l in range(self.L):
            q, k, v = (np.asarray(x, F64) for x in qkv_of_layer(l))
            src = self.lazy.get(l)
            if src is not None:
                q = src_q[src]                        # Eq. 6: the source layer's query ...
            elif l in self.lazy.values():
                src_q[l] = q
            B = q.shape[0]
            k_lt = int(self.keep[l, t])
            out_l, mass_l, len_l = [], [], []
            for b in range(B):
                ids, rho = self.ids[l][b], self.rho[l][b]
                nv = len(ids)
                if k_lt < nv:                  # Eq. 7: evict before this layer's attention
                    pos = select_topk(rho, ids, k_lt)
                    rows = np.concatenate([np.arange(ns), ns + pos,
                                           np.arange(ns + nv, self.V[l][b].shape[1])])
                    if src is None:
                        self.K[l][b] = self.K[l][b][:, rows]
                    self.V[l][b] = self.V[l][b][:, rows]
                    self.ids[l][b] = ids = ids[pos]
                    self.rho[l][b] = rho = rho[pos]
                if src is None:
                    self.K[l][b] = np.concatenate([self.K[l][b], self._into_cache(k[b][:, None, :], self.k_scale, b)],
                                                  axis=1)
                self.V[l][b] = np.concatenate([self.V[l][b], self._into_cache(v[b][:, None, :], self.v_scale, b)], axis=1)
                # ... and keys (its cache holds the same rows in the same order), this layer's values
                Kb = self.K[l][b] if src is None else self.K[src][b]
                o, m, _ = decode_attention(q[b:b + 1], Kb[None], self.V[l][b][None],
                                           ns, len(ids), self.scale)
                out_l.append(o[0]); mass_l.append(m[0]); len_l.append(self.V[l][b].shape[1])
                if self.mode == "current":
                    self.rho[l][b] = m[0].copy()
            res["out"].append(out_l); res["mass"].append(mass_l)
            res["ids"].append([x.copy() for x in self.ids[l]]); res["kv_len"].append(len_l)
        return res

    def cache_lens(self) -> List[int]:
        return [self.V[l][0].shape[1] for l in range(self.L)]
