"""Call sequencing of Alg. 3 (PVTP at prefill, VTA at decode) over the C-ABI.

This module owns torch buffers (KV caches, score/id columns, lengths, workspace)
and issues the library calls in the paper's order.  It computes nothing itself:
attention, mass, ranking, compaction, eviction and append all run in libst3's
kernels; the only torch operations are allocations and device-to-device copies
that place a layer's inputs where the kernels expect them.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import torch

from . import binding as st3


def keep_table_for(workload) -> List[List[int]]:
    """keep[l][t] from a workload's schedule parameters, via the library's host helpers."""
    ls, ss = workload.layer_schedule, workload.step_schedule
    L, nv, T = workload.layers, workload.n_vis, workload.steps
    if ls["kind"] == "table":
        keep0 = list(ls["keep"])
    elif ls["kind"] == "linear":
        keep0 = st3.st3_schedule_linear(L, nv, ls["last_full_layer"], ls["end_ratio_bp"])
    elif ls["kind"] == "pvtp":
        keep0 = st3.st3_schedule_pvtp(L, nv, 3, ls["S"], ls["P_bp"], ls["R_bp"])
    elif ls["kind"] == "full":
        keep0 = [nv] * L
    else:
        raise ValueError(ls["kind"])
    kinds = {"cos": (st3.ST3_ANNEAL_COS, "tau"), "linear": (st3.ST3_ANNEAL_LINEAR, "tau"),
             "exp": (st3.ST3_ANNEAL_EXP, "sigma"), "drop": (st3.ST3_ANNEAL_DROP, "per_step"),
             "none": (st3.ST3_ANNEAL_NONE, None)}
    kind, pname = kinds[ss["kind"]]
    return st3.st3_schedule_anneal(kind, ss[pname] if pname else 1.0, T, keep0)


class LayerCache:
    def __init__(self, B, H, d, cap, cap_v, dtype, device, ws_bytes, value_only=False, kv_scale=None):
        # a lazy layer (QK heredity) never forms K, so it caches V alone.
        # kv_scale: None = rows of `dtype`; a float = E4M3 codes worth that much per unit, every strip
        cdt = dtype if kv_scale is None else torch.uint8
        self.k = None if value_only else torch.empty((B, H, cap, d), dtype=cdt, device=device)
        self.v = torch.empty((B, H, cap, d), dtype=cdt, device=device)
        self.k_scale = self.v_scale = None
        if kv_scale is not None:
            self.k_scale = None if value_only else torch.full((B, H), kv_scale, dtype=torch.float32, device=device)
            self.v_scale = torch.full((B, H), kv_scale, dtype=torch.float32, device=device)
        self.score = torch.zeros((B, max(cap_v, 1)), dtype=torch.float32, device=device)
        self.ids = torch.zeros((B, max(cap_v, 1)), dtype=torch.int32, device=device)
        self.mass = torch.zeros((B, max(cap_v, 1)), dtype=torch.float32, device=device)
        self.vis_len = torch.zeros((B,), dtype=torch.int32, device=device)
        self.kv_len = torch.zeros((B,), dtype=torch.int32, device=device)
        self.tail_start = None      # set at prefill when the tail keeps its place (Generation(fixed_tail=True))
        self.h_tail = 0             # host copy of it
        self.kv = st3.kv_layer(self.k, self.v, self.k_scale, self.v_scale)
        # a workspace of its own: the attention leaves its logits here for the mass and for lazy layers
        self.ws = torch.empty((ws_bytes,), dtype=torch.uint8, device=device)
        # host-side bounds (exact here, since every sequence follows the same table)
        self.h_vis = 0
        self.h_kv = 0


class Generation:
    """One batch of sequences going through prefill and decode steps.

    keep: table keep[l][t] (t = 0 .. steps).  mode: "static" ranks by the column
    fixed at prefill, "current" by the layer's latest decode mass.
    lazy: {l: src} - QK heredity (Eq. 6, Alg. 2): layer l applies the attention probabilities of
    source layer src to its own values, at prefill and at every decode step.  Lazy layers follow
    their source directly and share its row of the keep table; their Q and K inputs are ignored.
    fixed_tail: the rows behind a layer's visual segment (instruction + generated tokens) stay where
    the prefill put them while the segment shrinks: an eviction then moves at most one row per evicted
    row instead of two (no closing up of the tail); False keeps every cache contiguous.
    kv_scale: None keeps the caches in `dtype`; a float makes them FP8 E4M3 (bf16 only) with that
    scale for every (b, h) strip of K and of V - the caller's calibration, e.g. 6 sigma / 448.
    """

    def __init__(self, layers: int, heads: int, head_dim: int, dtype: torch.dtype, batch: int,
                 n_sys: int, n_vis: int, n_txt: int, steps: int, keep: Sequence[Sequence[int]],
                 window: int = 1, mode: str = "static", compact_mode: int = st3.ST3_HOLE_FILL,
                 device: str = "cuda:0", lazy: Optional[Dict[int, int]] = None, kv_scale: Optional[float] = None,
                 fixed_tail: bool = True):
        self.L, self.H, self.d, self.B = layers, heads, head_dim, batch
        self.n_sys, self.n_vis, self.n_txt, self.T = n_sys, n_vis, n_txt, steps
        self.keep = [list(r) for r in keep]
        self.window, self.mode, self.compact_mode = window, mode, compact_mode
        self.dtype, self.device = dtype, device
        self.shape = st3.make_shape(batch, heads, head_dim, st3._dtype_code(torch.empty(0, dtype=dtype)))
        self.N0 = n_sys + n_vis + n_txt
        self.lazy = dict(lazy or {})
        for l, src in self.lazy.items():
            if not (0 <= src < l < layers) or src in self.lazy:
                raise ValueError("a lazy layer needs a non-lazy source layer before it")
            if any(self.lazy.get(m) != src for m in range(src + 1, l)):
                raise ValueError("lazy layers must follow their source directly")
            if self.keep[l] != self.keep[src]:
                raise ValueError("a lazy layer keeps what its source keeps")
        self.layers: List[LayerCache] = []
        for l in range(layers):
            cap = n_sys + self.keep[l][0] + n_txt + steps
            cap = max(cap, self.N0)                 # the unpruned prompt is staged in the cache first
            ws_bytes = st3.st3_workspace_bytes(self.shape, cap, n_vis, window)
            self.layers.append(LayerCache(batch, heads, head_dim, cap, n_vis, dtype, device, ws_bytes,
                                          value_only=l in self.lazy, kv_scale=kv_scale))
            st3.st3_workspace_init(self.shape, cap, self.layers[-1].ws)
        self.kv_scale = kv_scale
        self.fixed_tail = fixed_tail
        self.q_stage = torch.empty((batch, heads, self.N0, head_dim), dtype=dtype, device=device)
        # an E4M3 cache cannot serve as the prefill's K/V input: the prompt is attended unquantised
        # from staging buffers and its rows enter the cache through the quantiser afterwards
        self.k_stage = self.v_stage = None
        if kv_scale is not None:
            self.k_stage = torch.empty((batch, heads, self.N0, head_dim), dtype=dtype, device=device)
            self.v_stage = torch.empty((batch, heads, self.N0, head_dim), dtype=dtype, device=device)
        self.out_stage = torch.empty((batch, heads, self.N0, head_dim), dtype=dtype, device=device)
        self.dec_out = torch.empty((batch, heads, head_dim), dtype=dtype, device=device)
        self.dec_out_all = torch.empty((layers, batch, heads, head_dim), dtype=dtype, device=device)
        self._steps = None                  # ctypes array of LayerStep, built on first decode_step()
        self.keep_idx = torch.empty((batch, max(n_vis, 1)), dtype=torch.int32, device=device)
        self._alive = n_vis                 # visual tokens alive in the layer being prefetched
        self._inherit: Optional[torch.Tensor] = None
        self.t = 0
        eb = 2 if dtype == torch.bfloat16 else 4
        self._eb = eb

    # ------------------------------------------------------------------------------------
    def _compact_column(self, col: torch.Tensor, idx: torch.Tensor, k: int, n: int):
        st3.st3_compact_rows(col.data_ptr(), self.B, 1, col.stride(0) * 4, 0, 4, 4, idx, k, n, 0)

    def prefill_layer(self, l: int, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor):
        """Q, K, V: device tensors [B,H,N0,d] over the unpruned prompt (Alg. 3, PVTP branch).
        A lazy layer ignores Q and K (may be None): Eq. 6 attends with its source's.

        Returns (out view [B,H,n_l,d], mass view [B,keep_l]).
        """
        lc = self.layers[l]
        src = self.lazy.get(l)
        B, ns, nv, nx = self.B, self.n_sys, self.n_vis, self.n_txt
        k_l = self.keep[l][0]
        if l == 0:                  # a new job: nothing is inherited from the previous one
            self._alive = nv
            self._inherit = None
            self._decoding = False
            lc.ids[:, :nv] = torch.arange(nv, dtype=torch.int32, device=self.device)
        else:
            prev = self.layers[l - 1]
            lc.ids.copy_(prev.ids)
            if k_l < self._alive:
                # Eq. 3: keep the k_l visual tokens the PREVIOUS layer's last row attended to most
                st3.st3_select_topk(prev.mass, prev.ids, None, self._alive, k_l, None, self.keep_idx)
                self._compact_column(lc.ids, self.keep_idx, k_l, self._alive)
                if self._inherit is None:
                    self._inherit = torch.empty_like(prev.mass)
                self._inherit.copy_(prev.mass)
                self._compact_column(self._inherit, self.keep_idx, k_l, self._alive)
                self._alive = k_l
        alive = self._alive
        n_l = ns + alive + nx
        # stage the layer's inputs, K and V straight into the cache and Q into scratch, in ONE gather
        # launch (Alg. 1/3: X = [S, V[T], I]; ids are the ascending original positions of the survivors)
        fp8 = self.kv_scale is not None
        k_dst, v_dst = (self.k_stage, self.v_stage) if fp8 else (lc.k, lc.v)
        if src is None:
            pairs = [(Q, self.q_stage), (K, k_dst), (V, v_dst)]
            k_rows = k_dst
        else:
            # Self-attn(Q^src, K^src, V^l): the source's compacted queries are still staged (only
            # lazy layers came in between) and its keys are the first n_l rows of its cache (of the
            # key staging buffer when the caches are E4M3)
            pairs = [(V, v_dst)]
            k_rows = self.k_stage if fp8 else self.layers[src].k
        st3.st3_gather_rows(pairs, ns, lc.ids if alive < nv else None, alive, nv, nx)
        out = self.out_stage[:, :, :n_l]
        st3.st3_prefill_attention(self.shape, self.q_stage[:, :, :n_l], k_rows[:, :, :n_l], v_dst[:, :, :n_l],
                                  n_l, ns, alive, self.window, out, lc.mass, lc.ws)
        if fp8:
            if src is None:
                st3.st3_quantize_rows(self.shape, self.k_stage, lc.kv, 0, n_l)
            st3.st3_quantize_rows(self.shape, self.v_stage, lc.kv, 1, n_l)
        # ranking column: scores of the most recent prune event, else the layer's own mass
        lc.score.copy_(lc.mass if self._inherit is None else self._inherit)
        lc.vis_len.fill_(alive)
        lc.kv_len.fill_(n_l)
        lc.h_vis, lc.h_kv = alive, n_l
        if self.fixed_tail:         # [system | kept visual | instruction] is contiguous now: the tail starts here for good
            if lc.tail_start is None:
                lc.tail_start = torch.empty((self.B,), dtype=torch.int32, device=self.device)
            lc.h_tail = ns + alive
            lc.tail_start.fill_(lc.h_tail)
        self._decoding = False
        return out, lc.mass[:, :alive]

    # ------------------------------------------------------------------------------------
    def begin_decode(self):
        """The eviction that precedes the FIRST decode step (Alg. 3 truncates a layer's cache before
        its attention at every step; later steps do it right after the previous step's attention)."""
        for l, lc in enumerate(self.layers):
            target = min(self.keep[l][1], lc.h_vis) if self.T >= 1 else lc.h_vis
            if target < lc.h_vis:
                seg = st3.segments(self.n_sys, lc.h_vis, lc.h_kv, lc.vis_len, lc.kv_len, lc.tail_start)
                st3.st3_select_compact_layer(self.shape, lc.kv, seg, lc.score, lc.ids, target, self.compact_mode,
                                             lc.ws)
                if not self.fixed_tail:
                    lc.h_kv -= lc.h_vis - target
                lc.h_vis = target
        self._decoding = True

    def _keep_after(self, l: int, t: int) -> int:
        """Visual rows layer l holds after step t's attention = what step t+1 attends over."""
        lc = self.layers[l]
        return min(self.keep[l][t + 1], lc.h_vis) if t + 1 <= self.T else lc.h_vis

    def _mass_dst(self, lc: LayerCache) -> torch.Tensor:
        return lc.score if self.mode == "current" else lc.mass

    def decode_layer(self, l: int, t: int, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor):
        """q, k_new, v_new: device [B,H,d].  Alg. 3, VTA branch, layer l of step t >= 1: append, attend,
        then evict down to what step t+1 keeps.

        Returns (out [B,H,d] (reused buffer), mass view [B, keep[l][t]] in the cache order the
        attention saw; in "current" mode the mass lives in the score column, which the eviction
        compacts, so only its first keep[l][t+1] entries (the survivors) remain meaningful).
        """
        if self.lazy:
            raise RuntimeError("QK heredity needs the whole-step call: a group's evictions wait for its last lazy "
                               "layer, use decode_step()")
        if not getattr(self, "_decoding", False):
            self.begin_decode()
        lc = self.layers[l]
        n_attn = lc.h_vis
        target = self._keep_after(l, t)
        seg = st3.segments(self.n_sys, lc.h_vis, lc.h_kv, lc.vis_len, lc.kv_len, lc.tail_start, lc.h_vis, lc.h_tail)
        mass_dst = self._mass_dst(lc)
        st3.st3_decode_layer_step(self.shape, lc.kv, seg, lc.score, lc.ids, target if target < lc.h_vis else -1,
                                  self.compact_mode, q, k_new, v_new, self.dec_out, mass_dst, lc.ws)
        lc.h_kv = lc.h_kv + 1 - (0 if self.fixed_tail else lc.h_vis - target)
        lc.h_vis = target
        return self.dec_out, mass_dst[:, :n_attn]

    def _step_array(self):
        if self._steps is None:
            arr = (st3.LayerStep * self.L)()
            for l, lc in enumerate(self.layers):
                s = arr[l]
                s.kv = lc.kv
                s.seg = st3.segments(self.n_sys, 0, 0, lc.vis_len, lc.kv_len, lc.tail_start)
                s.score_col, s.id_col, s.col_stride = lc.score.data_ptr(), lc.ids.data_ptr(), lc.score.stride(0)
                md = self._mass_dst(lc)
                s.vis_mass, s.mass_stride = md.data_ptr(), md.stride(0)
                s.out = self.dec_out_all[l].data_ptr()
                s.workspace, s.workspace_bytes = lc.ws.data_ptr(), lc.ws.numel()
                s.inherit_from = self.lazy.get(l, -1)
            self._steps = arr
        return self._steps

    def _set_step_bounds(self, t: int):
        """Per-step scalars of every entry: what each layer keeps after this step's attention and the
        host-side bounds of its lengths before it."""
        arr = self._step_array()
        for l, lc in enumerate(self.layers):
            s = arr[l]
            target = self._keep_after(l, t)
            s.keep_after = target if target < lc.h_vis else -1
            s.seg.max_vis_len, s.seg.max_kv_len = lc.h_vis, lc.h_kv
            s.seg.vis_len_hint, s.seg.tail_start_hint = lc.h_vis, lc.h_tail     # every sequence holds these (equal images)
        return arr

    def _advance_host_lengths(self, t: int):
        for l, lc in enumerate(self.layers):
            target = self._keep_after(l, t)
            lc.h_kv = lc.h_kv + 1 - (0 if self.fixed_tail else lc.h_vis - target)
            lc.h_vis = target

    def decode_step(self, t: int, qkv: torch.Tensor):
        """All layers of decode step t from one library call.  qkv: device [L, 3, B, H, d]
        (q, k_new, v_new per layer).  Returns dec_out_all [L, B, H, d] (reused buffer)."""
        assert qkv.is_contiguous() and tuple(qkv.shape) == (self.L, 3, self.B, self.H, self.d)
        if not getattr(self, "_decoding", False):
            self.begin_decode()
        arr = self._set_step_bounds(t)
        base = qkv.data_ptr()
        one = self.B * self.H * self.d * self._eb
        for l in range(self.L):
            s = arr[l]
            s.q, s.k_new, s.v_new = base + (3 * l) * one, base + (3 * l + 1) * one, base + (3 * l + 2) * one
        self._advance_host_lengths(t)
        st3.st3_decode_step(self.shape, arr, self.L, self.compact_mode)
        return self.dec_out_all

    # -- the same step as a decoder with a dependency between its layers calls it --------------------
    def begin_step(self, t: int):
        """Opens decode step t for attend_layer() calls (Alg. 3, VTA branch, the loop over l)."""
        if not getattr(self, "_decoding", False):
            self.begin_decode()
        self._set_step_bounds(t)
        self._open_step = t
        self._step_stream = torch.cuda.current_stream().cuda_stream    # looked up once per step, not once per layer
        if getattr(self, "_out_views", None) is None:
            self._out_views = [self.dec_out_all[l] for l in range(self.L)]

    def attend_layer(self, l: int, q, k_new, v_new):
        """Layer l of the open step: append k_new/v_new and attend.  q, k_new, v_new: device [B,H,d] tensors or
        their device addresses, alive until the stream has run the call (a lazy layer ignores q and k_new, which
        may be None).  Returns out [B,H,d], complete once the stream has run the call - before any later layer's
        inputs need to exist."""
        arr = self._steps
        s = arr[l]
        v_ptr = v_new if isinstance(v_new, int) else v_new.data_ptr()
        s.q = v_ptr if q is None else (q if isinstance(q, int) else q.data_ptr())
        s.k_new = v_ptr if k_new is None else (k_new if isinstance(k_new, int) else k_new.data_ptr())
        s.v_new = v_ptr
        st3.st3_decode_layer_attend(self.shape, arr, self.L, l, self.compact_mode, self._step_stream)
        return self._out_views[l]

    def finish_step(self):
        """Closes the open step: masses, appended rows counted, evictions of every layer."""
        t = self._open_step
        st3.st3_decode_plans(self.shape, self._steps, self.L, self.compact_mode, self._step_stream)
        self._advance_host_lengths(t)
        self._open_step = None

    def kv_lens(self) -> List[int]:
        """Keys each layer holds (dead rows between a visual segment and a fixed tail do not count)."""
        if not self.fixed_tail:
            return [lc.h_kv for lc in self.layers]
        return [lc.h_kv - (lc.h_tail - self.n_sys - lc.h_vis) for lc in self.layers]

    def kv_bytes(self) -> int:
        lens = self.kv_lens()
        full = [n for l, n in enumerate(lens) if l not in self.lazy]
        half = [n for l, n in enumerate(lens) if l in self.lazy]          # V only
        edt = self.shape.dtype if self.kv_scale is None else st3.ST3_E4M3
        total = st3.st3_kv_bytes(self.B, self.H, self.d, edt, full)
        if half:
            total += st3.st3_kv_bytes(self.B, self.H, self.d, edt, half) // 2
        return total
