"""ctypes binding of libst3.so: same names as include/st3.h, argument marshalling only.

PyTorch supplies device memory (`tensor.data_ptr()`) and the stream handle; every
step of the path runs inside the library's HIP kernels.  There is no fallback: if
the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libst3.so")

ST3_OK = 0
ST3_ERR_INVALID_ARG = 1
ST3_ERR_UNSUPPORTED = 2
ST3_ERR_WORKSPACE_TOO_SMALL = 3
ST3_ERR_HIP = 4
ST3_F32, ST3_BF16, ST3_E4M3 = 0, 1, 2
ST3_KV_PLAIN, ST3_KV_E4M3 = 0, 1
ST3_STABLE, ST3_HOLE_FILL = 0, 1
ST3_ANNEAL_COS, ST3_ANNEAL_LINEAR, ST3_ANNEAL_EXP, ST3_ANNEAL_DROP, ST3_ANNEAL_NONE = 0, 1, 2, 3, 4

EXPORTED = [
    "st3_status_string", "st3_last_hip_error", "st3_version", "st3_workspace_bytes", "st3_workspace_init",
    "st3_prefill_attention", "st3_quantize_rows", "st3_kv_append", "st3_decode_attention", "st3_decode_attention_inherit",
    "st3_decode_attention_noalloc", "st3_select_topk",
    "st3_compact_rows", "st3_gather_rows", "st3_select_compact_layer", "st3_decode_layer_step", "st3_decode_step",
    "st3_decode_layer_attend", "st3_decode_plans",
    "st3_schedule_pvtp", "st3_schedule_linear", "st3_schedule_anneal", "st3_kv_bytes",
    "st3_debug_enabled", "st3_debug_set_prefill_path", "st3_debug_set_attend_tile", "st3_profile_enable", "st3_profile_read", "st3_overlap_topk",
    "st3_cosine_similarity",
]


class St3Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().st3_status_string(status).decode()
        if status == ST3_ERR_HIP:
            msg += f" (hipError_t {lib().st3_last_hip_error()})"
        super().__init__(f"{where}: {msg}")


class AttnShape(C.Structure):
    _fields_ = [("batch", C.c_int32), ("heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("softmax_scale", C.c_float)]


class Tensor4(C.Structure):
    _fields_ = [("data", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64),
                ("stride_t", C.c_int64)]


class KvLayer(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("stride_b", C.c_int64),
                ("stride_h", C.c_int64), ("stride_t", C.c_int64), ("capacity", C.c_int32), ("format", C.c_int32),
                ("k_scale", C.c_void_p), ("v_scale", C.c_void_p)]


class Segments(C.Structure):
    _fields_ = [("sys_len", C.c_int32), ("max_vis_len", C.c_int32), ("max_kv_len", C.c_int32),
                ("vis_len", C.c_void_p), ("kv_len", C.c_void_p), ("tail_start", C.c_void_p),
                ("vis_len_hint", C.c_int32), ("tail_start_hint", C.c_int32)]


class GatherPair(C.Structure):
    _fields_ = [("src", C.c_void_p), ("src_stride_b", C.c_int64), ("src_stride_inner", C.c_int64),
                ("src_stride_row", C.c_int64), ("dst", C.c_void_p), ("dst_stride_b", C.c_int64),
                ("dst_stride_inner", C.c_int64), ("dst_stride_row", C.c_int64)]


ST3_MAX_GATHER = 4
ST3_NOALLOC_SCRATCH_BYTES = 32 << 20


class LayerStep(C.Structure):
    _fields_ = [("kv", KvLayer), ("seg", Segments), ("score_col", C.c_void_p), ("id_col", C.c_void_p),
                ("col_stride", C.c_int64), ("keep_after", C.c_int32), ("inherit_from", C.c_int32), ("q", C.c_void_p),
                ("k_new", C.c_void_p),
                ("v_new", C.c_void_p), ("out", C.c_void_p), ("vis_mass", C.c_void_p), ("mass_stride", C.c_int64),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
                "There is no CPU fallback.")
        L = C.CDLL(LIB_PATH)
        L.st3_status_string.restype = C.c_char_p
        L.st3_status_string.argtypes = [C.c_int]
        L.st3_last_hip_error.restype = C.c_int
        L.st3_version.restype = C.c_uint32
        L.st3_workspace_bytes.restype = C.c_size_t
        L.st3_workspace_bytes.argtypes = [C.POINTER(AttnShape), C.c_int32, C.c_int32, C.c_int32]
        P = C.POINTER
        L.st3_workspace_init.argtypes = [P(AttnShape), C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.st3_workspace_init.restype = C.c_int
        L.st3_prefill_attention.argtypes = [P(AttnShape), P(Tensor4), P(Tensor4), P(Tensor4), C.c_int32, C.c_int32,
                                            C.c_int32, C.c_int32, P(Tensor4), C.c_void_p, C.c_int64, C.c_void_p,
                                            C.c_size_t, C.c_void_p]
        L.st3_quantize_rows.argtypes = [P(AttnShape), P(Tensor4), P(KvLayer), C.c_int32, C.c_int32, C.c_void_p]
        L.st3_quantize_rows.restype = C.c_int
        L.st3_kv_append.argtypes = [P(AttnShape), P(KvLayer), P(Segments), C.c_void_p, C.c_void_p, C.c_void_p]
        L.st3_decode_attention.argtypes = [P(AttnShape), C.c_void_p, P(KvLayer), P(Segments), C.c_void_p, C.c_void_p,
                                           C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
        L.st3_decode_attention_inherit.argtypes = [P(AttnShape), P(KvLayer), P(Segments), C.c_void_p, C.c_size_t,
                                                   C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.st3_decode_attention_inherit.restype = C.c_int
        L.st3_decode_attention_noalloc.argtypes = [P(AttnShape), C.c_void_p, P(KvLayer), P(Segments), C.c_void_p,
                                                   C.c_void_p, C.c_int64, C.c_void_p]
        L.st3_decode_attention_noalloc.restype = C.c_int
        L.st3_select_topk.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32,
                                      C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.st3_compact_rows.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int64, C.c_int32,
                                       C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.st3_gather_rows.argtypes = [P(GatherPair), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                      C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.st3_gather_rows.restype = C.c_int
        L.st3_select_compact_layer.argtypes = [P(AttnShape), P(KvLayer), P(Segments), C.c_void_p, C.c_void_p,
                                               C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.st3_decode_layer_step.argtypes = [P(AttnShape), P(KvLayer), P(Segments), C.c_void_p, C.c_void_p, C.c_int64,
                                            C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
        L.st3_decode_step.argtypes = [P(AttnShape), C.c_int32, P(LayerStep), C.c_int32, C.c_void_p]
        L.st3_decode_step.restype = C.c_int
        L.st3_decode_layer_attend.argtypes = [P(AttnShape), C.c_int32, P(LayerStep), C.c_int32, C.c_int32, C.c_void_p]
        L.st3_decode_layer_attend.restype = C.c_int
        L.st3_decode_plans.argtypes = [P(AttnShape), C.c_int32, P(LayerStep), C.c_int32, C.c_void_p]
        L.st3_decode_plans.restype = C.c_int
        L.st3_schedule_pvtp.argtypes = [C.c_int32] * 6 + [C.c_void_p]
        L.st3_schedule_linear.argtypes = [C.c_int32] * 4 + [C.c_void_p]
        L.st3_schedule_anneal.argtypes = [C.c_int32, C.c_double, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p]
        L.st3_kv_bytes.restype = C.c_int64
        L.st3_kv_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_int32]
        for name in ("st3_prefill_attention", "st3_quantize_rows", "st3_kv_append", "st3_decode_attention", "st3_decode_attention_inherit",
    "st3_select_topk",
                     "st3_compact_rows", "st3_select_compact_layer", "st3_decode_layer_step",
                     "st3_schedule_pvtp", "st3_schedule_linear", "st3_schedule_anneal"):
            getattr(L, name).restype = C.c_int
        L.st3_overlap_topk.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p]
        L.st3_overlap_topk.restype = C.c_int
        L.st3_cosine_similarity.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p,
                                            C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_void_p]
        L.st3_cosine_similarity.restype = C.c_int
        L.st3_profile_enable.argtypes = [C.c_int32]
        L.st3_profile_enable.restype = C.c_int
        L.st3_profile_read.argtypes = [P(C.c_double), P(C.c_int64), P(C.c_double), P(C.c_double)]
        L.st3_profile_read.restype = C.c_int
        L.st3_debug_set_prefill_path.argtypes = [C.c_int]
        L.st3_debug_set_prefill_path.restype = C.c_int
        L.st3_debug_set_attend_tile.argtypes = [C.c_int]
        L.st3_debug_set_attend_tile.restype = C.c_int
        L.st3_debug_enabled.restype = C.c_int
        _lib = L
    return _lib


# ---------------------------------------------------------------------------
# marshalling helpers
# ---------------------------------------------------------------------------
def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return ST3_F32
    if t.dtype == torch.bfloat16:
        return ST3_BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def make_shape(batch: int, heads: int, head_dim: int, dtype: int, softmax_scale: float = 0.0) -> AttnShape:
    return AttnShape(batch, heads, head_dim, dtype, softmax_scale)


def tensor4(t: torch.Tensor) -> Tensor4:
    assert t.dim() == 4 and t.stride(3) == 1 and t.is_cuda
    s = Tensor4(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))
    s._refs = (t,)          # the struct holds raw addresses: keep the tensor alive with it
    return s


def kv_layer(k: Optional[torch.Tensor], v: torch.Tensor, k_scale: Optional[torch.Tensor] = None,
             v_scale: Optional[torch.Tensor] = None) -> KvLayer:
    """k is None for a layer that caches values only (lazy layer of QK heredity).  uint8 tensors are
    E4M3 caches and come with float32 scales [B, H] (k_scale may be None when k is)."""
    assert v.dim() == 4 and v.stride(3) == 1 and v.is_cuda
    assert k is None or (k.stride() == v.stride() and k.shape == v.shape and k.is_cuda and k.dtype == v.dtype)
    fmt = ST3_KV_E4M3 if v.dtype == torch.uint8 else ST3_KV_PLAIN
    if fmt == ST3_KV_E4M3:
        for sc in (k_scale, v_scale):
            assert sc is None or (sc.dtype == torch.float32 and sc.is_contiguous() and sc.is_cuda)
        assert v_scale is not None and (k is None or k_scale is not None)
    s = KvLayer(None if k is None else k.data_ptr(), v.data_ptr(), v.stride(0), v.stride(1), v.stride(2), v.shape[2], fmt,
                _ptr(k_scale) if fmt else None, _ptr(v_scale) if fmt else None)
    s._refs = (k, v, k_scale, v_scale)
    return s


def segments(sys_len: int, max_vis_len: int, max_kv_len: int, vis_len: torch.Tensor, kv_len: torch.Tensor,
             tail_start: Optional[torch.Tensor] = None, vis_len_hint: int = 0, tail_start_hint: int = 0) -> Segments:
    assert vis_len.dtype == torch.int32 and kv_len.dtype == torch.int32 and vis_len.is_cuda and kv_len.is_cuda
    assert tail_start is None or (tail_start.dtype == torch.int32 and tail_start.is_cuda)
    s = Segments(sys_len, max_vis_len, max_kv_len, vis_len.data_ptr(), kv_len.data_ptr(), _ptr(tail_start),
                 vis_len_hint, tail_start_hint)
    s._refs = (vis_len, kv_len, tail_start)
    return s


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _check(status: int, where: str) -> None:
    if status != ST3_OK:
        raise St3Error(status, where)


# ---------------------------------------------------------------------------
# the calls of st3.h
# ---------------------------------------------------------------------------
def st3_version() -> int:
    return lib().st3_version()


def st3_workspace_bytes(shape: AttnShape, kv_capacity: int, max_vis_len: int, score_window: int = 1) -> int:
    return lib().st3_workspace_bytes(C.byref(shape), kv_capacity, max_vis_len, score_window)


def st3_workspace_init(shape: AttnShape, kv_capacity: int, workspace, stream=None) -> None:
    _check(lib().st3_workspace_init(C.byref(shape), kv_capacity, workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _stream(stream)),
           "st3_workspace_init")


def st3_prefill_attention(shape, q, k, v, n, sys_len, vis_len, score_window, out, vis_mass, workspace, stream=None):
    tq, tk, tv, to = tensor4(q), tensor4(k), tensor4(v), tensor4(out)
    ms = 0 if vis_mass is None else vis_mass.stride(0)
    _check(lib().st3_prefill_attention(C.byref(shape), C.byref(tq), C.byref(tk), C.byref(tv), n, sys_len, vis_len,
                                       score_window, C.byref(to), _ptr(vis_mass), ms, _ptr(workspace),
                                       0 if workspace is None else workspace.numel() * workspace.element_size(),
                                       _stream(stream)), "st3_prefill_attention")


def st3_quantize_rows(shape, src, kv: KvLayer, which: int, n: int, stream=None):
    _check(lib().st3_quantize_rows(C.byref(shape), C.byref(tensor4(src)), C.byref(kv), which, n, _stream(stream)),
           "st3_quantize_rows")


def st3_kv_append(shape, kv: KvLayer, seg: Segments, k_new, v_new, stream=None):
    _check(lib().st3_kv_append(C.byref(shape), C.byref(kv), C.byref(seg), _ptr(k_new), v_new.data_ptr(),
                               _stream(stream)), "st3_kv_append")


def st3_decode_attention(shape, q, kv: KvLayer, seg: Segments, out, vis_mass, workspace, stream=None):
    ms = 0 if vis_mass is None else vis_mass.stride(0)
    _check(lib().st3_decode_attention(C.byref(shape), q.data_ptr(), C.byref(kv), C.byref(seg), out.data_ptr(),
                                      _ptr(vis_mass), ms, workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), _stream(stream)),
           "st3_decode_attention")


def st3_decode_attention_noalloc(shape, q, kv: KvLayer, seg: Segments, out, vis_mass, stream=None):
    ms = 0 if vis_mass is None else vis_mass.stride(0)
    _check(lib().st3_decode_attention_noalloc(C.byref(shape), q.data_ptr(), C.byref(kv), C.byref(seg), out.data_ptr(),
                                              _ptr(vis_mass), ms, _stream(stream)), "st3_decode_attention_noalloc")


def st3_decode_attention_inherit(shape, kv: KvLayer, seg: Segments, src_workspace, src_kv_capacity, out, workspace,
                                 stream=None):
    _check(lib().st3_decode_attention_inherit(C.byref(shape), C.byref(kv), C.byref(seg), src_workspace.data_ptr(),
                                              src_workspace.numel() * src_workspace.element_size(), src_kv_capacity,
                                              out.data_ptr(), workspace.data_ptr(),
                                              workspace.numel() * workspace.element_size(), _stream(stream)),
           "st3_decode_attention_inherit")


def st3_select_topk(scores, tie_ids, n_dev, n, k, keep_mask, keep_idx, stream=None):
    assert scores.dtype == torch.float32 and scores.dim() == 2
    _check(lib().st3_select_topk(scores.data_ptr(), scores.stride(0), _ptr(tie_ids),
                                 0 if tie_ids is None else tie_ids.stride(0), scores.shape[0], _ptr(n_dev), n, k,
                                 _ptr(keep_mask), _ptr(keep_idx), 0 if keep_idx is None else keep_idx.stride(0),
                                 _stream(stream)), "st3_select_topk")


def st3_compact_rows(rows_ptr: int, batch, inner, stride_b_bytes, stride_inner_bytes, stride_row_bytes, row_bytes,
                     keep_idx, k, n, tail_rows, stream=None):
    _check(lib().st3_compact_rows(rows_ptr, batch, inner, stride_b_bytes, stride_inner_bytes, stride_row_bytes,
                                  row_bytes, keep_idx.data_ptr(), keep_idx.stride(0), k, n, tail_rows,
                                  _stream(stream)),
           "st3_compact_rows")


def st3_gather_rows(pairs, head_rows, keep_idx, k, n, tail_rows, stream=None):
    """pairs: list of (src, dst) tensors [B, inner, rows, width] with contiguous rows of equal byte length."""
    src0 = pairs[0][0]
    eb = src0.element_size()
    arr = (GatherPair * len(pairs))()
    for g, (src, dst) in zip(arr, pairs):
        assert src.dim() == 4 and dst.dim() == 4 and src.stride(3) == 1 and dst.stride(3) == 1
        assert src.shape[:2] == dst.shape[:2] and src.shape[3] == dst.shape[3] and src.element_size() == eb
        g.src, g.dst = src.data_ptr(), dst.data_ptr()
        g.src_stride_b, g.src_stride_inner, g.src_stride_row = (src.stride(i) * eb for i in range(3))
        g.dst_stride_b, g.dst_stride_inner, g.dst_stride_row = (dst.stride(i) * eb for i in range(3))
    ist = 0 if keep_idx is None else keep_idx.stride(0)
    _check(lib().st3_gather_rows(arr, len(pairs), src0.shape[0], src0.shape[1], src0.shape[3] * eb, head_rows,
                                 _ptr(keep_idx), ist, k, n, tail_rows, _stream(stream)), "st3_gather_rows")


def st3_select_compact_layer(shape, kv: KvLayer, seg: Segments, score_col, id_col, keep_count, mode, workspace,
                             stream=None):
    assert score_col.stride(0) == id_col.stride(0)
    _check(lib().st3_select_compact_layer(C.byref(shape), C.byref(kv), C.byref(seg), score_col.data_ptr(),
                                          id_col.data_ptr(), score_col.stride(0), keep_count, mode,
                                          workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                          _stream(stream)), "st3_select_compact_layer")


def st3_decode_layer_step(shape, kv: KvLayer, seg: Segments, score_col, id_col, keep_after, mode, q, k_new, v_new,
                          out, vis_mass, workspace, stream=None):
    ms = 0 if vis_mass is None else vis_mass.stride(0)
    cs = 0 if score_col is None else score_col.stride(0)
    _check(lib().st3_decode_layer_step(C.byref(shape), C.byref(kv), C.byref(seg), _ptr(score_col), _ptr(id_col), cs,
                                       keep_after, mode, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(),
                                       out.data_ptr(), _ptr(vis_mass), ms, workspace.data_ptr(),
                                       workspace.numel() * workspace.element_size(), _stream(stream)),
           "st3_decode_layer_step")


def st3_decode_step(shape, layer_steps, n_layers, mode, stream=None):
    """layer_steps: a ctypes array of LayerStep (the caller keeps the tensors it points to alive)."""
    _check(lib().st3_decode_step(C.byref(shape), n_layers, layer_steps, mode, _stream(stream)), "st3_decode_step")


def st3_decode_layer_attend(shape, layer_steps, n_layers, layer, mode, stream=None):
    _check(lib().st3_decode_layer_attend(C.byref(shape), n_layers, layer_steps, layer, mode, _stream(stream)),
           "st3_decode_layer_attend")


def st3_decode_plans(shape, layer_steps, n_layers, mode, stream=None):
    _check(lib().st3_decode_plans(C.byref(shape), n_layers, layer_steps, mode, _stream(stream)), "st3_decode_plans")


# -- host-only schedule helpers ---------------------------------------------------------------
def st3_schedule_pvtp(L, n_vis, first_layer, stride_S, P_bp, R_bp):
    out = (C.c_int32 * L)()
    _check(lib().st3_schedule_pvtp(L, n_vis, first_layer, stride_S, P_bp, R_bp, out), "st3_schedule_pvtp")
    return list(out)


def st3_schedule_linear(L, n_vis, last_full_layer, end_ratio_bp):
    out = (C.c_int32 * L)()
    _check(lib().st3_schedule_linear(L, n_vis, last_full_layer, end_ratio_bp, out), "st3_schedule_linear")
    return list(out)


def st3_schedule_anneal(kind, param, T, keep_l0):
    L = len(keep_l0)
    src = (C.c_int32 * L)(*keep_l0)
    out = (C.c_int32 * (L * (T + 1)))()
    _check(lib().st3_schedule_anneal(kind, float(param), T, src, L, out), "st3_schedule_anneal")
    return [list(out[l * (T + 1):(l + 1) * (T + 1)]) for l in range(L)]


def st3_kv_bytes(batch, heads, head_dim, dtype, kv_lens):
    arr = (C.c_int32 * len(kv_lens))(*kv_lens)
    return lib().st3_kv_bytes(batch, heads, head_dim, dtype, arr, len(kv_lens))


def st3_overlap_topk(score_a, ids_a, n_a, score_b, ids_b, n_b, k, id_space, overlap, topk_a, n_a_dev=None,
                     n_b_dev=None, stream=None):
    _check(lib().st3_overlap_topk(score_a.data_ptr(), ids_a.data_ptr(), score_a.stride(0), _ptr(n_a_dev), n_a,
                                  score_b.data_ptr(), ids_b.data_ptr(), score_b.stride(0), _ptr(n_b_dev), n_b,
                                  score_a.shape[0], k, id_space, overlap.data_ptr(), topk_a.data_ptr(),
                                  _stream(stream)), "st3_overlap_topk")


def st3_cosine_similarity(va, ids_a, n_a, vb, ids_b, n_b, id_space, cosine, n_a_dev=None, n_b_dev=None, stream=None):
    _check(lib().st3_cosine_similarity(va.data_ptr(), _ptr(ids_a), va.stride(0), _ptr(n_a_dev), n_a, vb.data_ptr(),
                                       _ptr(ids_b), vb.stride(0), _ptr(n_b_dev), n_b, va.shape[0], id_space,
                                       cosine.data_ptr(), _stream(stream)), "st3_cosine_similarity")


def st3_profile_enable(max_launches: int) -> None:
    _check(lib().st3_profile_enable(max_launches), "st3_profile_enable")


def st3_profile_read():
    """Returns (total_ms, launches, min_ms, max_ms) of the split-KV decode kernel since enable."""
    tot, mn, mx = C.c_double(), C.c_double(), C.c_double()
    cnt = C.c_int64()
    _check(lib().st3_profile_read(C.byref(tot), C.byref(cnt), C.byref(mn), C.byref(mx)), "st3_profile_read")
    return tot.value, cnt.value, mn.value, mx.value


def st3_debug_enabled() -> bool:
    """True when ST3_DEBUG=1 was in the environment as the library was loaded (the diagnostic block is live)."""
    return bool(lib().st3_debug_enabled())


def st3_debug_set_prefill_path(path: int) -> None:
    _check(lib().st3_debug_set_prefill_path(path), "st3_debug_set_prefill_path")


def st3_debug_set_attend_tile(tile_loads: int) -> None:
    _check(lib().st3_debug_set_attend_tile(tile_loads), "st3_debug_set_attend_tile")
