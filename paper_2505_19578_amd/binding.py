"""ctypes binding of libshareprefill.so: argument marshalling only.

Every function mirrors the C entry point of the same name (include/shareprefill.h).
Device buffers are torch tensors (used as typed device pointers); small id arrays
are host int32 sequences.  Calls enqueue on torch's current HIP stream.
"""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence

from .build import library_path

EXPORTED_SYMBOLS = [
    "sp_status_string", "sp_last_error", "sp_profile_enable", "sp_profile_read", "sp_workspace_bytes",
    "sp_dense_attn_with_block_scores", "sp_build_block_mask",
    "sp_block_sparse_attn", "sp_prefill_layer",
    "sp_score_workspace_bytes", "sp_mask_workspace_bytes", "sp_block_mean_logit_scores",
    "sp_build_block_mask_global", "sp_build_block_mask_global_static", "sp_prefill_layer_modes",
    "sp_determine_pattern", "sp_block_sparse_attn_gated", "sp_prefill_layer_gated", "sp_prefill_layer_dict",
    "sp_vs_workspace_bytes", "sp_search_vertical_slash", "sp_vs_token_workspace_bytes", "sp_vertical_slash_attn",
]

SP_FALLBACK_DENSE, SP_FALLBACK_VERTICAL_SLASH, SP_FALLBACK_VERTICAL_SLASH_TOKEN = 0, 1, 2
SP_STATIC_SCRATCH_BYTES = 2 << 20

SP_SCORE_BLOCK_MASS, SP_SCORE_MEAN_LOGIT = 0, 1
SP_SELECT_PER_ROW, SP_SELECT_GLOBAL = 0, 1


class SpShape(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("seq", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
        ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("block", ctypes.c_int32),
        ("q_stride_b", ctypes.c_int64), ("q_stride_t", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
        ("kv_stride_b", ctypes.c_int64), ("kv_stride_t", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64),
        ("o_stride_b", ctypes.c_int64), ("o_stride_t", ctypes.c_int64), ("o_stride_h", ctypes.c_int64),
        ("softmax_scale", ctypes.c_float),
    ]


class SpPatternDict(ctypes.Structure):
    _fields_ = [("n_clusters", ctypes.c_int32), ("valid", ctypes.c_void_p), ("a_tilde", ctypes.c_void_p),
                ("kb_idx", ctypes.c_void_p), ("kb_cnt", ctypes.c_void_p)]


class SpError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name}: {detail}")
        self.status = status
        self.status_name = name
        self.detail = detail


_lib = None


def lib() -> ctypes.CDLL:
    """Load libshareprefill.so (built on demand if absent); raises if that fails."""
    global _lib
    if _lib is None:
        # torch first: its bundled HIP runtime owns the device memory the calls receive, and the
        # library must bind to that same runtime instance rather than load a second copy
        import torch  # noqa: F401
        L = ctypes.CDLL(library_path())
        vp, ip, fp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p
        sp = ctypes.POINTER(SpShape)
        L.sp_status_string.restype = ctypes.c_char_p
        L.sp_status_string.argtypes = [ctypes.c_int]
        L.sp_last_error.restype = ctypes.c_char_p
        L.sp_last_error.argtypes = []
        L.sp_profile_enable.restype = ctypes.c_int
        L.sp_profile_enable.argtypes = [ctypes.c_int32]
        L.sp_profile_read.restype = ctypes.c_int
        L.sp_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float), ip, ctypes.c_int32]
        L.sp_workspace_bytes.restype = ctypes.c_int
        L.sp_workspace_bytes.argtypes = [sp, ctypes.c_int32, ctypes.POINTER(ctypes.c_size_t)]
        L.sp_dense_attn_with_block_scores.restype = ctypes.c_int
        L.sp_dense_attn_with_block_scores.argtypes = [sp, vp, vp, vp, ip, ctypes.c_int32, vp, fp, vp,
                                                      ctypes.c_size_t, vp]
        L.sp_build_block_mask.restype = ctypes.c_int
        L.sp_build_block_mask.argtypes = [fp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                          vp, vp, vp, vp]
        L.sp_block_sparse_attn.restype = ctypes.c_int
        L.sp_block_sparse_attn.argtypes = [sp, vp, vp, vp, ip, ip, ctypes.c_int32, vp, vp, ctypes.c_int32, vp,
                                           vp, ctypes.c_size_t, vp]
        L.sp_prefill_layer.restype = ctypes.c_int
        L.sp_prefill_layer.argtypes = [sp, vp, vp, vp, ip, ip, ctypes.c_int32, ctypes.c_float, vp, fp, vp, vp,
                                       vp, ctypes.c_size_t, vp]
        L.sp_score_workspace_bytes.restype = ctypes.c_int
        L.sp_score_workspace_bytes.argtypes = [sp, ctypes.c_int32, ctypes.POINTER(ctypes.c_size_t)]
        L.sp_mask_workspace_bytes.restype = ctypes.c_int
        L.sp_mask_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_size_t)]
        L.sp_block_mean_logit_scores.restype = ctypes.c_int
        L.sp_block_mean_logit_scores.argtypes = [sp, vp, vp, ip, ctypes.c_int32, fp, vp, ctypes.c_size_t, vp]
        L.sp_build_block_mask_global.restype = ctypes.c_int
        L.sp_build_block_mask_global.argtypes = [fp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                                 ctypes.c_int32, vp, vp, vp, ctypes.c_size_t, vp]
        L.sp_build_block_mask_global_static.restype = ctypes.c_int
        L.sp_build_block_mask_global_static.argtypes = [fp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                                        ctypes.c_float, ctypes.c_int32, vp, vp, vp]
        L.sp_prefill_layer_modes.restype = ctypes.c_int
        L.sp_prefill_layer_modes.argtypes = [sp, vp, vp, vp, ip, ip, ctypes.c_int32, ctypes.c_float, ctypes.c_int32,
                                             ctypes.c_int32, vp, fp, vp, vp, vp, ctypes.c_size_t, vp]
        L.sp_determine_pattern.restype = ctypes.c_int
        L.sp_determine_pattern.argtypes = [sp, vp, vp, ip, ctypes.c_int32, ip, ip, ctypes.c_float, ctypes.c_float,
                                           fp, fp, vp, vp, ctypes.c_size_t, vp]
        L.sp_block_sparse_attn_gated.restype = ctypes.c_int
        L.sp_block_sparse_attn_gated.argtypes = [sp, vp, vp, vp, ip, ctypes.c_int32, vp, vp, ctypes.c_int32, vp, vp,
                                                 vp, ctypes.c_size_t, vp]
        L.sp_prefill_layer_gated.restype = ctypes.c_int
        L.sp_prefill_layer_gated.argtypes = [sp, vp, vp, vp, ip, ip, ctypes.c_int32, ctypes.c_float, ctypes.c_float,
                                             ctypes.c_float, ctypes.c_int32, ctypes.c_int32, vp, fp, vp, vp, fp, fp,
                                             vp, vp, ctypes.c_size_t, vp]
        L.sp_prefill_layer_dict.restype = ctypes.c_int
        L.sp_prefill_layer_dict.argtypes = [sp, vp, vp, vp, ip, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                            ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                            ctypes.POINTER(SpPatternDict), vp, fp, vp, fp, fp, vp, vp, vp,
                                            ctypes.c_size_t, vp]
        L.sp_vs_workspace_bytes.restype = ctypes.c_int
        L.sp_vs_workspace_bytes.argtypes = [sp, ctypes.c_int32, ctypes.POINTER(ctypes.c_size_t)]
        L.sp_search_vertical_slash.restype = ctypes.c_int
        L.sp_search_vertical_slash.argtypes = [sp, vp, vp, ip, ctypes.c_int32, ctypes.c_float, ctypes.c_int32, fp, vp,
                                               vp, vp, ctypes.c_size_t, vp]
        L.sp_vs_token_workspace_bytes.restype = ctypes.c_int
        L.sp_vs_token_workspace_bytes.argtypes = [sp, ctypes.c_int32, ctypes.POINTER(ctypes.c_size_t)]
        L.sp_vertical_slash_attn.restype = ctypes.c_int
        L.sp_vertical_slash_attn.argtypes = [sp, vp, vp, vp, ip, ctypes.c_int32, ctypes.c_float, ctypes.c_int32, vp, vp,
                                             vp, vp, ctypes.c_size_t, vp]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        L = lib()
        raise SpError(rc, L.sp_status_string(rc).decode(), L.sp_last_error().decode())


def _ptr(t) -> Optional[int]:
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _ids(seq: Sequence[int]):
    arr = (ctypes.c_int32 * len(seq))(*[int(x) for x in seq])
    return arr


def _stream() -> ctypes.c_void_p:
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def shape_of(q, k, o=None, block: int = 128, softmax_scale: float = 0.0) -> SpShape:
    """sp_shape for token-major tensors q [b][t][hq][d], k/v [b][t][hkv][d] (any strides, d contiguous)."""
    assert q.dim() == 4 and k.dim() == 4 and q.stride(3) == 1 and k.stride(3) == 1
    o = q if o is None else o
    s = SpShape()
    s.batch, s.seq, s.n_q_heads, s.head_dim = q.shape
    s.n_kv_heads = k.shape[2]
    s.block = block
    s.q_stride_b, s.q_stride_t, s.q_stride_h = q.stride(0), q.stride(1), q.stride(2)
    s.kv_stride_b, s.kv_stride_t, s.kv_stride_h = k.stride(0), k.stride(1), k.stride(2)
    s.o_stride_b, s.o_stride_t, s.o_stride_h = o.stride(0), o.stride(1), o.stride(2)
    s.softmax_scale = softmax_scale
    return s


KERNEL_KINDS = ("pack", "dense", "mask", "sparse", "score", "vs")


def sp_profile_enable(on: bool):
    _check(lib().sp_profile_enable(1 if on else 0))


def sp_profile_read(reset: bool = True):
    """{kind: (total ms, launches)} since the last reset; synchronise the stream first."""
    ms = (ctypes.c_float * len(KERNEL_KINDS))()
    n = (ctypes.c_int32 * len(KERNEL_KINDS))()
    _check(lib().sp_profile_read(ms, n, 1 if reset else 0))
    return {k: (float(ms[a]), int(n[a])) for a, k in enumerate(KERNEL_KINDS)}


def sp_workspace_bytes(shape: SpShape, n_dense_heads: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().sp_workspace_bytes(ctypes.byref(shape), n_dense_heads, ctypes.byref(n)))
    return int(n.value)


def sp_dense_attn_with_block_scores(shape: SpShape, q, k, v, head_ids, o, block_scores, workspace):
    _check(lib().sp_dense_attn_with_block_scores(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ids(head_ids), len(head_ids), _ptr(o),
        _ptr(block_scores), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def sp_build_block_mask(block_scores, n_maps: int, nqb: int, nkb: int, gamma: float, kb_idx, kb_cnt,
                        bitmask=None):
    _check(lib().sp_build_block_mask(_ptr(block_scores), n_maps, nqb, nkb, ctypes.c_float(gamma),
                                     _ptr(kb_idx), _ptr(kb_cnt), _ptr(bitmask), _stream()))


def sp_block_sparse_attn(shape: SpShape, q, k, v, head_ids, head_map, kb_idx, kb_cnt, n_maps: int, o, workspace):
    assert len(head_ids) == len(head_map)
    _check(lib().sp_block_sparse_attn(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ids(head_ids), _ids(head_map), len(head_ids),
        _ptr(kb_idx), _ptr(kb_cnt), n_maps, _ptr(o), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream()))


def sp_prefill_layer(shape: SpShape, q, k, v, head_to_cluster, pivot_heads, gamma: float, o, block_scores,
                     kb_idx, kb_cnt, workspace):
    _check(lib().sp_prefill_layer(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ids(head_to_cluster), _ids(pivot_heads),
        len(pivot_heads), ctypes.c_float(gamma), _ptr(o), _ptr(block_scores), _ptr(kb_idx), _ptr(kb_cnt),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream()))


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def sp_score_workspace_bytes(shape: SpShape, n_heads: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().sp_score_workspace_bytes(ctypes.byref(shape), n_heads, ctypes.byref(n)))
    return int(n.value)


def sp_mask_workspace_bytes(n_maps: int, nqb: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().sp_mask_workspace_bytes(n_maps, nqb, ctypes.byref(n)))
    return int(n.value)


def sp_block_mean_logit_scores(shape: SpShape, q, k, head_ids, block_scores, workspace):
    _check(lib().sp_block_mean_logit_scores(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ids(head_ids), len(head_ids), _ptr(block_scores),
        _ptr(workspace), _nbytes(workspace), _stream()))


def sp_build_block_mask_global(block_scores, n_maps: int, nqb: int, nkb: int, gamma: float, forced: bool,
                               kb_idx, kb_cnt, workspace):
    _check(lib().sp_build_block_mask_global(_ptr(block_scores), n_maps, nqb, nkb, ctypes.c_float(gamma),
                                            1 if forced else 0, _ptr(kb_idx), _ptr(kb_cnt), _ptr(workspace),
                                            _nbytes(workspace), _stream()))


def sp_build_block_mask_global_static(block_scores, n_maps: int, nqb: int, nkb: int, gamma: float, forced: bool,
                                      kb_idx, kb_cnt):
    _check(lib().sp_build_block_mask_global_static(_ptr(block_scores), n_maps, nqb, nkb, ctypes.c_float(gamma),
                                                   1 if forced else 0, _ptr(kb_idx), _ptr(kb_cnt), _stream()))


def sp_prefill_layer_modes(shape: SpShape, q, k, v, head_to_cluster, pivot_heads, gamma: float, score_mode: int,
                           select_mode: int, o, block_scores, kb_idx, kb_cnt, workspace):
    _check(lib().sp_prefill_layer_modes(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ids(head_to_cluster), _ids(pivot_heads),
        len(pivot_heads), ctypes.c_float(gamma), int(score_mode), int(select_mode), _ptr(o), _ptr(block_scores),
        _ptr(kb_idx), _ptr(kb_cnt), _ptr(workspace), _nbytes(workspace), _stream()))


def sp_determine_pattern(shape: SpShape, q, k, head_ids, ref_pos, shared_map, delta: float, tau: float, a_hat, dist,
                         head_pattern, workspace):
    assert len(head_ids) == len(ref_pos) == len(shared_map)
    _check(lib().sp_determine_pattern(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ids(head_ids), len(head_ids), _ids(ref_pos), _ids(shared_map),
        ctypes.c_float(delta), ctypes.c_float(tau), _ptr(a_hat), _ptr(dist), _ptr(head_pattern), _ptr(workspace),
        _nbytes(workspace), _stream()))


def sp_block_sparse_attn_gated(shape: SpShape, q, k, v, head_ids, kb_idx, kb_cnt, n_maps: int, head_pattern, o,
                               workspace):
    _check(lib().sp_block_sparse_attn_gated(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ids(head_ids), len(head_ids), _ptr(kb_idx), _ptr(kb_cnt),
        n_maps, _ptr(head_pattern), _ptr(o), _ptr(workspace), _nbytes(workspace), _stream()))


def sp_prefill_layer_gated(shape: SpShape, q, k, v, head_to_cluster, pivot_heads, gamma: float, delta: float,
                           tau: float, score_mode: int, select_mode: int, o, block_scores, kb_idx, kb_cnt, a_hat,
                           dist, head_pattern, workspace):
    _check(lib().sp_prefill_layer_gated(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ids(head_to_cluster), _ids(pivot_heads),
        len(pivot_heads), ctypes.c_float(gamma), ctypes.c_float(delta), ctypes.c_float(tau), int(score_mode),
        int(select_mode), _ptr(o), _ptr(block_scores), _ptr(kb_idx), _ptr(kb_cnt), _ptr(a_hat), _ptr(dist),
        _ptr(head_pattern), _ptr(workspace), _nbytes(workspace), _stream()))


def pattern_dict_of(valid, a_tilde, kb_idx, kb_cnt) -> SpPatternDict:
    """sp_pattern_dict over caller-owned device tensors valid [b][C], a_tilde [b][C][nkb],
    kb_idx [b][C][nqb][nkb], kb_cnt [b][C][nqb] (the returned struct only points at them: keep them alive)."""
    d = SpPatternDict()
    d.n_clusters = valid.shape[1]
    d.valid, d.a_tilde, d.kb_idx, d.kb_cnt = valid.data_ptr(), a_tilde.data_ptr(), kb_idx.data_ptr(), kb_cnt.data_ptr()
    return d


def sp_prefill_layer_dict(shape: SpShape, q, k, v, head_to_cluster, gamma: float, delta: float, tau: float,
                          score_mode: int, select_mode: int, pattern_dict: SpPatternDict, o, block_scores, role,
                          a_hat, dist, workspace, fallback_mode: int = 0, vs_idx=None, vs_cnt=None):
    _check(lib().sp_prefill_layer_dict(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ids(head_to_cluster), ctypes.c_float(gamma),
        ctypes.c_float(delta), ctypes.c_float(tau), int(score_mode), int(select_mode), int(fallback_mode),
        ctypes.byref(pattern_dict), _ptr(o), _ptr(block_scores), _ptr(role), _ptr(a_hat), _ptr(dist), _ptr(vs_idx),
        _ptr(vs_cnt), _ptr(workspace), _nbytes(workspace), _stream()))


def sp_vs_workspace_bytes(shape: SpShape, n_heads: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().sp_vs_workspace_bytes(ctypes.byref(shape), n_heads, ctypes.byref(n)))
    return int(n.value)


def sp_search_vertical_slash(shape: SpShape, q, k, head_ids, gamma: float, forced: bool, sums, kb_idx, kb_cnt,
                             workspace):
    _check(lib().sp_search_vertical_slash(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ids(head_ids), len(head_ids), ctypes.c_float(gamma),
        1 if forced else 0, _ptr(sums), _ptr(kb_idx), _ptr(kb_cnt), _ptr(workspace), _nbytes(workspace), _stream()))


def sp_vs_token_workspace_bytes(shape: SpShape, n_heads: int) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().sp_vs_token_workspace_bytes(ctypes.byref(shape), n_heads, ctypes.byref(n)))
    return int(n.value)


def sp_vertical_slash_attn(shape: SpShape, q, k, v, head_ids, gamma: float, forced: bool, o, keep_bits, pairs,
                           workspace):
    _check(lib().sp_vertical_slash_attn(
        ctypes.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ids(head_ids), len(head_ids), ctypes.c_float(gamma),
        1 if forced else 0, _ptr(o), _ptr(keep_bits), _ptr(pairs), _ptr(workspace), _nbytes(workspace), _stream()))
