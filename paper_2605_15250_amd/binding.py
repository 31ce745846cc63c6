"""ctypes binding of libgqla.so: same names as the C entry points, argument marshalling only.

Tensors are torch tensors used purely as device-memory handles (data_ptr) and streams; every step of the
path runs in the library's kernels.  A non-OK status raises GqlaError."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# GQLA_LIB_PATH: another build of the same library (the CPU tests point it at the build whose host code is
# instrumented by the sanitizers); there is still no fallback if the file is missing.
LIB_PATH = os.environ.get("GQLA_LIB_PATH") or os.path.join(_HERE, "libgqla.so")

GQLA_OK = 0
GQLA_ERR_NULL, GQLA_ERR_SHAPE, GQLA_ERR_DTYPE, GQLA_ERR_ALIGN, GQLA_ERR_SEQLEN = 1, 2, 3, 4, 5
GQLA_ERR_PAGE, GQLA_ERR_WORKSPACE, GQLA_ERR_DEVICE, GQLA_ERR_PLAN = 6, 7, 8, 9
GQLA_F32, GQLA_BF16 = 0, 1
GQLA_PATH_ABSORB, GQLA_PATH_GQA = 0, 1

EXPORTS = [
    "gqla_plan_create", "gqla_plan_destroy", "gqla_plan_num_chunks", "gqla_plan_chunk_pages", "gqla_plan_export",
    "gqla_plan_workspace_bytes", "gqla_plan_upload", "gqla_absorb_query", "gqla_decode_absorb", "gqla_expand_cache",
    "gqla_expand_workspace_bytes", "gqla_expand_cache_tail", "gqla_append_latent", "gqla_probe_stream_read",
    "gqla_probe_mfma_bf16", "gqla_probe_mfma_flops", "gqla_estimate_paths", "gqla_select_path",
    "gqla_quantize_latent", "gqla_decode_absorb_fp8", "gqla_latent_fp8_bytes_per_token",
    "gqla_quantize_expanded", "gqla_decode_gqa_fp8", "gqla_expanded_fp8_bytes_per_token", "gqla_expand_cache_tail_fp8", "gqla_expand_cache_fp8",
    "gqla_left_inverse", "gqla_compress_cache", "gqla_rope_step", "gqla_output_projection",
    "gqla_output_projection_workspace_bytes",
    "gqla_decode_gqa", "gqla_latent_elems_per_token", "gqla_expanded_elems_per_token", "gqla_latent_offset",
    "gqla_expanded_k_offset", "gqla_expanded_v_offset", "gqla_expanded_kr_offset", "gqla_status_string",
    "gqla_expanded_elems_per_token_dv", "gqla_expanded_k_offset_dv", "gqla_expanded_v_offset_dv", "gqla_expanded_kr_offset_dv",
    "gqla_time_next_decode_kernel", "gqla_expand_cache_tail_static", "gqla_expand_cache_tail_static_max_workspace",
    "gqla_pack_expand_weights", "gqla_expand_cache_tail_packed",
]


class GqlaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


class gqla_shape(C.Structure):
    _fields_ = [("batch", C.c_int32), ("h_q", C.c_int32), ("g", C.c_int32), ("d_h", C.c_int32), ("r_kv", C.c_int32),
                ("d_r", C.c_int32), ("s_q", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float), ("d_v", C.c_int32)]


class gqla_cache(C.Structure):
    _fields_ = [("pool", C.c_void_p), ("seq_lens", C.c_void_p), ("page_table", C.c_void_p), ("page_size", C.c_int32),
                ("max_pages", C.c_int32), ("num_pages", C.c_int32), ("groups", C.c_int32)]


class gqla_path_estimate(C.Structure):
    _fields_ = [("absorb_bytes", C.c_double), ("absorb_flops", C.c_double), ("absorb_intensity", C.c_double),
                ("absorb_seconds", C.c_double), ("gqa_bytes", C.c_double), ("gqa_flops", C.c_double),
                ("gqa_intensity", C.c_double), ("gqa_seconds", C.c_double), ("ridge", C.c_double), ("faster_path", C.c_int32)]


class gqla_path_choice(C.Structure):
    _fields_ = [("absorb_seconds", C.c_double), ("gqa_seconds", C.c_double), ("faster_path", C.c_int32)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libgqla.so is missing at %s: build it with `python -m paper_2605_15250_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        sp, cp = C.POINTER(gqla_shape), C.POINTER(gqla_cache)
        L.gqla_plan_create.argtypes = [sp, vp, i32, i32, i32, i32, C.POINTER(vp)]
        L.gqla_plan_create.restype = i32
        L.gqla_plan_destroy.argtypes = [vp]
        L.gqla_plan_destroy.restype = None
        L.gqla_plan_num_chunks.argtypes = [vp]
        L.gqla_plan_num_chunks.restype = i32
        L.gqla_plan_chunk_pages.argtypes = [vp]
        L.gqla_plan_chunk_pages.restype = i32
        L.gqla_plan_export.argtypes = [vp, vp, vp, C.POINTER(i32)]
        L.gqla_plan_export.restype = i32
        L.gqla_plan_workspace_bytes.argtypes = [vp]
        L.gqla_plan_workspace_bytes.restype = sz
        L.gqla_plan_upload.argtypes = [vp, vp, sz, vp]
        L.gqla_plan_upload.restype = i32
        L.gqla_absorb_query.argtypes = [sp, vp, vp, vp, vp]
        L.gqla_absorb_query.restype = i32
        L.gqla_decode_absorb.argtypes = [sp, vp, vp, vp, cp, vp, vp, vp, vp, sz, vp]
        L.gqla_decode_absorb.restype = i32
        L.gqla_expand_cache.argtypes = [sp, cp, vp, vp, i32, i32, cp, vp, C.c_size_t, vp]
        L.gqla_expand_cache.restype = i32
        L.gqla_expand_cache_tail.argtypes = [sp, cp, vp, vp, i32, i32, cp, i32, vp, C.c_size_t, vp]
        L.gqla_expand_cache_tail.restype = i32
        L.gqla_pack_expand_weights.argtypes = [sp, vp, vp, i32, i32, vp, C.c_size_t, vp]
        L.gqla_pack_expand_weights.restype = i32
        L.gqla_expand_cache_tail_packed.argtypes = [sp, cp, vp, C.c_size_t, i32, cp, i32, vp]
        L.gqla_expand_cache_tail_packed.restype = i32
        L.gqla_expand_cache_tail_static.argtypes = [sp, cp, vp, vp, i32, i32, cp, i32, vp]
        L.gqla_expand_cache_tail_static.restype = i32
        L.gqla_expand_cache_tail_static_max_workspace.argtypes = []
        L.gqla_expand_cache_tail_static_max_workspace.restype = C.c_size_t
        L.gqla_append_latent.argtypes = [sp, vp, cp, vp]
        L.gqla_append_latent.restype = i32
        L.gqla_estimate_paths.argtypes = [sp, i64, C.c_double, C.c_double, C.POINTER(gqla_path_estimate)]
        L.gqla_estimate_paths.restype = i32
        L.gqla_select_path.argtypes = [sp, i64, C.POINTER(gqla_path_choice)]
        L.gqla_select_path.restype = i32
        L.gqla_quantize_expanded.argtypes = [sp, cp, cp, C.c_float, C.c_float, vp]
        L.gqla_quantize_expanded.restype = i32
        L.gqla_decode_gqa_fp8.argtypes = [sp, vp, vp, vp, cp, C.c_float, C.c_float, vp, vp, vp, sz, vp]
        L.gqla_decode_gqa_fp8.restype = i32
        L.gqla_expand_cache_tail_fp8.argtypes = [sp, cp, vp, vp, i32, i32, cp, i32, C.c_float, C.c_float, vp, C.c_size_t, vp]
        L.gqla_expand_cache_tail_fp8.restype = i32
        L.gqla_expand_cache_fp8.argtypes = [sp, cp, vp, vp, i32, i32, cp, C.c_float, C.c_float, vp, C.c_size_t, vp]
        L.gqla_expand_cache_fp8.restype = i32
        L.gqla_left_inverse.argtypes = [sp, vp, vp]
        L.gqla_left_inverse.restype = i32
        L.gqla_compress_cache.argtypes = [sp, cp, vp, cp, vp]
        L.gqla_compress_cache.restype = i32
        L.gqla_rope_step.argtypes = [sp, vp, C.c_float, vp, vp, vp]
        L.gqla_rope_step.restype = i32
        L.gqla_output_projection.argtypes = [sp, i32, vp, vp, vp, vp, C.c_size_t, vp]
        L.gqla_output_projection.restype = i32
        L.gqla_output_projection_workspace_bytes.argtypes = [sp, i32]
        L.gqla_output_projection_workspace_bytes.restype = C.c_size_t
        L.gqla_quantize_latent.argtypes = [sp, cp, cp, C.c_float, vp]
        L.gqla_quantize_latent.restype = i32
        L.gqla_decode_absorb_fp8.argtypes = [sp, vp, vp, vp, cp, C.c_float, vp, vp, vp, vp, sz, vp]
        L.gqla_decode_absorb_fp8.restype = i32
        L.gqla_latent_fp8_bytes_per_token.argtypes = [i32, i32]
        L.gqla_latent_fp8_bytes_per_token.restype = i64
        L.gqla_expanded_fp8_bytes_per_token.argtypes = [i32, i32, i32]
        L.gqla_expanded_fp8_bytes_per_token.restype = i64
        L.gqla_probe_stream_read.argtypes = [vp, C.c_size_t, vp, i32, vp]
        L.gqla_probe_stream_read.restype = i32
        L.gqla_probe_mfma_bf16.argtypes = [vp, i32, i32, vp]
        L.gqla_probe_mfma_bf16.restype = i32
        L.gqla_probe_mfma_flops.argtypes = [i32, i32]
        L.gqla_probe_mfma_flops.restype = C.c_double
        L.gqla_expand_workspace_bytes.argtypes = [sp, i32]
        L.gqla_expand_workspace_bytes.restype = C.c_size_t
        L.gqla_decode_gqa.argtypes = [sp, vp, vp, vp, cp, vp, vp, vp, sz, vp]
        L.gqla_decode_gqa.restype = i32
        L.gqla_latent_elems_per_token.argtypes = [i32, i32]
        L.gqla_latent_elems_per_token.restype = i64
        L.gqla_expanded_elems_per_token.argtypes = [i32, i32, i32]
        L.gqla_expanded_elems_per_token.restype = i64
        L.gqla_latent_offset.argtypes = [i64, i32, i32, i32, i32, i32]
        L.gqla_latent_offset.restype = i64
        for name in ("gqla_expanded_k_offset", "gqla_expanded_v_offset"):
            getattr(L, name).argtypes = [i64, i32, i32, i32, i32, i32, i32, i32]
            getattr(L, name).restype = i64
        L.gqla_expanded_kr_offset.argtypes = [i64, i32, i32, i32, i32, i32, i32]
        L.gqla_expanded_kr_offset.restype = i64
        L.gqla_expanded_elems_per_token_dv.argtypes = [i32, i32, i32, i32]
        L.gqla_expanded_elems_per_token_dv.restype = i64
        for name in ("gqla_expanded_k_offset_dv", "gqla_expanded_v_offset_dv"):
            getattr(L, name).argtypes = [i64, i32, i32, i32, i32, i32, i32, i32, i32]
            getattr(L, name).restype = i64
        L.gqla_expanded_kr_offset_dv.argtypes = [i64, i32, i32, i32, i32, i32, i32, i32]
        L.gqla_expanded_kr_offset_dv.restype = i64
        L.gqla_time_next_decode_kernel.argtypes = [vp, vp]
        L.gqla_time_next_decode_kernel.restype = i32
        L.gqla_status_string.argtypes = [i32]
        L.gqla_status_string.restype = C.c_char_p
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().gqla_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != GQLA_OK:
        raise GqlaError(status, where)


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_shape(batch, h_q, g, d_h, r_kv, d_r, s_q, dtype, scale=0.0, d_v=0) -> gqla_shape:
    return gqla_shape(batch, h_q, g, d_h, r_kv, d_r, s_q, dtype, scale, d_v)


def make_cache(pool, seq_lens, page_table, page_size, max_pages, num_pages, groups=0) -> gqla_cache:
    return gqla_cache(_ptr(pool), _ptr(seq_lens), _ptr(page_table), page_size, max_pages, num_pages, groups)


# ---- plan -------------------------------------------------------------------------------------------------
def gqla_plan_create(shape: gqla_shape, seq_lens_host, page_size: int, num_cus: int, path: int,
                     chunk_pages_override: int = 0) -> int:
    lens = np.ascontiguousarray(seq_lens_host, dtype=np.int32)
    out = C.c_void_p()
    _check(lib().gqla_plan_create(C.byref(shape), lens.ctypes.data if lens.size else None, page_size, num_cus, path,
                                  chunk_pages_override, C.byref(out)), "gqla_plan_create")
    return out.value


def gqla_plan_destroy(plan):
    lib().gqla_plan_destroy(plan)


def gqla_plan_num_chunks(plan) -> int:
    return lib().gqla_plan_num_chunks(plan)


def gqla_plan_chunk_pages(plan) -> int:
    return lib().gqla_plan_chunk_pages(plan)


def gqla_plan_export(plan, batch: int):
    n = C.c_int32(gqla_plan_num_chunks(plan))
    triples = np.zeros((max(n.value, 1), 3), dtype=np.int32)
    first = np.zeros((max(batch, 1),), dtype=np.int32)
    _check(lib().gqla_plan_export(plan, triples.ctypes.data, first.ctypes.data, C.byref(n)), "gqla_plan_export")
    return triples[: n.value], first[:batch]


def gqla_plan_workspace_bytes(plan) -> int:
    return lib().gqla_plan_workspace_bytes(plan)


def gqla_plan_upload(plan, ws, ws_bytes=None, stream=None):
    nbytes = ws_bytes if ws_bytes is not None else ws.numel() * ws.element_size()
    _check(lib().gqla_plan_upload(plan, _ptr(ws), nbytes, _stream(stream)), "gqla_plan_upload")


# ---- the decode paths -----------------------------------------------------------------------------------------
def gqla_absorb_query(shape, q_c, w_uk, q_hat, stream=None):
    _check(lib().gqla_absorb_query(C.byref(shape), _ptr(q_c), _ptr(w_uk), _ptr(q_hat), _stream(stream)), "gqla_absorb_query")


def gqla_decode_absorb(shape, plan, q_hat, q_r, latent: gqla_cache, w_uv, out, lse, ws, ws_bytes=None, stream=None):
    nbytes = ws_bytes if ws_bytes is not None else ws.numel() * ws.element_size()
    _check(lib().gqla_decode_absorb(C.byref(shape), plan, _ptr(q_hat), _ptr(q_r), C.byref(latent), _ptr(w_uv), _ptr(out),
                                    _ptr(lse), _ptr(ws), nbytes, _stream(stream)), "gqla_decode_absorb")


def gqla_estimate_paths(shape, cached_tokens, hbm_bytes_per_s, mfma_flops_per_s) -> dict:
    est = gqla_path_estimate()
    _check(lib().gqla_estimate_paths(C.byref(shape), int(cached_tokens), float(hbm_bytes_per_s), float(mfma_flops_per_s),
                                     C.byref(est)), "gqla_estimate_paths")
    return {name: getattr(est, name) for name, _ in gqla_path_estimate._fields_}


def gqla_select_path(shape, cached_tokens) -> dict:
    ch = gqla_path_choice()
    _check(lib().gqla_select_path(C.byref(shape), int(cached_tokens), C.byref(ch)), "gqla_select_path")
    return {name: getattr(ch, name) for name, _ in gqla_path_choice._fields_}


def gqla_probe_stream_read(src, nbytes, sink, num_cus, stream=None):
    _check(lib().gqla_probe_stream_read(_ptr(src), nbytes, _ptr(sink), num_cus, _stream(stream)), "gqla_probe_stream_read")


def gqla_probe_mfma_bf16(sink, iters, num_cus, stream=None):
    _check(lib().gqla_probe_mfma_bf16(_ptr(sink), iters, num_cus, _stream(stream)), "gqla_probe_mfma_bf16")


def gqla_time_next_decode_kernel(event_begin, event_end):
    """event_begin / event_end: raw hipEvent_t handles (ints), torch.cuda.Event objects that have been recorded at
    least once (torch creates the underlying event on first use), or None for both."""
    def raw(e):
        return e if e is None or isinstance(e, int) else e.cuda_event
    _check(lib().gqla_time_next_decode_kernel(raw(event_begin), raw(event_end)), "gqla_time_next_decode_kernel")


def gqla_probe_mfma_flops(iters, num_cus) -> float:
    return lib().gqla_probe_mfma_flops(iters, num_cus)


def gqla_expand_workspace_bytes(shape, group_count) -> int:
    return lib().gqla_expand_workspace_bytes(C.byref(shape), group_count)


def gqla_expand_cache(shape, latent: gqla_cache, w_uk, w_uv, group_begin, group_count, expanded: gqla_cache, ws=None,
                      ws_bytes=None, stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(lib().gqla_expand_cache(C.byref(shape), C.byref(latent), _ptr(w_uk), _ptr(w_uv), group_begin, group_count,
                                   C.byref(expanded), _ptr(ws), ws_bytes, _stream(stream)), "gqla_expand_cache")


def gqla_expand_cache_tail(shape, latent: gqla_cache, w_uk, w_uv, group_begin, group_count, expanded: gqla_cache,
                           tail_tokens, ws=None, ws_bytes=None, stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(lib().gqla_expand_cache_tail(C.byref(shape), C.byref(latent), _ptr(w_uk), _ptr(w_uv), group_begin, group_count,
                                        C.byref(expanded), tail_tokens, _ptr(ws), ws_bytes, _stream(stream)),
           "gqla_expand_cache_tail")


def gqla_pack_expand_weights(shape, w_uk, w_uv, group_begin, group_count, packed, packed_bytes=None, stream=None):
    if packed_bytes is None:
        packed_bytes = packed.numel() * packed.element_size() if packed is not None and hasattr(packed, "numel") else 0
    _check(lib().gqla_pack_expand_weights(C.byref(shape), _ptr(w_uk), _ptr(w_uv), group_begin, group_count, _ptr(packed),
                                          packed_bytes, _stream(stream)), "gqla_pack_expand_weights")


def gqla_expand_cache_tail_packed(shape, latent: gqla_cache, packed, group_count, expanded: gqla_cache, tail_tokens,
                                  packed_bytes=None, stream=None):
    if packed_bytes is None:
        packed_bytes = packed.numel() * packed.element_size() if packed is not None and hasattr(packed, "numel") else 0
    _check(lib().gqla_expand_cache_tail_packed(C.byref(shape), C.byref(latent), _ptr(packed), packed_bytes, group_count,
                                               C.byref(expanded), tail_tokens, _stream(stream)), "gqla_expand_cache_tail_packed")


def gqla_expand_cache_tail_static(shape, latent: gqla_cache, w_uk, w_uv, group_begin, group_count, expanded: gqla_cache,
                                  tail_tokens, stream=None):
    _check(lib().gqla_expand_cache_tail_static(C.byref(shape), C.byref(latent), _ptr(w_uk), _ptr(w_uv), group_begin, group_count,
                                               C.byref(expanded), tail_tokens, _stream(stream)), "gqla_expand_cache_tail_static")


def gqla_expand_cache_tail_static_max_workspace() -> int:
    return lib().gqla_expand_cache_tail_static_max_workspace()


def gqla_append_latent(shape, rows, latent: gqla_cache, stream=None):
    _check(lib().gqla_append_latent(C.byref(shape), _ptr(rows), C.byref(latent), _stream(stream)), "gqla_append_latent")


def gqla_decode_gqa(shape, plan, q_c, q_r, expanded: gqla_cache, out, lse, ws, ws_bytes=None, stream=None):
    nbytes = ws_bytes if ws_bytes is not None else ws.numel() * ws.element_size()
    _check(lib().gqla_decode_gqa(C.byref(shape), plan, _ptr(q_c), _ptr(q_r), C.byref(expanded), _ptr(out), _ptr(lse),
                                 _ptr(ws), nbytes, _stream(stream)), "gqla_decode_gqa")


def gqla_quantize_latent(shape, latent: gqla_cache, latent_fp8: gqla_cache, c_scale, stream=None):
    _check(lib().gqla_quantize_latent(C.byref(shape), C.byref(latent), C.byref(latent_fp8), float(c_scale), _stream(stream)),
           "gqla_quantize_latent")


def gqla_decode_absorb_fp8(shape, plan, q_hat, q_r, latent_fp8: gqla_cache, c_scale, w_uv, out, lse, ws, ws_bytes=None, stream=None):
    nbytes = ws_bytes if ws_bytes is not None else ws.numel() * ws.element_size()
    _check(lib().gqla_decode_absorb_fp8(C.byref(shape), plan, _ptr(q_hat), _ptr(q_r), C.byref(latent_fp8), float(c_scale),
                                        _ptr(w_uv), _ptr(out), _ptr(lse), _ptr(ws), nbytes, _stream(stream)), "gqla_decode_absorb_fp8")


def gqla_latent_fp8_bytes_per_token(r_kv, d_r) -> int:
    return lib().gqla_latent_fp8_bytes_per_token(r_kv, d_r)


def gqla_quantize_expanded(shape, expanded: gqla_cache, expanded_fp8: gqla_cache, k_scale, v_scale, stream=None):
    _check(lib().gqla_quantize_expanded(C.byref(shape), C.byref(expanded), C.byref(expanded_fp8), float(k_scale), float(v_scale),
                                        _stream(stream)), "gqla_quantize_expanded")


def gqla_decode_gqa_fp8(shape, plan, q_c, q_r, expanded_fp8: gqla_cache, k_scale, v_scale, out, lse, ws, ws_bytes=None, stream=None):
    nbytes = ws_bytes if ws_bytes is not None else ws.numel() * ws.element_size()
    _check(lib().gqla_decode_gqa_fp8(C.byref(shape), plan, _ptr(q_c), _ptr(q_r), C.byref(expanded_fp8), float(k_scale),
                                     float(v_scale), _ptr(out), _ptr(lse), _ptr(ws), nbytes, _stream(stream)), "gqla_decode_gqa_fp8")


def gqla_expand_cache_tail_fp8(shape, latent: gqla_cache, w_uk, w_uv, group_begin, group_count, expanded_fp8: gqla_cache,
                               tail_tokens, k_scale, v_scale, ws=None, ws_bytes=None, stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(lib().gqla_expand_cache_tail_fp8(C.byref(shape), C.byref(latent), _ptr(w_uk), _ptr(w_uv), group_begin, group_count,
                                            C.byref(expanded_fp8), tail_tokens, float(k_scale), float(v_scale), _ptr(ws), ws_bytes,
                                            _stream(stream)), "gqla_expand_cache_tail_fp8")


def gqla_left_inverse(shape, w_uk_host: np.ndarray) -> np.ndarray:
    """Host fp32 [g, r_kv, d_h] -> host fp32 [r_kv, g * d_h]."""
    w = np.ascontiguousarray(w_uk_host, dtype=np.float32)
    out = np.empty((shape.r_kv, shape.g * shape.d_h), dtype=np.float32)
    _check(lib().gqla_left_inverse(C.byref(shape), w.ctypes.data, out.ctypes.data), "gqla_left_inverse")
    return out


def gqla_compress_cache(shape, expanded: gqla_cache, w_inv, latent: gqla_cache, stream=None):
    _check(lib().gqla_compress_cache(C.byref(shape), C.byref(expanded), _ptr(w_inv), C.byref(latent), _stream(stream)),
           "gqla_compress_cache")


def gqla_expand_cache_fp8(shape, latent: gqla_cache, w_uk, w_uv, group_begin, group_count, expanded_fp8: gqla_cache, k_scale,
                          v_scale, ws=None, ws_bytes=None, stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(lib().gqla_expand_cache_fp8(C.byref(shape), C.byref(latent), _ptr(w_uk), _ptr(w_uv), group_begin, group_count,
                                       C.byref(expanded_fp8), float(k_scale), float(v_scale), _ptr(ws), ws_bytes,
                                       _stream(stream)), "gqla_expand_cache_fp8")


def gqla_rope_step(shape, seq_lens, rope_base, q_r, rows, stream=None):
    _check(lib().gqla_rope_step(C.byref(shape), _ptr(seq_lens), float(rope_base), _ptr(q_r), _ptr(rows), _stream(stream)),
           "gqla_rope_step")


def gqla_output_projection(shape, d_model, o, w_o, y, ws=None, ws_bytes=None, stream=None):
    if ws_bytes is None:
        ws_bytes = ws.numel() * ws.element_size() if ws is not None else 0
    _check(lib().gqla_output_projection(C.byref(shape), int(d_model), _ptr(o), _ptr(w_o), _ptr(y), _ptr(ws), ws_bytes,
                                        _stream(stream)), "gqla_output_projection")


def gqla_output_projection_workspace_bytes(shape, d_model) -> int:
    return lib().gqla_output_projection_workspace_bytes(C.byref(shape), int(d_model))


def gqla_expanded_fp8_bytes_per_token(groups, d_h, d_r) -> int:
    return lib().gqla_expanded_fp8_bytes_per_token(groups, d_h, d_r)


# ---- sizes ----------------------------------------------------------------------------------------------------------
def gqla_latent_elems_per_token(r_kv, d_r) -> int:
    return lib().gqla_latent_elems_per_token(r_kv, d_r)


def gqla_expanded_elems_per_token(groups, d_h, d_r) -> int:
    return lib().gqla_expanded_elems_per_token(groups, d_h, d_r)


def gqla_latent_offset(page, slot, col, page_size, r_kv, d_r) -> int:
    return lib().gqla_latent_offset(page, slot, col, page_size, r_kv, d_r)


def gqla_expanded_k_offset(page, j, slot, d, page_size, groups, d_h, d_r) -> int:
    return lib().gqla_expanded_k_offset(page, j, slot, d, page_size, groups, d_h, d_r)


def gqla_expanded_v_offset(page, j, slot, d, page_size, groups, d_h, d_r) -> int:
    return lib().gqla_expanded_v_offset(page, j, slot, d, page_size, groups, d_h, d_r)


def gqla_expanded_kr_offset(page, slot, d, page_size, groups, d_h, d_r) -> int:
    return lib().gqla_expanded_kr_offset(page, slot, d, page_size, groups, d_h, d_r)


def gqla_expanded_elems_per_token_dv(groups, d_h, d_v, d_r) -> int:
    return lib().gqla_expanded_elems_per_token_dv(groups, d_h, d_v, d_r)


def gqla_expanded_k_offset_dv(page, j, slot, d, page_size, groups, d_h, d_v, d_r) -> int:
    return lib().gqla_expanded_k_offset_dv(page, j, slot, d, page_size, groups, d_h, d_v, d_r)


def gqla_expanded_v_offset_dv(page, j, slot, d, page_size, groups, d_h, d_v, d_r) -> int:
    return lib().gqla_expanded_v_offset_dv(page, j, slot, d, page_size, groups, d_h, d_v, d_r)


def gqla_expanded_kr_offset_dv(page, slot, d, page_size, groups, d_h, d_v, d_r) -> int:
    return lib().gqla_expanded_kr_offset_dv(page, slot, d, page_size, groups, d_h, d_v, d_r)
