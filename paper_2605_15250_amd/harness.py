"""Device-side plumbing around the binding: moves seeded host arrays into HBM in the library's documented
formats, owns plans and workspaces, and calls the entry points.  No arithmetic of the method happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

NUM_CUS = 256


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def lib_dtype(dtype: str) -> int:
    return B.GQLA_BF16 if dtype == "bf16" else B.GQLA_F32


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    """Host fp32 array (already holding storage-representable values) -> device tensor of the storage type."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch_dtype(dtype)).cuda()


def build_latent_pool(cfg, lens, table, num_pages, row_fn, fill=float("nan")) -> torch.Tensor:
    """Latent pool [num_pages, P, r_kv + d_r] on the device; row_fn(b, L_b) returns sequence b's rows.
    Slots no token owns hold `fill` (NaN by default: a decode that touched them would show)."""
    P, W = cfg.page_size, cfg.r_kv + cfg.d_r
    pool = torch.full((num_pages, P, W), fill, dtype=torch_dtype(cfg.dtype), device="cuda")
    flat = pool.view(num_pages * P, W)
    for b in range(len(lens)):
        L = int(lens[b])
        rows = torch.from_numpy(row_fn(b, L)).to(torch_dtype(cfg.dtype))
        t = np.arange(L)
        idx = torch.from_numpy(table[b][t // P].astype(np.int64) * P + t % P).cuda()
        flat[idx] = rows.cuda()
    return pool


class Decoder:
    """Holds the device-resident state of one configuration and runs the four entry points on it."""

    def __init__(self, cfg, lens, table, num_pages, groups=None, group_begin=0, use_page_table=True,
                 chunk_pages_absorb=0, chunk_pages_gqa=0, num_cus=NUM_CUS):
        self.cfg = cfg
        self.lens = np.ascontiguousarray(lens, dtype=np.int32)
        self.table = np.ascontiguousarray(table, dtype=np.int32)
        self.num_pages = int(num_pages)
        self.max_pages = self.table.shape[1]
        self.groups = cfg.g if groups is None else groups       # groups held by the expanded cache (TP slice if < g)
        self.group_begin = group_begin
        self.shape = B.make_shape(cfg.B, cfg.h_q, cfg.g, cfg.d_h, cfg.r_kv, cfg.d_r, cfg.s_q, lib_dtype(cfg.dtype), 0.0, cfg.d_v)
        # the library has bf16 kernels over the expanded cache for (d_h, d_v) = (128, 128) and (192, 256) only
        self.absorb_only = cfg.dtype == "bf16" and (cfg.d_h, cfg.dv) not in ((128, 128), (192, 256))
        G = cfg.h_q // cfg.g
        # shape seen by the GQA decode: for a slice, only the heads and groups of the slice
        self.shape_gqa = B.make_shape(cfg.B, G * self.groups, self.groups, cfg.d_h, cfg.r_kv, cfg.d_r, cfg.s_q,
                                      lib_dtype(cfg.dtype), 0.0, cfg.d_v)
        self.d_lens = torch.from_numpy(self.lens).cuda()
        self.d_table = torch.from_numpy(self.table).cuda() if use_page_table else None
        self.plan_a = B.gqla_plan_create(self.shape, self.lens, cfg.page_size, num_cus, B.GQLA_PATH_ABSORB, chunk_pages_absorb)
        self.ws_a = torch.empty(B.gqla_plan_workspace_bytes(self.plan_a), dtype=torch.uint8, device="cuda")
        B.gqla_plan_upload(self.plan_a, self.ws_a)
        self.plan_g = self.ws_g = None
        if not self.absorb_only:
            self.plan_g = B.gqla_plan_create(self.shape_gqa, self.lens, cfg.page_size, num_cus, B.GQLA_PATH_GQA, chunk_pages_gqa)
            self.ws_g = torch.empty(B.gqla_plan_workspace_bytes(self.plan_g), dtype=torch.uint8, device="cuda")
            B.gqla_plan_upload(self.plan_g, self.ws_g)
        self.latent_pool = None
        self.expanded_pool = None
        self.expanded_fp8_pool = None
        self.latent_fp8_pool = None
        self.ws_e = None                                        # scratch of the expand call
        self.ws_o = None                                        # scratch of the output projection

    def close(self):
        for p in (self.plan_a, self.plan_g):
            if p:
                B.gqla_plan_destroy(p)
        self.plan_a = self.plan_g = None

    # -- caches -------------------------------------------------------------------------------------------
    def latent_cache(self):
        return B.make_cache(self.latent_pool, self.d_lens, self.d_table, self.cfg.page_size, self.max_pages, self.num_pages, 0)

    def expanded_cache(self):
        return B.make_cache(self.expanded_pool, self.d_lens, self.d_table, self.cfg.page_size, self.max_pages,
                            self.num_pages, self.groups)

    def expanded_page_elems(self):
        c = self.cfg
        return c.page_size * (self.groups * (c.d_h + c.dv) + c.d_r)

    def alloc_expanded(self, fill=float("nan")):
        self.expanded_pool = torch.full((self.num_pages * self.expanded_page_elems(),), fill,
                                        dtype=torch_dtype(self.cfg.dtype), device="cuda")
        return self.expanded_pool

    # -- entry points ---------------------------------------------------------------------------------------
    def absorb_query(self, q_c, w_uk, q_hat=None):
        c = self.cfg
        if q_hat is None:
            q_hat = torch.empty((c.B, c.s_q, c.h_q, c.r_kv), dtype=torch_dtype(c.dtype), device="cuda")
        B.gqla_absorb_query(self.shape, q_c, w_uk, q_hat)
        return q_hat

    def decode_absorb(self, q_hat, q_r, w_uv, out=None, lse=None):
        c = self.cfg
        if out is None:
            out = torch.empty((c.B, c.s_q, c.h_q, c.dv), dtype=torch_dtype(c.dtype), device="cuda")
        if lse is None:
            lse = torch.empty((c.B, c.s_q, c.h_q), dtype=torch.float32, device="cuda")
        B.gqla_decode_absorb(self.shape, self.plan_a, q_hat, q_r, self.latent_cache(), w_uv, out, lse, self.ws_a)
        return out, lse

    def expand(self, w_uk, w_uv):
        if self.expanded_pool is None:
            self.alloc_expanded()
        if self.ws_e is None:
            nbytes = B.gqla_expand_workspace_bytes(self.shape, self.groups)
            self.ws_e = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")
        B.gqla_expand_cache(self.shape, self.latent_cache(), w_uk, w_uv, self.group_begin, self.groups,
                            self.expanded_cache(), self.ws_e)
        return self.expanded_pool

    def expand_tail(self, w_uk, w_uv, tail_tokens):
        if self.ws_e is None:
            nbytes = B.gqla_expand_workspace_bytes(self.shape, self.groups)
            self.ws_e = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")
        B.gqla_expand_cache_tail(self.shape, self.latent_cache(), w_uk, w_uv, self.group_begin, self.groups,
                                 self.expanded_cache(), tail_tokens, self.ws_e)
        return self.expanded_pool

    def pack_expand_weights(self, w_uk, w_uv):
        """The slice's weights in the expansion kernels' operand order, kept for expand_tail_packed."""
        nbytes = B.gqla_expand_workspace_bytes(self.shape, self.groups)
        self.packed_w = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")
        B.gqla_pack_expand_weights(self.shape, w_uk, w_uv, self.group_begin, self.groups, self.packed_w)
        return self.packed_w

    def expand_tail_packed(self, tail_tokens):
        B.gqla_expand_cache_tail_packed(self.shape, self.latent_cache(), self.packed_w, self.groups, self.expanded_cache(), tail_tokens)
        return self.expanded_pool

    def append_latent(self, rows):
        """rows: [B, s_q, r_kv + d_r] contiguous, the cache's element type."""
        B.gqla_append_latent(self.shape, rows, self.latent_cache())

    def rope_step(self, rope_base, q_r=None, rows=None):
        """In place: q_r [B, s_q, h_q, d_r] and the k_R part of rows [B, s_q, r_kv + d_r]."""
        B.gqla_rope_step(self.shape, self.d_lens, rope_base, q_r, rows)

    def output_projection(self, o, w_o, y=None):
        """o [B, s_q, h_q, d_h], w_o [d_model, h_q * d_h] -> y [B, s_q, d_model]."""
        c = self.cfg
        d_model = w_o.shape[0]
        if y is None:
            y = torch.empty((c.B, c.s_q, d_model), dtype=torch_dtype(c.dtype), device="cuda")
        nbytes = B.gqla_output_projection_workspace_bytes(self.shape, d_model)
        if nbytes and (self.ws_o is None or self.ws_o.numel() < nbytes):
            self.ws_o = torch.empty((nbytes,), dtype=torch.uint8, device="cuda")
        B.gqla_output_projection(self.shape, d_model, o, w_o, y, self.ws_o if nbytes else None)
        return y

    def compress(self, w_inv):
        """Expanded cache -> latent cache (all g groups must be held)."""
        B.gqla_compress_cache(self.shape, self.expanded_cache(), w_inv, self.latent_cache())
        return self.latent_pool

    # -- 8-bit expanded cache ------------------------------------------------------------------------------
    def fp8_page_bytes(self):
        c = self.cfg
        return c.page_size * B.gqla_expanded_fp8_bytes_per_token(self.groups, c.d_h, c.d_r)

    def alloc_expanded_fp8(self, fill=0xAA):
        self.expanded_fp8_pool = torch.full((self.num_pages * self.fp8_page_bytes(),), fill, dtype=torch.uint8, device="cuda")
        return self.expanded_fp8_pool

    def expanded_fp8_cache(self):
        return B.make_cache(self.expanded_fp8_pool, self.d_lens, self.d_table, self.cfg.page_size, self.max_pages,
                            self.num_pages, self.groups)

    def quantize_expanded(self, k_scale, v_scale):
        B.gqla_quantize_expanded(self.shape, self.expanded_cache(), self.expanded_fp8_cache(), k_scale, v_scale)
        return self.expanded_fp8_pool

    def expand_fp8(self, w_uk, w_uv, k_scale, v_scale):
        if self.expanded_fp8_pool is None:
            self.alloc_expanded_fp8()
        if self.ws_e is None:
            nbytes = B.gqla_expand_workspace_bytes(self.shape, self.groups)
            self.ws_e = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")
        B.gqla_expand_cache_fp8(self.shape, self.latent_cache(), w_uk, w_uv, self.group_begin, self.groups,
                                self.expanded_fp8_cache(), k_scale, v_scale, self.ws_e)
        return self.expanded_fp8_pool

    def expand_tail_fp8(self, w_uk, w_uv, tail_tokens, k_scale, v_scale):
        if self.ws_e is None:
            nbytes = B.gqla_expand_workspace_bytes(self.shape, self.groups)
            self.ws_e = torch.empty((max(nbytes, 16),), dtype=torch.uint8, device="cuda")
        B.gqla_expand_cache_tail_fp8(self.shape, self.latent_cache(), w_uk, w_uv, self.group_begin, self.groups,
                                     self.expanded_fp8_cache(), tail_tokens, k_scale, v_scale, self.ws_e)
        return self.expanded_fp8_pool

    def decode_gqa_fp8(self, q_c, q_r, k_scale, v_scale, out=None, lse=None):
        c = self.cfg
        heads = self.groups * (c.h_q // c.g)
        if out is None:
            out = torch.empty((c.B, c.s_q, heads, c.d_h), dtype=torch_dtype(c.dtype), device="cuda")
        if lse is None:
            lse = torch.empty((c.B, c.s_q, heads), dtype=torch.float32, device="cuda")
        B.gqla_decode_gqa_fp8(self.shape_gqa, self.plan_g, q_c, q_r, self.expanded_fp8_cache(), k_scale, v_scale, out, lse, self.ws_g)
        return out, lse

    # -- 8-bit latent cache --------------------------------------------------------------------------------
    def latent_fp8_page_bytes(self):
        c = self.cfg
        return c.page_size * B.gqla_latent_fp8_bytes_per_token(c.r_kv, c.d_r)

    def alloc_latent_fp8(self, fill=0xAA):
        self.latent_fp8_pool = torch.full((self.num_pages * self.latent_fp8_page_bytes(),), fill, dtype=torch.uint8, device="cuda")
        return self.latent_fp8_pool

    def latent_fp8_cache(self):
        return B.make_cache(self.latent_fp8_pool, self.d_lens, self.d_table, self.cfg.page_size, self.max_pages, self.num_pages, 0)

    def quantize_latent(self, c_scale):
        B.gqla_quantize_latent(self.shape, self.latent_cache(), self.latent_fp8_cache(), c_scale)
        return self.latent_fp8_pool

    def decode_absorb_fp8(self, q_hat, q_r, c_scale, w_uv, out=None, lse=None):
        c = self.cfg
        if out is None:
            out = torch.empty((c.B, c.s_q, c.h_q, c.dv), dtype=torch_dtype(c.dtype), device="cuda")
        if lse is None:
            lse = torch.empty((c.B, c.s_q, c.h_q), dtype=torch.float32, device="cuda")
        B.gqla_decode_absorb_fp8(self.shape, self.plan_a, q_hat, q_r, self.latent_fp8_cache(), c_scale, w_uv, out, lse, self.ws_a)
        return out, lse

    def decode_gqa(self, q_c, q_r, out=None, lse=None):
        """q_c, q_r: [B, s_q, heads of the slice, d] contiguous."""
        c = self.cfg
        hq = (c.h_q // c.g) * self.groups
        if out is None:
            out = torch.empty((c.B, c.s_q, hq, c.dv), dtype=torch_dtype(c.dtype), device="cuda")
        if lse is None:
            lse = torch.empty((c.B, c.s_q, hq), dtype=torch.float32, device="cuda")
        B.gqla_decode_gqa(self.shape_gqa, self.plan_g, q_c, q_r, self.expanded_cache(), out, lse, self.ws_g)
        return out, lse
