"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and its host
logic (split plan, offsets, argument validation) agrees with the oracle's independent bookkeeping."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import layout as Lay
from paper_2605_15250_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gqla.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(gqla_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_struct_sizes_match_header_layout():
    assert C.sizeof(B.gqla_shape) == 40      # nine 4-byte fields and d_v
    assert C.sizeof(B.gqla_cache) == 40


@pytest.mark.parametrize("path,opath", [(B.GQLA_PATH_ABSORB, Lay.PATH_ABSORB), (B.GQLA_PATH_GQA, Lay.PATH_GQA)])
@pytest.mark.parametrize("lens,h_q,g,s_q", [
    ([8192] * 64, 128, 8, 1), ([8192] * 64, 128, 8, 2), ([4096] * 32, 32, 8, 1), ([8192] * 64, 16, 1, 2),
    (list(range(1024, 32768, 499)), 128, 8, 2), ([1, 2, 63, 64, 65, 4097], 128, 8, 1), ([2], 128, 8, 2),
])
def test_plan_is_bit_exact_against_oracle_rule(path, opath, lens, h_q, g, s_q):
    sh = B.make_shape(len(lens), h_q, g, 128, 512, 64, s_q, B.GQLA_BF16)
    if min(lens) < s_q:
        with pytest.raises(B.GqlaError) as e:
            B.gqla_plan_create(sh, lens, 64, 256, path)
        assert e.value.status == B.GQLA_ERR_SEQLEN
        return
    p = B.gqla_plan_create(sh, lens, 64, 256, path)
    try:
        cp = Lay.plan_chunk_pages(lens, 64, 256, opath, h_q, g, s_q)
        chunks, first = Lay.plan_chunks(lens, 64, cp)
        triples, first_lib = B.gqla_plan_export(p, len(lens))
        assert B.gqla_plan_chunk_pages(p) == cp
        assert B.gqla_plan_num_chunks(p) == len(chunks)
        assert triples.tolist() == [list(c) for c in chunks]
        assert first_lib.tolist() == first
        assert B.gqla_plan_workspace_bytes(p) > 0
    finally:
        B.gqla_plan_destroy(p)


def test_plan_override_and_random_lengths():
    r = np.random.default_rng(0)
    for _ in range(20):
        B_ = int(r.integers(1, 40))
        lens = r.integers(2, 5000, size=B_).tolist()
        cp = int(r.integers(1, 9))
        sh = B.make_shape(B_, 8, 2, 16, 32, 8, 2, B.GQLA_F32)
        p = B.gqla_plan_create(sh, lens, 16, 256, B.GQLA_PATH_GQA, cp)
        chunks, first = Lay.plan_chunks(lens, 16, cp)
        triples, first_lib = B.gqla_plan_export(p, B_)
        assert triples.tolist() == [list(c) for c in chunks] and first_lib.tolist() == first
        B.gqla_plan_destroy(p)


def test_offsets_match_oracle_layout():
    r = np.random.default_rng(1)
    for P, gc, d_h, d_r in ((64, 8, 128, 64), (16, 2, 16, 8), (128, 1, 128, 64)):
        for _ in range(200):
            page, j, slot = int(r.integers(0, 1000)), int(r.integers(0, gc)), int(r.integers(0, P))
            d, dr = int(r.integers(0, d_h)), int(r.integers(0, d_r))
            assert B.gqla_expanded_k_offset(page, j, slot, d, P, gc, d_h, d_r) == Lay.expanded_k_offset(page, j, slot, d, P, gc, d_h, d_r)
            assert B.gqla_expanded_v_offset(page, j, slot, d, P, gc, d_h, d_r) == Lay.expanded_v_offset(page, j, slot, d, P, gc, d_h, d_r)
            assert B.gqla_expanded_kr_offset(page, slot, dr, P, gc, d_h, d_r) == Lay.expanded_kr_offset(page, slot, dr, P, gc, d_h, d_r)
            assert B.gqla_latent_offset(page, slot, d, P, 512, d_r) == Lay.latent_offset(page, slot, d, P, 512, d_r)
    assert B.gqla_latent_elems_per_token(512, 64) == 576
    assert B.gqla_expanded_elems_per_token(8, 128, 64) == 2112
    assert B.gqla_expanded_elems_per_token(4, 128, 64) * 2 == 2176
    # large pools do not overflow 32 bits: page 600000 of a g = 8 pool
    assert B.gqla_expanded_k_offset(600000, 0, 0, 0, 64, 8, 128, 64) == 600000 * 64 * 2112


def _expect(status, fn, *args, **kw):
    with pytest.raises(B.GqlaError) as e:
        fn(*args, **kw)
    assert e.value.status == status, (e.value.status, status)


def test_argument_validation_happens_on_the_host():
    """Every rejected call returns before touching a device (this container has none)."""
    ok = B.make_shape(2, 128, 8, 128, 512, 64, 1, B.GQLA_BF16)
    lens = [100, 200]
    _expect(B.GQLA_ERR_SHAPE, B.gqla_plan_create, B.make_shape(2, 10, 4, 128, 512, 64, 1, B.GQLA_BF16), lens, 64, 256, 0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_plan_create, B.make_shape(2, 128, 8, 128, 512, 64, 3, B.GQLA_BF16), lens, 64, 256, 0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_plan_create, B.make_shape(2, 128, 8, 96, 512, 64, 1, B.GQLA_BF16), lens, 64, 256, 0)
    _expect(B.GQLA_ERR_DTYPE, B.gqla_plan_create, B.make_shape(2, 128, 8, 128, 512, 64, 1, 7), lens, 64, 256, 0)
    _expect(B.GQLA_ERR_PAGE, B.gqla_plan_create, ok, lens, 48, 256, 0)
    _expect(B.GQLA_ERR_PLAN, B.gqla_plan_create, ok, lens, 64, 256, 5)
    _expect(B.GQLA_ERR_SEQLEN, B.gqla_plan_create, ok, [100, 0], 64, 256, 0)
    # fake but aligned "device" addresses: validation never dereferences them
    A = 0x10000
    _expect(B.GQLA_ERR_NULL, B.gqla_absorb_query, ok, None, A, A, stream=0)
    _expect(B.GQLA_ERR_ALIGN, B.gqla_absorb_query, ok, A + 2, A, A, stream=0)
    plan_a = B.gqla_plan_create(ok, lens, 64, 256, B.GQLA_PATH_ABSORB)
    plan_g = B.gqla_plan_create(ok, lens, 64, 256, B.GQLA_PATH_GQA)
    try:
        big = 1 << 30
        cache = B.make_cache(A, A, None, 64, 4, 8, 0)
        # table not uploaded into this workspace
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_decode_absorb, ok, plan_a, A, A, cache, A, A, None, A, big, stream=0)
        # wrong path for the plan
        _expect(B.GQLA_ERR_PLAN, B.gqla_decode_absorb, ok, plan_g, A, A, cache, A, A, None, A, big, stream=0)
        # plan built for another shape
        other = B.make_shape(2, 128, 8, 128, 512, 64, 2, B.GQLA_BF16)
        _expect(B.GQLA_ERR_PLAN, B.gqla_decode_gqa, other, plan_g, A, A, cache, A, None, A, big, stream=0)
        # cache too short for the planned lengths (max_pages * page_size < 200)
        short = B.make_cache(A, A, None, 64, 2, 8, 8)
        _expect(B.GQLA_ERR_SEQLEN, B.gqla_decode_gqa, ok, plan_g, A, A, short, A, None, A, big, stream=0)
        # identity page map needs batch * max_pages pages
        small = B.make_cache(A, A, None, 64, 4, 7, 8)
        _expect(B.GQLA_ERR_PAGE, B.gqla_decode_gqa, ok, plan_g, A, A, small, A, None, A, big, stream=0)
        # page size differs from the plan's
        _expect(B.GQLA_ERR_PAGE, B.gqla_decode_gqa, ok, plan_g, A, A, B.make_cache(A, A, None, 128, 4, 8, 8), A, None, A, big, stream=0)
        # workspace too small for the upload
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_plan_upload, plan_g, A, 16, stream=0)
        # expand: group range and geometry
        lat = B.make_cache(A, A, None, 64, 4, 8, 0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache, ok, lat, A, A, 6, 3, B.make_cache(A, A, None, 64, 4, 8, 3), stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache, ok, lat, A, A, 0, 8, B.make_cache(A, A, None, 64, 4, 8, 4), stream=0)
        _expect(B.GQLA_ERR_PAGE, B.gqla_expand_cache, ok, lat, A, A, 0, 8, B.make_cache(A, A, None, 64, 5, 8, 8), stream=0)
        _expect(B.GQLA_ERR_NULL, B.gqla_expand_cache, ok, B.make_cache(A, None, None, 64, 4, 8, 0), A, A, 0, 8,
                B.make_cache(A, A, None, 64, 4, 8, 8), stream=0)
        # expand scratch: both weight slices of the expanded groups, bf16; none for fp32
        assert B.gqla_expand_workspace_bytes(ok, 8) == 2 * 8 * 512 * 128 * 2
        assert B.gqla_expand_workspace_bytes(ok, 1) == 2 * 512 * 128 * 2
        assert B.gqla_expand_workspace_bytes(B.make_shape(2, 128, 8, 128, 512, 64, 1, B.GQLA_F32), 8) == 0
        full = B.make_cache(A, A, None, 64, 4, 8, 8)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache, ok, lat, A, A, 0, 8, full, None, 0, stream=0)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache, ok, lat, A, A, 0, 8, full, A, 2 * 8 * 512 * 128 * 2 - 1, stream=0)
        # the per-step cache updates: the tail expansion takes the same checks plus 1 <= tail_tokens <= page_size
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail, ok, lat, A, A, 0, 8, full, 0, A, 1 << 24, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail, ok, lat, A, A, 0, 8, full, 65, A, 1 << 24, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail, ok, lat, A, A, 6, 3, B.make_cache(A, A, None, 64, 4, 8, 3), 1, A, 1 << 24, stream=0)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache_tail, ok, lat, A, A, 0, 8, full, 2, None, 0, stream=0)
        # the weights repacked ahead of time: bf16 only, the slice inside the shape's groups, scratch large enough
        need8 = B.gqla_expand_workspace_bytes(ok, 8)
        _expect(B.GQLA_ERR_NULL, B.gqla_pack_expand_weights, ok, None, A, 0, 8, A, need8, stream=0)
        _expect(B.GQLA_ERR_NULL, B.gqla_pack_expand_weights, ok, A, A, 0, 8, None, need8, stream=0)
        _expect(B.GQLA_ERR_ALIGN, B.gqla_pack_expand_weights, ok, A, A + 8, 0, 8, A, need8, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_pack_expand_weights, ok, A, A, 6, 3, A, need8, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_pack_expand_weights, ok, A, A, 0, 0, A, need8, stream=0)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_pack_expand_weights, ok, A, A, 0, 8, A, need8 - 1, stream=0)
        f32 = B.make_shape(2, 8, 2, 16, 32, 8, 1, B.GQLA_F32)
        _expect(B.GQLA_ERR_DTYPE, B.gqla_pack_expand_weights, f32, A, A, 0, 2, A, 1 << 20, stream=0)
        _expect(B.GQLA_ERR_DTYPE, B.gqla_expand_cache_tail_packed, f32, B.make_cache(A, A, None, 8, 4, 8, 0), A, 2,
                B.make_cache(A, A, None, 8, 4, 8, 2), 1, packed_bytes=1 << 20, stream=0)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache_tail_packed, ok, lat, A, 8, full, 1, packed_bytes=need8 - 1, stream=0)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache_tail_packed, ok, lat, None, 8, full, 1, packed_bytes=0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail_packed, ok, lat, A, 8, full, 0, packed_bytes=need8, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail_packed, ok, lat, A, 8, full, 65, packed_bytes=need8, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail_packed, ok, lat, A, 3, full, 1, packed_bytes=need8, stream=0)   # the cache holds 8 groups
        _expect(B.GQLA_ERR_NULL, B.gqla_expand_cache_tail_packed, ok, B.make_cache(None, A, None, 64, 4, 8, 0), A, 8, full, 1, packed_bytes=need8, stream=0)
        # the variant with the scratch inside the library: the size limit and the shape checks come before anything
        # touches a device
        assert B.gqla_expand_cache_tail_static_max_workspace() == 2 << 20
        wide = B.make_shape(2, 128, 16, 128, 512, 64, 1, B.GQLA_BF16)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache_tail_static, wide, lat, A, A, 0, 16, B.make_cache(A, A, None, 64, 4, 8, 16), 1, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail_static, ok, lat, A, A, 0, 8, full, 0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail_static, ok, lat, A, A, 0, 0, full, 1, stream=0)
        _expect(B.GQLA_ERR_NULL, B.gqla_append_latent, ok, None, lat, stream=0)
        _expect(B.GQLA_ERR_NULL, B.gqla_append_latent, ok, A, B.make_cache(A, None, None, 64, 4, 8, 0), stream=0)
        _expect(B.GQLA_ERR_ALIGN, B.gqla_append_latent, ok, A + 4, lat, stream=0)
        _expect(B.GQLA_ERR_PAGE, B.gqla_append_latent, ok, A, B.make_cache(A, A, None, 48, 4, 8, 0), stream=0)
        _expect(B.GQLA_ERR_PAGE, B.gqla_append_latent, ok, A, B.make_cache(A, A, None, 64, 4, 7, 0), stream=0)
        # the 8-bit expanded cache: bf16 shapes only, positive finite scales, matching geometry
        f32 = B.make_shape(2, 8, 2, 16, 32, 8, 1, B.GQLA_F32)
        full8 = B.make_cache(A, A, None, 64, 4, 8, 8)
        _expect(B.GQLA_ERR_DTYPE, B.gqla_quantize_expanded, f32, B.make_cache(A, A, None, 8, 4, 8, 2), B.make_cache(A, A, None, 8, 4, 8, 2), 1.0, 1.0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_quantize_expanded, ok, full, full8, 0.0, 1.0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_quantize_expanded, ok, full, full8, 1.0, float("inf"), stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_quantize_expanded, ok, full, B.make_cache(A, A, None, 64, 4, 8, 4), 1.0, 1.0, stream=0)
        _expect(B.GQLA_ERR_PAGE, B.gqla_quantize_expanded, ok, full, B.make_cache(A, A, None, 64, 5, 8, 8), 1.0, 1.0, stream=0)
        _expect(B.GQLA_ERR_NULL, B.gqla_quantize_expanded, ok, B.make_cache(A, None, None, 64, 4, 8, 8), full8, 1.0, 1.0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_decode_gqa_fp8, ok, plan_g, A, A, full8, -1.0, 1.0, A, None, A, big, stream=0)
        _expect(B.GQLA_ERR_PLAN, B.gqla_decode_gqa_fp8, ok, plan_a, A, A, full8, 1.0, 1.0, A, None, A, big, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail_fp8, ok, lat, A, A, 0, 8, full8, 0, 1.0, 1.0, A, 1 << 24, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail_fp8, ok, lat, A, A, 0, 8, full8, 2, 1.0, 0.0, A, 1 << 24, stream=0)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache_tail_fp8, ok, lat, A, A, 0, 8, full8, 2, 1.0, 1.0, None, 0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_fp8, ok, lat, A, A, 0, 8, full8, 1.0, -2.0, A, 1 << 24, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_fp8, ok, lat, A, A, 4, 8, full8, 1.0, 1.0, A, 1 << 24, stream=0)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache_fp8, ok, lat, A, A, 0, 8, full8, 1.0, 1.0, None, 0, stream=0)
        _expect(B.GQLA_ERR_DTYPE, B.gqla_expand_cache_fp8, f32, B.make_cache(A, A, None, 8, 4, 8, 0), A, A, 0, 2,
                B.make_cache(A, A, None, 8, 4, 8, 2), 1.0, 1.0, A, 1 << 24, stream=0)
        assert B.gqla_expanded_fp8_bytes_per_token(8, 128, 64) == 2176 and B.gqla_expanded_fp8_bytes_per_token(4, 128, 64) == 1152
        # the 8-bit latent cache: the same rules
        lat8 = B.make_cache(A, A, None, 64, 4, 8, 0)
        _expect(B.GQLA_ERR_DTYPE, B.gqla_quantize_latent, f32, B.make_cache(A, A, None, 8, 4, 8, 0), B.make_cache(A, A, None, 8, 4, 8, 0), 1.0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_quantize_latent, ok, lat, lat8, 0.0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_quantize_latent, ok, lat, lat8, float("nan"), stream=0)
        _expect(B.GQLA_ERR_PAGE, B.gqla_quantize_latent, ok, lat, B.make_cache(A, A, None, 128, 4, 8, 0), 1.0, stream=0)
        _expect(B.GQLA_ERR_PAGE, B.gqla_quantize_latent, ok, lat, B.make_cache(A, A, None, 64, 4, 7, 0), 1.0, stream=0)
        _expect(B.GQLA_ERR_NULL, B.gqla_quantize_latent, ok, B.make_cache(A, None, None, 64, 4, 8, 0), lat8, 1.0, stream=0)
        _expect(B.GQLA_ERR_ALIGN, B.gqla_quantize_latent, ok, lat, B.make_cache(A + 8, A, None, 64, 4, 8, 0), 1.0, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_decode_absorb_fp8, ok, plan_a, A, A, lat8, -1.0, A, A, None, A, big, stream=0)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_decode_absorb_fp8, ok, plan_a, A, A, lat8, float("inf"), A, A, None, A, big, stream=0)
        _expect(B.GQLA_ERR_PLAN, B.gqla_decode_absorb_fp8, ok, plan_g, A, A, lat8, 1.0, A, A, None, A, big, stream=0)
        _expect(B.GQLA_ERR_WORKSPACE, B.gqla_decode_absorb_fp8, ok, plan_a, A, A, lat8, 1.0, A, A, None, A, big, stream=0)
        _expect(B.GQLA_ERR_SEQLEN, B.gqla_decode_absorb_fp8, ok, plan_a, A, A, B.make_cache(A, A, None, 64, 2, 8, 0), 1.0, A, A, None, A, big, stream=0)
        f32_plan = B.gqla_plan_create(f32, lens, 8, 256, B.GQLA_PATH_ABSORB)
        try:
            _expect(B.GQLA_ERR_DTYPE, B.gqla_decode_absorb_fp8, f32, f32_plan, A, A, B.make_cache(A, A, None, 8, 32, 64, 0), 1.0, A, A, None, A, big, stream=0)
        finally:
            B.gqla_plan_destroy(f32_plan)
        assert B.gqla_latent_fp8_bytes_per_token(512, 64) == 640
    finally:
        B.gqla_plan_destroy(plan_a)
        B.gqla_plan_destroy(plan_g)
    assert B.status_string(B.GQLA_OK) == "ok"


def test_empty_batch_is_ok_without_launch():
    sh = B.make_shape(0, 128, 8, 128, 512, 64, 1, B.GQLA_BF16)
    A = 0x10000
    B.gqla_absorb_query(sh, A, A, A, stream=0)      # returns GQLA_OK, launches nothing
    lat = B.make_cache(A, A, None, 64, 4, 8, 0)
    B.gqla_append_latent(sh, A, lat, stream=0)
    B.gqla_expand_cache_tail(sh, lat, A, A, 0, 8, B.make_cache(A, A, None, 64, 4, 8, 8), 1, A, 1 << 24, stream=0)
    p = B.gqla_plan_create(sh, [], 64, 256, B.GQLA_PATH_GQA)
    assert B.gqla_plan_num_chunks(p) == 0
    B.gqla_plan_destroy(p)


def test_path_estimate_matches_the_papers_model():
    """gqla_estimate_paths against the oracle's transcription of Sec. 4.2 and against the paper's own Table 2
    (H100: 989 TFLOP/s, 3.35 TB/s; H20: 148 TFLOP/s, 4.0 TB/s; canonical shape, L = 8192, B = 1)."""
    from oracle import roofline as R
    L = 8192
    for (peak, bw, g, s_q, want_path) in [
        (989e12, 3.35e12, 8, 1, B.GQLA_PATH_ABSORB),   # H100: absorb 2.82 us (memory) beats GQA 10.3 us
        (989e12, 3.35e12, 8, 2, B.GQLA_PATH_ABSORB),
        (148e12, 4.0e12, 8, 1, B.GQLA_PATH_GQA),       # H20: GQA 8.65 us beats absorb 15.42 us (compute)
        (148e12, 4.0e12, 8, 2, B.GQLA_PATH_GQA),
        (148e12, 4.0e12, 4, 1, B.GQLA_PATH_GQA),
        (2500e12, 8.0e12, 8, 1, B.GQLA_PATH_ABSORB),   # MI355X published peaks
    ]:
        sh = B.make_shape(1, 128, g, 128, 512, 64, s_q, B.GQLA_BF16)
        est = B.gqla_estimate_paths(sh, L, bw, peak)
        oa = R.operating_point(R.absorb_bytes(L, 512, 64), R.absorb_flops(L, 128, s_q, 512, 64), s_q, peak, bw)
        og = R.operating_point(R.gqa_bytes(L, g, 128, 64), R.gqa_flops(L, 128, s_q, 128, 64), s_q, peak, bw)
        assert est["absorb_bytes"] == R.absorb_bytes(L, 512, 64) and est["gqa_bytes"] == R.gqa_bytes(L, g, 128, 64)
        assert est["absorb_flops"] == R.absorb_flops(L, 128, s_q, 512, 64) and est["gqa_flops"] == R.gqa_flops(L, 128, s_q, 128, 64)
        assert abs(est["absorb_seconds"] - oa["step_s"]) <= 1e-15 and abs(est["gqa_seconds"] - og["step_s"]) <= 1e-15
        assert abs(est["absorb_intensity"] - R.absorb_intensity(128, s_q, 512, 64)) < 1e-9
        assert abs(est["gqa_intensity"] - R.gqa_intensity(128, g, s_q, 128, 64)) < 1e-9
        assert abs(est["ridge"] - R.ridge(peak, bw)) < 1e-9
        assert est["faster_path"] == want_path
    # the printed values of Table 2 (microseconds, rounded as printed)
    h20 = B.gqla_estimate_paths(B.make_shape(1, 128, 8, 128, 512, 64, 1, B.GQLA_BF16), L, 4.0e12, 148e12)
    assert abs(h20["absorb_seconds"] * 1e6 - 15.42) < 0.01 and abs(h20["gqa_seconds"] * 1e6 - 8.65) < 0.01
    h100 = B.gqla_estimate_paths(B.make_shape(1, 128, 8, 128, 512, 64, 1, B.GQLA_BF16), L, 3.35e12, 989e12)
    assert abs(h100["absorb_seconds"] * 1e6 - 2.82) < 0.01
    # argument checks
    sh = B.make_shape(1, 128, 8, 128, 512, 64, 1, B.GQLA_BF16)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_estimate_paths, sh, -1, 1.0, 1.0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_estimate_paths, sh, 10, 0.0, 1.0)


def test_calibrated_path_choice_matches_the_measured_operating_points():
    """gqla_select_path against the committed measurements (profiles/operating_points_bench.txt,
    profiles/batch_sweep_bench.txt and profiles/all_configs_bench.txt: microseconds of absorb_query + decode_absorb and
    of decode_gqa on one MI355X): predicted times within 25 % of every measured row, and the measured faster path
    wherever the two paths are more than 12 % apart (the model is good to about that per path)."""
    measured = [  # B, h_q, g, s_q, cached tokens, absorb us, gqa us
        (1, 128, 8, 1, 8192, 46.0, 33.7), (1, 128, 8, 2, 8192, 51.4, 37.7), (1, 128, 4, 1, 8192, 46.6, 25.7),
        (1, 128, 4, 2, 8192, 50.1, 35.8), (64, 128, 8, 1, 524288, 165.1, 327.2), (64, 128, 8, 2, 524288, 292.4, 337.0),
        (64, 128, 4, 1, 524288, 168.4, 189.0), (64, 128, 4, 2, 524288, 290.2, 190.7),
        (64, 64, 8, 1, 524288, 134.2, 324.6), (64, 64, 8, 2, 524288, 165.1, 326.5),   # 64 heads
        (32, 32, 8, 1, 131072, 46.1 + 7.5, 89.7),          # configs[1]; its absorb figure there is the decode call alone
        (128, 128, 8, 2, 2234929, 1208.2 + 12.0, 1536.2),  # configs[4], same remark
        # batch sweep, canonical shape, 8192 tokens per sequence
        (2, 128, 8, 1, 16384, 51.7, 36.7), (4, 128, 8, 1, 32768, 55.1, 42.2), (8, 128, 8, 1, 65536, 57.3, 58.3),
        (16, 128, 8, 1, 131072, 68.4, 94.8), (32, 128, 8, 1, 262144, 96.1, 171.7), (128, 128, 8, 1, 1048576, 310.0, 643.7),
        (2, 128, 8, 2, 16384, 52.8, 41.6), (4, 128, 8, 2, 32768, 56.4, 46.0), (8, 128, 8, 2, 65536, 64.9, 62.8),
        (16, 128, 8, 2, 131072, 91.5, 102.2), (32, 128, 8, 2, 262144, 153.1, 178.2), (128, 128, 8, 2, 1048576, 567.4, 644.7),
    ]
    for Bn, h_q, g, s_q, tokens, t_a, t_g in measured:
        ch = B.gqla_select_path(B.make_shape(Bn, h_q, g, 128, 512, 64, s_q, B.GQLA_BF16), tokens)
        assert abs(ch["absorb_seconds"] * 1e6 / t_a - 1.0) < 0.25, (Bn, g, s_q, ch["absorb_seconds"] * 1e6, t_a)
        assert abs(ch["gqa_seconds"] * 1e6 / t_g - 1.0) < 0.25, (Bn, g, s_q, ch["gqa_seconds"] * 1e6, t_g)
        if abs(t_a - t_g) / min(t_a, t_g) > 0.12:
            assert ch["faster_path"] == (B.GQLA_PATH_GQA if t_g < t_a else B.GQLA_PATH_ABSORB), (Bn, g, s_q)
    with pytest.raises(B.GqlaError):
        B.gqla_select_path(B.make_shape(1, 8, 2, 16, 32, 8, 1, B.GQLA_F32), 64)


def test_left_inverse_on_the_host_matches_the_oracle():
    """gqla_left_inverse (Cholesky of A^T A in double, host only) against the oracle's left inverse, on the tiny config
    and on a canonical-size group count; error codes for a rank that cannot be inverted."""
    from oracle import gqla_oracle as O
    rng = np.random.default_rng(12)
    for g, r_kv, d_h in ((2, 32, 16), (4, 64, 32)):
        w = rng.normal(size=(g, r_kv, d_h)).astype(np.float32) / np.sqrt(r_kv)
        sh = B.make_shape(1, g * 4, g, d_h, r_kv, 8, 1, B.GQLA_F32)
        got = B.gqla_left_inverse(sh, w)
        want = O.left_inverse_uk(w)
        assert got.shape == want.shape == (r_kv, g * d_h)
        assert np.max(np.abs(got - want)) <= 1e-5 * np.max(np.abs(want))
    # g d_h < r_kv: no left inverse
    _expect(B.GQLA_ERR_SHAPE, B.gqla_left_inverse, B.make_shape(1, 8, 1, 16, 32, 8, 1, B.GQLA_F32), np.zeros((1, 32, 16), np.float32))
    # rank-deficient keys (two identical rows of every W_UK[j])
    w = rng.normal(size=(2, 32, 16)).astype(np.float32)
    w[:, 1, :] = w[:, 0, :]
    _expect(B.GQLA_ERR_SHAPE, B.gqla_left_inverse, B.make_shape(1, 8, 2, 16, 32, 8, 1, B.GQLA_F32), w)


def test_step_ops_validate_on_the_host():
    """gqla_rope_step, gqla_compress_cache and gqla_output_projection reject bad arguments before any launch; the
    scratch size of the output projection follows the documented k-range rule."""
    A = 0x10000
    ok = B.make_shape(2, 32, 8, 128, 512, 64, 2, B.GQLA_BF16)
    _expect(B.GQLA_ERR_NULL, B.gqla_rope_step, ok, None, 10000.0, A, A, stream=0)
    _expect(B.GQLA_ERR_NULL, B.gqla_rope_step, ok, A, 10000.0, None, None, stream=0)
    _expect(B.GQLA_ERR_ALIGN, B.gqla_rope_step, ok, A, 10000.0, A + 8, A, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_rope_step, ok, A, 1.0, A, A, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_rope_step, ok, A, float("inf"), A, A, stream=0)
    # output projection: M = 4 rows, K = 4096
    _expect(B.GQLA_ERR_NULL, B.gqla_output_projection, ok, 4096, A, None, A, A, 1 << 30, stream=0)
    _expect(B.GQLA_ERR_ALIGN, B.gqla_output_projection, ok, 4096, A, A, A + 2, A, 1 << 30, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_output_projection, ok, 0, A, A, A, A, 1 << 30, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_output_projection, ok, 4000, A, A, A, A, 1 << 30, stream=0)          # not a multiple of 128
    _expect(B.GQLA_ERR_SHAPE, B.gqla_output_projection, B.make_shape(2, 1, 1, 128, 512, 64, 2, B.GQLA_BF16), 4096, A, A, A, A, 1 << 30, stream=0)  # K = 128
    need = B.gqla_output_projection_workspace_bytes(ok, 4096)
    # 32 column tiles x 1 row block -> 256 // 32 = 8 k-ranges of two 256-element pieces each
    assert need == 8 * 4 * 4096 * 4
    _expect(B.GQLA_ERR_NULL, B.gqla_output_projection, ok, 4096, A, A, A, None, 0, stream=0)
    _expect(B.GQLA_ERR_WORKSPACE, B.gqla_output_projection, ok, 4096, A, A, A, A, need - 1, stream=0)
    assert B.gqla_output_projection_workspace_bytes(ok, 4000) == 0
    assert B.gqla_output_projection_workspace_bytes(B.make_shape(2, 8, 2, 16, 32, 8, 1, B.GQLA_F32), 24) == 0
    # 7168 columns (56 tiles), K = 16384 (64 pieces): 256 // 56 = 4 ranges of 16 pieces
    big = B.make_shape(64, 128, 8, 128, 512, 64, 1, B.GQLA_BF16)
    assert B.gqla_output_projection_workspace_bytes(big, 7168) == 4 * 64 * 7168 * 4
    # compress: needs all groups, matching geometry, g d_h >= r_kv
    full = B.make_cache(A, A, None, 64, 4, 8, 8)
    lat = B.make_cache(A, A, None, 64, 4, 8, 0)
    ok8 = B.make_shape(2, 128, 8, 128, 512, 64, 1, B.GQLA_BF16)
    _expect(B.GQLA_ERR_NULL, B.gqla_compress_cache, ok8, full, None, lat, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_compress_cache, ok8, B.make_cache(A, A, None, 64, 4, 8, 4), A, lat, stream=0)
    _expect(B.GQLA_ERR_PAGE, B.gqla_compress_cache, ok8, full, A, B.make_cache(A, A, None, 64, 5, 8, 0), stream=0)
    _expect(B.GQLA_ERR_ALIGN, B.gqla_compress_cache, ok8, full, A + 4, lat, stream=0)
    # empty batch: nothing to do
    B.gqla_rope_step(B.make_shape(0, 32, 8, 128, 512, 64, 2, B.GQLA_BF16), A, 10000.0, A, A, stream=0)
    B.gqla_output_projection(B.make_shape(0, 32, 8, 128, 512, 64, 2, B.GQLA_BF16), 4096, A, A, A, None, 0, stream=0)


def test_value_dim_of_its_own_is_accepted_where_the_kernels_exist():
    """gqla_shape.d_v: 0 means d_h; on the absorb path bf16 takes d_h in {128, 192} and d_v in {128, 256}; what reads or
    writes a 16-bit expanded cache takes (d_h, d_v) = (128, 128) or (192, 256); the 8-bit expanded cache and the
    calibrated path choice take (128, 128) only."""
    A = 0x10000
    glm = B.make_shape(2, 20, 4, 192, 512, 64, 1, B.GQLA_BF16, 0.0, 256)
    lens = [300, 4000]
    p = B.gqla_plan_create(glm, lens, 64, 256, B.GQLA_PATH_ABSORB)
    pg = B.gqla_plan_create(glm, lens, 64, 256, B.GQLA_PATH_GQA)
    try:
        assert B.gqla_plan_num_chunks(p) > 0 and B.gqla_plan_num_chunks(pg) > 0
        # a plan made for another value dim does not fit
        other = B.make_shape(2, 20, 4, 192, 512, 64, 1, B.GQLA_BF16, 0.0, 128)
        lat = B.make_cache(A, A, None, 64, 63, 126, 0)
        _expect(B.GQLA_ERR_PLAN, B.gqla_decode_absorb, other, p, A, A, lat, A, A, None, A, 1 << 30, stream=0)
        # the GQA plan's workspace holds partials of d_v floats per row, in whole blocks of 32 rows
        n = B.gqla_plan_num_chunks(pg)
        assert B.gqla_plan_workspace_bytes(pg) >= n * 32 * 256 * 4
        # the 8-bit expanded cache has no kernels for this shape
        exp8 = B.make_cache(A, A, None, 64, 63, 126, 4)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_decode_gqa_fp8, glm, pg, A, A, exp8, 1.0, 1.0, A, None, A, 1 << 30, stream=0)
    finally:
        B.gqla_plan_destroy(p)
        B.gqla_plan_destroy(pg)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_plan_create, B.make_shape(2, 20, 4, 160, 512, 64, 1, B.GQLA_BF16), lens, 64, 256, B.GQLA_PATH_ABSORB)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_plan_create, B.make_shape(2, 20, 4, 128, 512, 64, 1, B.GQLA_BF16, 0.0, 192), lens, 64, 256, B.GQLA_PATH_ABSORB)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_plan_create, B.make_shape(2, 20, 4, 192, 512, 64, 1, B.GQLA_BF16), lens, 64, 256, B.GQLA_PATH_ABSORB)  # d_v = d_h = 192
    # mixed pairs exist on the absorb path only
    for d_h, d_v in ((128, 256), (192, 128)):
        mixed = B.make_shape(2, 32, 8, d_h, 512, 64, 1, B.GQLA_BF16, 0.0, d_v)
        pm = B.gqla_plan_create(mixed, lens, 64, 256, B.GQLA_PATH_ABSORB)
        B.gqla_plan_destroy(pm)
        _expect(B.GQLA_ERR_SHAPE, B.gqla_plan_create, mixed, lens, 64, 256, B.GQLA_PATH_GQA)
        assert B.gqla_expand_workspace_bytes(mixed, 8) == 0
    lat = B.make_cache(A, A, None, 64, 4, 8, 0)
    full = B.make_cache(A, A, None, 64, 4, 8, 4)
    assert B.gqla_expand_workspace_bytes(glm, 4) == 4 * 512 * (192 + 256) * 2
    _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache, glm, lat, A, A, 0, 4, full, A, 4 * 512 * (192 + 256) * 2 - 1, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache, glm, lat, A, A, 2, 3, B.make_cache(A, A, None, 64, 4, 8, 3), A, 1 << 24, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_fp8, glm, lat, A, A, 0, 4, full, 1.0, 1.0, A, 1 << 24, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_expand_cache_tail_fp8, glm, lat, A, A, 0, 4, full, 1, 1.0, 1.0, A, 1 << 24, stream=0)
    _expect(B.GQLA_ERR_SHAPE, B.gqla_quantize_expanded, glm, full, full, 1.0, 1.0, stream=0)
    # the variant with its scratch inside the library holds 4 groups of this shape, not 5
    glm5 = B.make_shape(2, 20, 5, 192, 512, 64, 1, B.GQLA_BF16, 0.0, 256)
    _expect(B.GQLA_ERR_WORKSPACE, B.gqla_expand_cache_tail_static, glm5, lat, A, A, 0, 5, B.make_cache(A, A, None, 64, 4, 8, 5), 1, stream=0)
    # compress needs g d_h >= r_kv: 2 groups of 192 are too few
    _expect(B.GQLA_ERR_SHAPE, B.gqla_compress_cache, B.make_shape(2, 20, 2, 192, 512, 64, 1, B.GQLA_BF16, 0.0, 256),
            B.make_cache(A, A, None, 64, 4, 8, 2), A, lat, stream=0)
    # sizes and offsets with a value dim of its own, against the oracle's layout
    from oracle import layout as Lay
    P, gc, d_h, d_v, d_r = 64, 4, 192, 256, 64
    assert B.gqla_expanded_elems_per_token_dv(gc, d_h, d_v, d_r) == Lay.expanded_elems_per_token(gc, d_h, d_r, d_v) == 4 * 448 + 64
    assert B.gqla_expanded_elems_per_token_dv(8, 128, 128, 64) == B.gqla_expanded_elems_per_token(8, 128, 64)
    for page, j, slot in ((0, 0, 0), (3, 2, 17), (1, 3, 63)):
        for d in (0, 7, 8, 191):
            assert B.gqla_expanded_k_offset_dv(page, j, slot, d, P, gc, d_h, d_v, d_r) == Lay.expanded_k_offset(page, j, slot, d, P, gc, d_h, d_r, d_v)
        for d in (0, 5, 192, 255):
            assert B.gqla_expanded_v_offset_dv(page, j, slot, d, P, gc, d_h, d_v, d_r) == Lay.expanded_v_offset(page, j, slot, d, P, gc, d_h, d_r, d_v)
        for d in (0, 9, 63):
            assert B.gqla_expanded_kr_offset_dv(page, slot, d, P, gc, d_h, d_v, d_r) == Lay.expanded_kr_offset(page, slot, d, P, gc, d_h, d_r, d_v)
        assert B.gqla_expanded_v_offset_dv(page, j, slot, 100, P, gc, 128, 128, d_r) == B.gqla_expanded_v_offset(page, j, slot, 100, P, gc, 128, d_r)
        assert B.gqla_expanded_kr_offset_dv(page, slot, 9, P, gc, 128, 128, d_r) == B.gqla_expanded_kr_offset(page, slot, 9, P, gc, 128, d_r)
    # W^O takes h_q * d_v columns: 20 * 256 = 5120 = 20 pieces of 256
    # 32 column tiles -> 8 ranges wanted -> 3 pieces each -> 7 ranges (the last of 2 pieces)
    assert B.gqla_output_projection_workspace_bytes(glm, 4096) == 7 * 2 * 4096 * 4
