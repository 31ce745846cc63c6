"""The entry point for callers that cannot allocate (gqla_expand_cache_tail_static): through the C ABI, its output
must equal gqla_expand_cache_tail's bit for bit, on two calls in a row of which the second has the smaller input (the
library's fixed scratch array still holds the first call's content then)."""
import numpy as np
import pytest
import torch

import synth_inputs as S

pytestmark = pytest.mark.gpu


def _run_pair(cfg, lens, groups, group_begin, tail):
    """(pool from gqla_expand_cache_tail, pool from gqla_expand_cache_tail_static) for one case."""
    from paper_2605_15250_amd import binding as B
    from paper_2605_15250_amd.harness import Decoder, build_latent_pool, to_device
    lens = np.asarray(lens, np.int32)
    table, num_pages = S.page_table(cfg.with_(L=0), lens)
    rows = [S.sequence_rows(cfg, b, lens[b]) for b in range(cfg.B)]
    dec = Decoder(cfg, lens, table, num_pages, groups=groups, group_begin=group_begin)
    try:
        dec.latent_pool = build_latent_pool(cfg, lens, table, num_pages, lambda b, L: rows[b])
        w_uk, w_uv = S.weights(cfg)
        d_w_uk, d_w_uv = to_device(w_uk, cfg.dtype), to_device(w_uv, cfg.dtype)
        dec.alloc_expanded()
        dec.expand_tail(d_w_uk, d_w_uv, tail)
        torch.cuda.synchronize()
        ref = dec.expanded_pool.clone()
        dec.alloc_expanded()
        B.gqla_expand_cache_tail_static(dec.shape, dec.latent_cache(), d_w_uk, d_w_uv, group_begin, groups, dec.expanded_cache(), tail)
        torch.cuda.synchronize()
        got = dec.expanded_pool.clone()
        written = int((~torch.isnan(got.float())).sum().item())
        per_tok = 2 * groups * cfg.d_h + cfg.d_r
        assert written == int(np.minimum(lens, tail).sum()) * per_tok, "the static variant wrote a different set of slots"
        return ref, got
    finally:
        dec.close()


def _same_bits(a, b):
    view = torch.int16 if a.dtype == torch.bfloat16 else torch.int32
    return torch.equal(a.view(view), b.view(view))


def test_static_scratch_variant_equals_workspace_variant_twice_in_a_row():
    from paper_2605_15250_amd import binding as B
    assert B.gqla_expand_cache_tail_static_max_workspace() == 2 << 20
    # first call: all 8 groups (the whole 2 MiB of scratch), 5 sequences, 3 tail tokens
    big = S.CONFIGS["C3"].with_(B=5, L=0, paged=True, seed=4242)
    ref, got = _run_pair(big, [300, 2, 64, 129, 1000], groups=8, group_begin=0, tail=3)
    assert _same_bits(ref, got), "first call (8 groups)"
    # second call, smaller input: a 2-group slice of other weights, 2 sequences, 1 tail token -- the scratch still
    # holds the first call's 8 groups behind the part this call rewrites
    small = S.CONFIGS["C3"].with_(B=2, s_q=1, L=0, paged=True, seed=777)
    ref, got = _run_pair(small, [70, 1], groups=2, group_begin=5, tail=1)
    assert _same_bits(ref, got), "second call (2-group slice)"
    # and the fp32 kernels (no scratch at all) go through the same entry point
    tiny = S.CONFIGS["C0"].with_(B=3, L=0, paged=True, page_size=8, s_q=2, seed=99)
    ref, got = _run_pair(tiny, [40, 7, 2], groups=2, group_begin=0, tail=2)
    assert _same_bits(ref, got), "fp32 call"


def test_static_scratch_variant_rejects_a_slice_beyond_its_scratch():
    from paper_2605_15250_amd import binding as B
    from paper_2605_15250_amd.harness import Decoder
    cfg = S.CONFIGS["C3"].with_(B=1, L=0, g=16, paged=True, seed=1)
    lens = np.array([100], np.int32)
    table, num_pages = S.page_table(cfg.with_(L=0), lens)
    dec = Decoder(cfg, lens, table, num_pages)
    try:
        dec.latent_pool = torch.zeros((num_pages, cfg.page_size, cfg.r_kv + cfg.d_r), dtype=torch.bfloat16, device="cuda")
        dec.alloc_expanded()
        w = torch.zeros((16, cfg.r_kv, cfg.d_h), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(B.GqlaError) as ei:
            B.gqla_expand_cache_tail_static(dec.shape, dec.latent_cache(), w, w, 0, 16, dec.expanded_cache(), 1)
        assert ei.value.status == B.GQLA_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert bool(torch.isnan(dec.expanded_pool.float()).all()), "a rejected call must not launch anything"
    finally:
        dec.close()
