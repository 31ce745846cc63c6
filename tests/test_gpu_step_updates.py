"""GPU parity of the per-step cache updates (append of the step's latent rows, expansion of just those positions)
against the CPU oracle, and the decode step built from them: prefix cached and expanded earlier, then append +
tail expansion + GQA decode (and absorb decode on the appended latent cache)."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import gqla_oracle as O
from oracle import layout as Lay
from test_gpu_parity import Case, check, host

pytestmark = pytest.mark.gpu


def _prefix_pool(case, s_q):
    """Latent pool holding only the tokens cached before the step (positions < L_b - s_q); the rest NaN."""
    from paper_2605_15250_amd.harness import build_latent_pool
    cfg = case.cfg
    before = np.maximum(case.lens - s_q, 0).astype(np.int32)
    return build_latent_pool(cfg, before, case.table, case.num_pages, lambda b, L: case.rows[b][:L]), before


@pytest.mark.parametrize("key,lens,page_size,s_q", [
    ("C3", [300, 2, 64, 129, 1000], 64, 2),     # L == s_q (nothing cached before), a step that starts a new page (129 -> slot 0 of page 2)
    ("C3", [65, 64, 1], 64, 1),                 # s_q = 1; a single-token sequence
    ("C0", [40, 7, 2, 17], 8, 2),               # fp32 kernels, 8-token pages
])
def test_append_then_tail_expand_then_decode(key, lens, page_size, s_q):
    cfg = S.CONFIGS[key].with_(B=len(lens), s_q=s_q, L=0, paged=True, page_size=page_size, seed=2718 + s_q)
    case = Case(cfg, lens=lens)
    dec = case.dec
    try:
        W = cfg.r_kv + cfg.d_r
        per_tok = 2 * cfg.g * cfg.d_h + cfg.d_r
        full_lens = dec.d_lens
        # -- before the step: prefix in the latent cache, prefix expanded in one shot
        dec.latent_pool, before = _prefix_pool(case, s_q)
        dec.d_lens = torch.from_numpy(before).cuda()
        dec.alloc_expanded()
        dec.expand(case.d_w_uk, case.d_w_uv)
        torch.cuda.synchronize()
        nan_before = int(torch.isnan(dec.expanded_pool.float()).sum().item())
        assert nan_before == dec.expanded_pool.numel() - int(before.sum()) * per_tok
        # -- the step: lengths now count the new tokens; append their rows
        dec.d_lens = full_lens
        new_rows = np.stack([case.rows[b][int(case.lens[b]) - s_q:] for b in range(cfg.B)])   # [B, s_q, W]
        dec.append_latent(case.to_device(new_rows, cfg.dtype))
        torch.cuda.synchronize()
        ref_pool = Lay.pack_latent_pool(case.rows, case.table, case.num_pages, cfg.page_size, W)
        assert np.array_equal(host(dec.latent_pool).reshape(ref_pool.shape), ref_pool, equal_nan=True), "latent cache after the append"
        # -- expansion of the step's positions only
        dec.expand_tail(case.d_w_uk, case.d_w_uv, s_q)
        torch.cuda.synchronize()
        pool_h = host(dec.expanded_pool)
        assert int(np.isnan(pool_h).sum()) == pool_h.size - int(case.lens.sum()) * per_tok
        exp_ref = {}
        for b in range(cfg.B):
            KC, V = O.expand_latent(case.c(b), case.w_uk, case.w_uv)
            exp_ref[b] = (KC, V)
            k2, v2, r2 = Lay.unpack_expanded_seq(pool_h, case.table[b], case.lens[b], cfg.page_size, cfg.g, cfg.d_h, cfg.d_r)
            check("K_C seq %d (prefix one-shot + tail)" % b, k2, KC, cfg.dtype, scale_abs=2.0)
            check("V seq %d (prefix one-shot + tail)" % b, v2, V, cfg.dtype, scale_abs=2.0)
            assert np.array_equal(r2, case.kR(b)), "k_R must be copied bit for bit"
        # the same positions from a one-shot expansion of the whole cache: identical bits
        tail_pool = dec.expanded_pool.clone()
        dec.alloc_expanded()
        dec.expand(case.d_w_uk, case.d_w_uv)
        torch.cuda.synchronize()
        assert torch.equal(tail_pool.view(torch.uint8), dec.expanded_pool.view(torch.uint8)), \
            "tail expansion and one-shot expansion disagree in some bit"
        # -- the decode step on the updated caches
        dec.expanded_pool = tail_pool
        out_g, _ = dec.decode_gqa(case.d_q_c, case.d_q_r)
        q_hat = dec.absorb_query(case.d_q_c, case.d_w_uk)
        out_a, _ = dec.decode_absorb(q_hat, case.d_q_r, case.d_w_uv)
        torch.cuda.synchronize()
        ref = np.stack([O.decode_gqa(case.q_c[b], case.q_r[b], exp_ref[b][0], exp_ref[b][1], case.kR(b))[0] for b in range(cfg.B)])
        check("decode_gqa after append + tail expansion", host(out_g), ref, cfg.dtype)
        check("decode_absorb after append", host(out_a), ref, cfg.dtype)
    finally:
        case.close()


def test_tail_expand_of_a_group_slice():
    """One rank's share under head-axis tensor parallelism: 2 of 8 groups, 3 tail tokens; one sequence is shorter than
    the tail (its positions below 0 do not exist and nothing is written for them)."""
    cfg = S.CONFIGS["C3"].with_(B=4, L=0, paged=True, seed=1618)
    case = Case(cfg, lens=[200, 3, 70, 2], groups=2, group_begin=5)
    dec = case.dec
    try:
        tail, gc, j0 = 3, 2, 5
        per_tok = 2 * gc * cfg.d_h + cfg.d_r
        dec.alloc_expanded()
        dec.expand_tail(case.d_w_uk, case.d_w_uv, tail)
        torch.cuda.synchronize()
        pool_h = host(dec.expanded_pool)
        assert int(np.isnan(pool_h).sum()) == pool_h.size - int(np.minimum(case.lens, tail).sum()) * per_tok
        for b in range(cfg.B):
            L = int(case.lens[b])
            KC, V = O.expand_latent(case.c(b), case.w_uk[j0:j0 + gc], case.w_uv[j0:j0 + gc])
            k2, v2, r2 = Lay.unpack_expanded_seq(pool_h, case.table[b], L, cfg.page_size, gc, cfg.d_h, cfg.d_r)
            lo = max(L - tail, 0)
            assert np.isnan(k2[:lo]).all() and np.isnan(v2[:lo]).all() and np.isnan(r2[:lo]).all()
            check("K_C tail seq %d" % b, k2[lo:], KC[lo:], cfg.dtype, scale_abs=2.0)
            check("V tail seq %d" % b, v2[lo:], V[lo:], cfg.dtype, scale_abs=2.0)
            assert np.array_equal(r2[lo:], case.kR(b)[lo:])
    finally:
        case.close()
