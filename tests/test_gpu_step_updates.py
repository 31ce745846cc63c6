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
            check("K_C seq %d (prefix one-shot + tail)" % b, k2, KC, cfg.dtype)
            check("V seq %d (prefix one-shot + tail)" % b, v2, V, cfg.dtype)
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
            check("K_C tail seq %d" % b, k2[lo:], KC[lo:], cfg.dtype)
            check("V tail seq %d" % b, v2[lo:], V[lo:], cfg.dtype)
            assert np.array_equal(r2[lo:], case.kR(b)[lo:])
    finally:
        case.close()


@pytest.mark.parametrize("dims,groups,group_begin,lens,tail", [
    ((128, 128), 8, 0, [200, 3, 70, 2, 1000], 2),
    ((128, 128), 2, 5, [200, 3, 70, 2], 3),           # a group slice: the packed copy holds the slice's groups from 0
    ((192, 256), 4, 0, [130, 64, 1], 1),              # the MLA checkpoint's dims (Sec. 3.2.2)
])
def test_tail_expand_from_packed_weights_is_bit_identical(dims, groups, group_begin, lens, tail):
    """gqla_pack_expand_weights once, then gqla_expand_cache_tail_packed (a serving loop's form of the step's expansion):
    the same bits as gqla_expand_cache_tail, which repacks on every call, and nothing else written; the packed copy
    serves a second call, on other lengths, unchanged."""
    from paper_2605_15250_amd import binding as B
    d_h, d_v = dims
    if dims == (128, 128):
        cfg = S.CONFIGS["C3"].with_(B=len(lens), L=0, paged=True, seed=2718)
    else:
        cfg = S.CONFIGS["C2"].with_(B=len(lens), h_q=20, g=4, d_h=d_h, d_v=d_v, s_q=1, L=0, paged=True, seed=2719)
    case = Case(cfg, lens=lens, groups=groups, group_begin=group_begin)
    dec = case.dec
    try:
        dec.alloc_expanded()
        dec.expand_tail(case.d_w_uk, case.d_w_uv, tail)
        torch.cuda.synchronize()
        want = dec.expanded_pool.clone()
        packed = dec.pack_expand_weights(case.d_w_uk, case.d_w_uv)
        snapshot = packed.clone()
        for _ in range(2):
            dec.alloc_expanded()
            dec.expand_tail_packed(tail)
            torch.cuda.synchronize()
            assert torch.equal(dec.expanded_pool.view(torch.uint8), want.view(torch.uint8)), "packed and unpacked tail expansion differ"
        assert torch.equal(packed, snapshot), "the packed weights are read-only for the expansion"
        # the packed copy does not depend on the cache: one token fewer per sequence, same copy
        shorter = np.maximum(np.asarray(lens) - 1, 0).astype(np.int32)
        dec.d_lens.copy_(torch.from_numpy(shorter))
        dec.alloc_expanded()
        dec.expand_tail(case.d_w_uk, case.d_w_uv, tail)
        torch.cuda.synchronize()
        want2 = dec.expanded_pool.clone()
        dec.alloc_expanded()
        dec.expand_tail_packed(tail)
        torch.cuda.synchronize()
        assert torch.equal(dec.expanded_pool.view(torch.uint8), want2.view(torch.uint8))
    finally:
        case.close()


@pytest.mark.parametrize("key,lens,page_size", [
    ("C3", [300, 2, 129, 1000], 64),
    ("C3", [257, 128, 70], 128),             # 128-token pages: a workgroup's two 64-token halves share a page
    ("C0", [40, 7, 17], 8),
])
def test_compress_is_the_reverse_cache_switch(key, lens, page_size):
    """Sec. 3.1 (the cache is converted once, in either direction): expanded cache -> latent cache through the left inverse of the stacked
    key up-projection.  Isolated: GPU and oracle both consume the oracle's expansion rounded to the storage type and
    the same (rounded) left inverse.  Round trip on the GPU: expand, compress, decode on the recovered latent."""
    from paper_2605_15250_amd import binding as B
    if key == "C0":
        cfg = S.CONFIGS[key].with_(B=len(lens), L=0, paged=True, page_size=page_size, seed=3141, g=4, h_q=8)   # g d_h = 64 >= r_kv = 32
    else:
        cfg = S.CONFIGS[key].with_(B=len(lens), L=0, paged=True, page_size=page_size, seed=3141)
    case = Case(cfg, lens=lens)
    dec = case.dec
    try:
        W = cfg.r_kv + cfg.d_r
        w_inv = B.gqla_left_inverse(dec.shape, case.w_uk)                 # host, fp32
        w_inv_q = S.quantize(w_inv, cfg.dtype)
        d_w_inv = case.to_device(w_inv_q, cfg.dtype)
        KCq, Vq, kR = [], [], []
        for b in range(cfg.B):
            KC, V = O.expand_latent(case.c(b), case.w_uk, case.w_uv)
            KCq.append(S.quantize(KC, cfg.dtype)); Vq.append(S.quantize(V, cfg.dtype)); kR.append(case.kR(b))
        dec.expanded_pool = case.to_device(Lay.pack_expanded_pool(KCq, Vq, kR, case.table, case.num_pages, cfg.page_size, fill=0.0), cfg.dtype)
        truth = dec.latent_pool
        dec.latent_pool = torch.full_like(truth, float("nan"))
        dec.compress(d_w_inv)
        torch.cuda.synchronize()
        got = host(dec.latent_pool).reshape(case.num_pages, cfg.page_size, W)
        assert int(np.isnan(got).sum()) == got.size - int(case.lens.sum()) * W      # nothing beyond the tokens is written
        for b in range(cfg.B):
            L = int(case.lens[b])
            t = np.arange(L)
            rows = got[case.table[b][t // cfg.page_size], t % cfg.page_size]
            ref = KCq[b].reshape(L, -1).astype(np.float64) @ w_inv_q.astype(np.float64).T
            check("compress c_kv seq %d" % b, rows[:, :cfg.r_kv], ref, cfg.dtype)
            assert np.array_equal(rows[:, cfg.r_kv:], case.kR(b)), "k_R must be copied bit for bit"
            # and it is the latent again, up to what the 16-bit roundings of the keys and of the left inverse cost
            err = np.linalg.norm(rows[:, :cfg.r_kv] - case.c(b)) / np.linalg.norm(case.c(b))
            print("recovered latent vs the original, seq %d: rel_l2 %.3e" % (b, err), flush=True)
            assert err < (2e-2 if cfg.dtype == "bf16" else 1e-4)
        # round trip on the GPU: the decode on the recovered latent cache
        q_hat = dec.absorb_query(case.d_q_c, case.d_w_uk)
        out, _ = dec.decode_absorb(q_hat, case.d_q_r, case.d_w_uv)
        torch.cuda.synchronize()
        ref_o = np.stack([O.decode_gqa(case.q_c[b], case.q_r[b], *O.expand_latent(case.c(b), case.w_uk, case.w_uv), case.kR(b))[0]
                          for b in range(cfg.B)])
        o = host(out)
        rl = float(np.linalg.norm(o - ref_o) / np.linalg.norm(ref_o))
        print("decode on the recovered latent vs the exact decode: rel_l2 %.3e" % rl, flush=True)
        assert np.isfinite(o).all() and rl < (3e-2 if cfg.dtype == "bf16" else 1e-4)
    finally:
        case.close()


@pytest.mark.parametrize("key,use_table", [("C3", True), ("C3", False), ("C0", True)])
def test_device_length_beyond_the_table_row_writes_nothing(key, use_table):
    """The cache-update calls read L_b on the device, where the host cannot check it.  A length whose step positions
    fall beyond max_pages * page_size must write nothing: not through the entries that follow the sequence's table row
    (the next sequence's row, or whatever lies behind the last one), and, without a table, not into the next
    sequence's pages."""
    from paper_2605_15250_amd.harness import Decoder
    page_size = 64 if key == "C3" else 8
    cfg = S.CONFIGS[key].with_(B=3, s_q=2, L=0, paged=True, page_size=page_size, seed=5150)
    lens = np.array([3 * page_size, 2 * page_size, 3 * page_size], dtype=np.int32)
    table, num_pages = S.page_table(cfg, lens)
    dec = Decoder(cfg, lens, table, num_pages, use_page_table=use_table)
    if not use_table:
        dec.num_pages = cfg.B * dec.max_pages
    try:
        W = cfg.r_kv + cfg.d_r
        tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        dec.latent_pool = torch.full((dec.num_pages, cfg.page_size, W), float("nan"), dtype=tdt, device="cuda")
        dec.alloc_expanded()
        # sequence 0 claims a length one page beyond its table row, the last sequence one far beyond the whole table
        bad = lens.copy()
        bad[0] = dec.max_pages * page_size + 2
        bad[2] = (dec.max_pages + 40) * page_size + 1
        dec.d_lens = torch.from_numpy(bad).cuda()
        rows = torch.ones((cfg.B, cfg.s_q, W), dtype=tdt, device="cuda")
        w_uk, w_uv = S.weights(cfg)
        from paper_2605_15250_amd.harness import to_device
        dec.append_latent(rows)
        dec.expand_tail(to_device(w_uk, cfg.dtype), to_device(w_uv, cfg.dtype), cfg.s_q)
        torch.cuda.synchronize()
        lat = dec.latent_pool.float().cpu().numpy()
        # only sequence 1 (the honest one) received its two rows
        written = np.argwhere(~np.isnan(lat).all(axis=2))
        pg1 = int(table[1][(lens[1] - 1) // page_size]) if use_table else 1 * dec.max_pages + (int(lens[1]) - 1) // page_size
        expect = {(pg1, (int(lens[1]) - 2) % page_size), (pg1, (int(lens[1]) - 1) % page_size)}
        assert {tuple(int(v) for v in x) for x in written} == expect, written
        per_tok = 2 * cfg.g * cfg.d_h + cfg.d_r
        exp = dec.expanded_pool.float().cpu().numpy()
        assert int((~np.isnan(exp)).sum()) == 2 * per_tok
    finally:
        dec.close()
