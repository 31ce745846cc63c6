"""GPU parity of the 8-bit latent cache of the MQA-absorb path: the quantising cache switch bit for bit against the
oracle's quantiser and page format, and the decode over such a cache against the oracle's MQA-absorb decode (Sec. 3.1) on
the dequantised latent.  Both sides consume the same codes, so the decode is held to the plain 16-bit tolerance."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import fp8_cache as F8
from oracle import gqla_oracle as O
from test_gpu_parity import Case, check, host, rel_l2

pytestmark = pytest.mark.gpu


def _bf16_bits(x):
    """16-bit patterns of fp32 values that are representable in bf16."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def _oracle_pool(case, c_scale, fill=0xAA):
    cfg = case.cfg
    codes = [F8.quantize_tensor(case.c(b), c_scale) for b in range(cfg.B)]
    pool = F8.pack_latent_fp8_pool(codes, [_bf16_bits(case.kR(b)) for b in range(cfg.B)], case.table, case.num_pages,
                                   cfg.page_size, fill=fill)
    return codes, pool


def _decode_and_check(case, c_scale, codes, label):
    cfg, dec = case.cfg, case.dec
    q_hat = dec.absorb_query(case.d_q_c, case.d_w_uk)
    out, lse = dec.decode_absorb_fp8(q_hat, case.d_q_r, c_scale, case.d_w_uv)
    torch.cuda.synchronize()
    q_hat_h = host(q_hat)
    ref_o, ref_l, exact = [], [], []
    for b in range(cfg.B):
        c_deq = F8.dequantize_e4m3(codes[b]) * float(np.float32(c_scale))
        o, l = O.decode_absorb(q_hat_h[b], case.q_r[b], c_deq, case.kR(b), case.w_uv, d_h=cfg.d_h)
        ref_o.append(o); ref_l.append(l)
        exact.append(O.decode_absorb(q_hat_h[b], case.q_r[b], case.c(b), case.kR(b), case.w_uv, d_h=cfg.d_h)[0])
    check(label, host(out), np.stack(ref_o), cfg.dtype)
    check(label + " lse", host(lse), np.stack(ref_l), cfg.dtype)
    print("8-bit latent vs the 16-bit latent (what the quantisation itself costs): rel_l2 %.3e"
          % rel_l2(np.stack(ref_o), np.stack(exact)), flush=True)
    return host(out)


@pytest.mark.parametrize("h_q,g,s_q,lens,paged,cp,c_scale", [
    (128, 8, 2, [300, 2, 129, 65], True, (0, 0), 1.0),      # 256 rows per sequence, ragged tails, L == s_q
    (128, 8, 1, [513, 40], False, (1, 0), 0.37),            # contiguous pages, one-page chunks, a scale that is no power of two
    (16, 8, 1, [777, 40], True, (0, 0), 2.5),               # 16 rows: four waves share them
    (16, 4, 2, [2, 300, 1029], True, (1, 0), 0.02),         # 32 shared rows; a small scale: part of the latent saturates at 448
    (48, 8, 1, [700, 64, 1], True, (2, 0), 0.75),           # 48 rows: the second wave half padding, the last two without rows
    (8, 8, 1, [130], False, (0, 0), 1.0),                   # 8 rows
])
@pytest.mark.parametrize("num_cus", [256, 2])   # few chunks on a whole chip: every 32 rows get a workgroup; a sliver: 128 rows share one
def test_fp8_latent_quantise_and_decode(h_q, g, s_q, lens, paged, cp, c_scale, num_cus):
    cfg = S.CONFIGS["C2"].with_(B=len(lens), h_q=h_q, g=g, s_q=s_q, L=0, paged=paged, seed=990 + h_q + s_q)
    case = Case(cfg, lens=lens, use_page_table=paged, chunk_pages=cp, num_cus=num_cus)
    dec = case.dec
    try:
        codes, ref_pool = _oracle_pool(case, c_scale)
        # -- the quantising cache switch, bit for bit (bytes no token owns keep the fill pattern)
        dec.alloc_latent_fp8(fill=0xAA)
        dec.quantize_latent(c_scale)
        torch.cuda.synchronize()
        got_pool = dec.latent_fp8_pool.cpu().numpy()
        assert got_pool.shape == ref_pool.shape
        assert np.array_equal(got_pool, ref_pool), "%d of %d bytes differ" % (int((got_pool != ref_pool).sum()), got_pool.size)
        # -- decode over the oracle-packed cache
        dec.latent_fp8_pool = torch.from_numpy(ref_pool).cuda()
        _decode_and_check(case, c_scale, codes, "decode_absorb_fp8")
    finally:
        case.close()


def test_fp8_latent_unowned_slots_do_not_matter():
    """Slots no token owns may hold anything (here: the NaN code in every byte, NaN patterns in the k_R plane): the
    output is bit for bit the one over a zero-filled pool."""
    cfg = S.CONFIGS["C2"].with_(B=3, h_q=128, g=8, s_q=2, L=0, paged=True, seed=993)
    case = Case(cfg, lens=[200, 2, 65])
    dec = case.dec
    try:
        outs = []
        for fill in (0x00, 0xFF):
            codes, pool = _oracle_pool(case, 1.0, fill=fill)
            dec.latent_fp8_pool = torch.from_numpy(pool).cuda()
            outs.append(_decode_and_check(case, 1.0, codes, "decode_absorb_fp8, fill %#x" % fill))
        assert np.array_equal(outs[0], outs[1])
    finally:
        case.close()


def test_fp8_latent_page_id_outside_the_pool():
    """A page id outside the pool makes that page's tokens contribute nothing (as for the 16-bit cache): the result is
    the decode of the sequence with those tokens masked, and nothing is read out of bounds."""
    cfg = S.CONFIGS["C2"].with_(B=2, h_q=128, g=8, s_q=1, L=0, paged=True, seed=994)
    case = Case(cfg, lens=[64 * 5, 64 * 3])
    dec = case.dec
    try:
        codes, pool = _oracle_pool(case, 1.0)
        dec.latent_fp8_pool = torch.from_numpy(pool).cuda()
        bad = case.table.copy()
        bad[0, 2] = case.num_pages + 7      # third page of sequence 0
        bad[1, 0] = -1                      # first page of sequence 1
        dec.d_table = torch.from_numpy(bad).cuda()
        q_hat = dec.absorb_query(case.d_q_c, case.d_w_uk)
        out, lse = dec.decode_absorb_fp8(q_hat, case.d_q_r, 1.0, case.d_w_uv)
        torch.cuda.synchronize()
        q_hat_h = host(q_hat)
        P = cfg.page_size
        keep = [np.r_[0:2 * P, 3 * P:5 * P], np.r_[P:3 * P]]
        ref_o, ref_l = [], []
        for b in range(cfg.B):
            # the masked tokens all lie before the last one, so the bottom-right causal mask of the kept ones is unchanged
            c_deq = F8.dequantize_e4m3(codes[b])[keep[b]]
            o, l = O.decode_absorb(q_hat_h[b], case.q_r[b], c_deq, case.kR(b)[keep[b]], case.w_uv, d_h=cfg.d_h)
            ref_o.append(o); ref_l.append(l)
        check("decode_absorb_fp8, pages outside the pool", host(out), np.stack(ref_o), cfg.dtype)
        check("decode_absorb_fp8, pages outside the pool, lse", host(lse), np.stack(ref_l), cfg.dtype)
    finally:
        case.close()


def test_fp8_latent_chain_on_the_gpu():
    """quantise -> decode, both on the GPU, at a few thousand tokens and 256 rows per sequence."""
    cfg = S.CONFIGS["C2"].with_(B=3, L=0, paged=True, seed=995)
    case = Case(cfg, lens=[3000, 257, 1024])
    dec = case.dec
    try:
        c_scale = 0.5
        dec.alloc_latent_fp8()
        dec.quantize_latent(c_scale)
        codes = [F8.quantize_tensor(case.c(b), c_scale) for b in range(cfg.B)]
        _decode_and_check(case, c_scale, codes, "quantise -> decode_absorb_fp8")
    finally:
        case.close()
