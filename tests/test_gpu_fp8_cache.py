"""GPU parity of the 8-bit expanded cache: the quantising cache switch bit for bit against the oracle's quantiser and
page format, the decode over such a cache against the oracle's GQA-path decode on the dequantised values, and the
whole chain (expand, quantise, decode) on the GPU."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import fp8_cache as F8
from oracle import gqla_oracle as O
from oracle import layout as Lay
from test_gpu_parity import Case, check, host, rel_l2

pytestmark = pytest.mark.gpu


def _bf16_bits(x):
    """16-bit patterns of fp32 values that are representable in bf16."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


@pytest.mark.parametrize("h_q,g,s_q,lens,paged,scales", [
    (128, 8, 2, [300, 2, 129, 65], True, (1.0, 1.0)),      # ragged tails inside 16-token code vectors
    (32, 8, 1, [513, 40], False, (0.37, 2.5)),             # scales that are not powers of two
    (64, 4, 1, [700], True, (0.02, 0.01)),                 # small scales: part of the values saturate at 448
    (128, 4, 2, [300, 65], True, (0.5, 2.0)),              # 64 rows per group: a wave takes both 32-row blocks
    (16, 1, 2, [300, 33, 2], True, (1.0, 0.5)),            # one group, 32 rows: eight waves share a chunk and merge their partials
])
def test_fp8_cache_quantise_and_decode(h_q, g, s_q, lens, paged, scales):
    cfg = S.CONFIGS["C2"].with_(B=len(lens), h_q=h_q, g=g, s_q=s_q, L=0, paged=paged, seed=880 + h_q)
    case = Case(cfg, lens=lens, use_page_table=paged)
    dec = case.dec
    ks, vs = scales
    try:
        # the 16-bit expanded cache both sides start from: the oracle's expansion rounded once to bf16
        KCq, Vq = [], []
        for b in range(cfg.B):
            KC, V = O.expand_latent(case.c(b), case.w_uk, case.w_uv)
            KCq.append(S.quantize(KC, cfg.dtype)); Vq.append(S.quantize(V, cfg.dtype))
        kR = [case.kR(b) for b in range(cfg.B)]
        dec.expanded_pool = case.to_device(Lay.pack_expanded_pool(KCq, Vq, kR, case.table, case.num_pages, cfg.page_size, fill=0.0), cfg.dtype)
        # -- the quantising cache switch, bit for bit (bytes no token owns keep the fill pattern)
        dec.alloc_expanded_fp8(fill=0xAA)
        dec.quantize_expanded(ks, vs)
        torch.cuda.synchronize()
        kc_codes = [F8.quantize_tensor(x, ks) for x in KCq]
        v_codes = [F8.quantize_tensor(x, vs) for x in Vq]
        ref_pool = F8.pack_fp8_pool(kc_codes, v_codes, [_bf16_bits(x) for x in kR], case.table, case.num_pages, cfg.page_size, fill=0xAA)
        got_pool = dec.expanded_fp8_pool.cpu().numpy()
        assert got_pool.shape == ref_pool.shape
        assert np.array_equal(got_pool, ref_pool), "%d of %d bytes differ" % (int((got_pool != ref_pool).sum()), got_pool.size)
        # -- decode over the oracle-packed 8-bit cache against the oracle on the dequantised values
        dec.expanded_fp8_pool = torch.from_numpy(ref_pool).cuda()
        out, lse = dec.decode_gqa_fp8(case.d_q_c, case.d_q_r, ks, vs)
        torch.cuda.synchronize()
        ref_o, ref_l, exact = [], [], []
        for b in range(cfg.B):
            o, l = O.decode_gqa(case.q_c[b], case.q_r[b], F8.dequantize_e4m3(kc_codes[b]) * ks, F8.dequantize_e4m3(v_codes[b]) * vs, kR[b])
            ref_o.append(o); ref_l.append(l)
            exact.append(O.decode_gqa(case.q_c[b], case.q_r[b], KCq[b], Vq[b], kR[b])[0])
        check("decode_gqa_fp8", host(out), np.stack(ref_o), cfg.dtype)
        check("decode_gqa_fp8 lse", host(lse), np.stack(ref_l), cfg.dtype)
        print("8-bit cache vs the 16-bit cache (what the quantisation itself costs): rel_l2 %.3e" % rel_l2(np.stack(ref_o), np.stack(exact)), flush=True)
    finally:
        case.close()


def test_fp8_chain_on_the_gpu():
    """expand -> quantise -> decode, all on the GPU, against the oracle's chain (its expansion rounded to bf16, then
    quantised): the few codes that differ because the GPU's bf16 rounding of an expanded value differs by one unit do
    not show at the output tolerance."""
    cfg = S.CONFIGS["C3"].with_(B=2, L=0, paged=True, seed=881)
    case = Case(cfg, lens=[1000, 257])
    dec = case.dec
    try:
        dec.alloc_expanded(fill=0.0)
        dec.expand(case.d_w_uk, case.d_w_uv)
        dec.alloc_expanded_fp8()
        dec.quantize_expanded(1.0, 1.0)
        out, _ = dec.decode_gqa_fp8(case.d_q_c, case.d_q_r, 1.0, 1.0)
        torch.cuda.synchronize()
        ref = []
        n_codes = n_diff = 0
        pool = dec.expanded_fp8_pool.cpu().numpy()
        for b in range(cfg.B):
            KC, V = O.expand_latent(case.c(b), case.w_uk, case.w_uv)
            kc = F8.quantize_tensor(S.quantize(KC, cfg.dtype), 1.0)
            vv = F8.quantize_tensor(S.quantize(V, cfg.dtype), 1.0)
            ref.append(O.decode_gqa(case.q_c[b], case.q_r[b], F8.dequantize_e4m3(kc), F8.dequantize_e4m3(vv), case.kR(b))[0])
            # how many of the GPU's codes differ from the oracle's (sampled tokens)
            for s in (0, 100, int(case.lens[b]) - 1):
                page, slot = int(case.table[b][s // cfg.page_size]), s % cfg.page_size
                for j in range(cfg.g):
                    for d in range(cfg.d_h):
                        n_codes += 2
                        n_diff += int(pool[F8.k8_offset(page, j, slot, d, cfg.page_size, cfg.g, cfg.d_h, cfg.d_r)] != kc[s, j, d])
                        n_diff += int(pool[F8.v8_offset(page, j, slot, d, cfg.page_size, cfg.g, cfg.d_h, cfg.d_r)] != vv[s, j, d])
        print("codes that differ between the GPU chain and the oracle chain: %d of %d sampled" % (n_diff, n_codes), flush=True)
        assert n_diff <= 0.02 * n_codes
        check("expand -> quantise -> decode_gqa_fp8", host(out), np.stack(ref), cfg.dtype)
    finally:
        case.close()


def test_fp8_tail_expansion_equals_expand_then_quantise():
    """The step's positions expanded straight into the 8-bit cache hold the codes of the two-step route (expand into a
    16-bit cache, convert it), bit for bit, and nothing else is written."""
    cfg = S.CONFIGS["C3"].with_(B=4, L=0, paged=True, seed=882)
    case = Case(cfg, lens=[200, 2, 65, 1000])
    dec = case.dec
    ks, vs = 0.6, 1.7
    try:
        tail = cfg.s_q
        dec.alloc_expanded(fill=0.0)
        dec.expand(case.d_w_uk, case.d_w_uv)
        dec.alloc_expanded_fp8(fill=0xAA)
        dec.quantize_expanded(ks, vs)
        torch.cuda.synchronize()
        two_step = dec.expanded_fp8_pool.clone()
        dec.alloc_expanded_fp8(fill=0xAA)
        dec.expand_tail_fp8(case.d_w_uk, case.d_w_uv, tail, ks, vs)
        torch.cuda.synchronize()
        got = dec.expanded_fp8_pool.cpu().numpy()
        ref = two_step.cpu().numpy()
        per_tok = 2 * cfg.g * cfg.d_h + 2 * cfg.d_r
        written = got != 0xAA
        # codes equal to the fill pattern exist, so count with a margin: at most the tail's bytes were touched, most of them differ from the fill
        assert int(written.sum()) <= cfg.B * tail * per_tok and int(written.sum()) >= 0.9 * cfg.B * tail * per_tok
        assert np.array_equal(got[written], ref[written])
        # every byte of every tail token (also those that happen to equal the fill) against the two-step route
        for b in range(cfg.B):
            for s in range(int(case.lens[b]) - tail, int(case.lens[b])):
                page, slot = int(case.table[b][s // cfg.page_size]), s % cfg.page_size
                for j in (0, cfg.g - 1):
                    for d in range(cfg.d_h):
                        ko = F8.k8_offset(page, j, slot, d, cfg.page_size, cfg.g, cfg.d_h, cfg.d_r)
                        vo = F8.v8_offset(page, j, slot, d, cfg.page_size, cfg.g, cfg.d_h, cfg.d_r)
                        assert got[ko] == ref[ko] and got[vo] == ref[vo]
                for d in range(cfg.d_r):
                    o = F8.kr16_offset(page, slot, d, cfg.page_size, cfg.g, cfg.d_h, cfg.d_r)
                    assert got[o] == ref[o] and got[o + 1] == ref[o + 1]
    finally:
        case.close()


@pytest.mark.parametrize("lens,page_size,groups,group_begin", [
    ([200, 2, 65, 1000, 256, 31], 64, None, 0),     # ragged tails inside a 32-token tile, a full page, a tiny sequence
    ([300, 129], 128, None, 0),                     # 128-token pages
    ([257, 64], 64, 2, 5),                          # a two-group slice
])
def test_fp8_one_shot_expansion_equals_expand_then_quantise(lens, page_size, groups, group_begin):
    """The whole cache switch latent -> 8-bit expanded in one pass holds the bytes of the two-step route (expand into a
    16-bit cache, convert it) -- the two-step route itself is checked against the oracle above -- and leaves every byte
    no token owns as it was."""
    cfg = S.CONFIGS["C3"].with_(B=len(lens), L=0, paged=True, page_size=page_size, seed=883)
    case = Case(cfg, lens=lens, groups=groups, group_begin=group_begin)
    dec = case.dec
    ks, vs = 0.6, 1.7
    try:
        dec.alloc_expanded(fill=0.0)
        dec.expand(case.d_w_uk, case.d_w_uv)
        dec.alloc_expanded_fp8(fill=0xAA)
        dec.quantize_expanded(ks, vs)
        torch.cuda.synchronize()
        ref = dec.expanded_fp8_pool.clone()
        dec.alloc_expanded_fp8(fill=0xAA)
        dec.expand_fp8(case.d_w_uk, case.d_w_uv, ks, vs)
        torch.cuda.synchronize()
        assert torch.equal(dec.expanded_fp8_pool, ref), "one-shot 8-bit expansion differs from expand + quantise in %d bytes" % int(
            (dec.expanded_fp8_pool != ref).sum().item())
    finally:
        case.close()
