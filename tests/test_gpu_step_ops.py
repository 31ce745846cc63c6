"""GPU parity of the steps either side of the decode path -- the rotary embedding of the step's q_R and k_R and the
output projection W^O -- against the CPU oracle, and the whole decode step built from every entry point:
raw step inputs -> rope -> append -> tail expansion -> both decodes -> W^O."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import gqla_oracle as O
from test_gpu_parity import Case, check, host
from test_gpu_step_updates import _prefix_pool

pytestmark = pytest.mark.gpu

ROPE_BASE = 10000.0


@pytest.mark.parametrize("key,lens,s_q,base", [
    ("C3", [300, 2, 64, 129, 70000], 2, 10000.0),     # a position beyond 2^16: the angle needs more than fp32
    ("C1", [65, 64, 1], 1, 500000.0),
    ("C0", [40, 7, 2, 17, 1], 2, 10000.0),            # fp32; the last sequence has L < s_q: its first row has no position
    ("C0", [100000, 65537, 3], 2, 10000.0),           # fp32 at large positions: the fp32 bar needs the angle reduced in double
])
def test_rope_step_matches_the_oracle(key, lens, s_q, base):
    from paper_2605_15250_amd import binding as B
    from paper_2605_15250_amd.harness import to_device, lib_dtype
    cfg = S.CONFIGS[key].with_(B=len(lens), s_q=s_q, L=0, seed=1618)
    lens = np.asarray(lens, np.int32)
    W = cfg.r_kv + cfg.d_r
    r = S.rng(cfg.seed, 7)
    q_raw = S.quantize(r.standard_normal((cfg.B, s_q, cfg.h_q, cfg.d_r), dtype=np.float32), cfg.dtype)
    rows_raw = S.quantize(r.standard_normal((cfg.B, s_q, W), dtype=np.float32), cfg.dtype)
    shape = B.make_shape(cfg.B, cfg.h_q, cfg.g, cfg.d_h, cfg.r_kv, cfg.d_r, s_q, lib_dtype(cfg.dtype))
    d_lens = torch.from_numpy(lens).cuda()
    d_q, d_rows = to_device(q_raw, cfg.dtype), to_device(rows_raw, cfg.dtype)
    B.gqla_rope_step(shape, d_lens, base, d_q, d_rows)
    torch.cuda.synchronize()
    got_q, got_rows = host(d_q), host(d_rows)
    assert np.array_equal(got_rows[..., :cfg.r_kv], rows_raw[..., :cfg.r_kv]), "c_kv must not be touched"
    for b in range(cfg.B):
        for i in range(s_q):
            t = int(lens[b]) - s_q + i
            if t < 0:
                assert np.array_equal(got_q[b, i], q_raw[b, i]) and np.array_equal(got_rows[b, i], rows_raw[b, i])
                continue
            check("rope q_R seq %d tok %d (t=%d)" % (b, i, t), got_q[b, i], O.rope(q_raw[b, i], t, base), cfg.dtype)
            check("rope k_R seq %d tok %d" % (b, i), got_rows[b, i, cfg.r_kv:], O.rope(rows_raw[b, i, cfg.r_kv:], t, base), cfg.dtype)
    # either pointer alone
    d_q2, d_rows2 = to_device(q_raw, cfg.dtype), to_device(rows_raw, cfg.dtype)
    B.gqla_rope_step(shape, d_lens, base, d_q2, None)
    B.gqla_rope_step(shape, d_lens, base, None, d_rows2)
    torch.cuda.synchronize()
    assert torch.equal(d_q2, d_q) and torch.equal(d_rows2, d_rows)


@pytest.mark.parametrize("key,Bsz,s_q,d_model,h_q", [
    ("C1", 5, 2, 256, 32),      # 10 rows: one ragged row tile, 16 k-ranges
    ("C1", 70, 2, 128, 32),     # 140 rows: two row blocks, the second ragged
    ("C3", 3, 1, 384, 128),     # K = 16384
    ("C1", 64, 1, 4096, 32),    # the bench shape of configs[1]
    ("C1", 40, 2, 384, 24),     # K = 3072: 36 workgroups, not a multiple of the eight dies they are dealt over
    ("C1", 150, 2, 256, 32),    # 300 rows: three row blocks, the last ragged
    ("C1", 20, 2, 4096, 40),    # K = 5120: seven k-ranges, the last one shorter
    ("C0", 3, 2, 24, 8),        # fp32 kernel
])
def test_output_projection_matches_the_oracle(key, Bsz, s_q, d_model, h_q):
    from paper_2605_15250_amd import binding as B
    from paper_2605_15250_amd.harness import Decoder, to_device
    cfg = S.CONFIGS[key].with_(B=Bsz, s_q=s_q, L=64, seed=1414, h_q=h_q)
    lens = S.seq_lens(cfg)
    table, npg = S.page_table(cfg, lens)
    dec = Decoder(cfg, lens, table, npg)
    try:
        w_o = S.output_weights(cfg, d_model)
        o = S.quantize(S.rng(cfg.seed, 8).standard_normal((cfg.B, s_q, cfg.h_q, cfg.d_h), dtype=np.float32), cfg.dtype)
        y = torch.full((cfg.B, s_q, d_model), float("nan"), dtype=torch.bfloat16 if cfg.dtype == "bf16" else torch.float32, device="cuda")
        dec.output_projection(to_device(o, cfg.dtype), to_device(w_o, cfg.dtype), y)
        torch.cuda.synchronize()
        ref = np.stack([O.output_projection(o[b], w_o) for b in range(cfg.B)])
        check("output projection", host(y), ref, cfg.dtype)
        if cfg.dtype == "bf16":
            assert B.gqla_output_projection_workspace_bytes(dec.shape, d_model) > 0
            y2 = torch.empty_like(y)
            dec.output_projection(to_device(o, cfg.dtype), to_device(w_o, cfg.dtype), y2)
            torch.cuda.synchronize()
            assert torch.equal(y.view(torch.int16), y2.view(torch.int16)), "the partial sums are added in a fixed order"
    finally:
        dec.close()


@pytest.mark.parametrize("key,lens,page_size,s_q,d_model", [
    ("C3", [300, 2, 64, 129, 1000], 64, 2, 256),
    ("C1", [65, 64, 1, 4000], 64, 1, 384),
    ("C0", [40, 7, 2, 17], 8, 2, 24),
])
def test_whole_decode_step_from_raw_inputs(key, lens, page_size, s_q, d_model):
    """Both path equations of Sec. 3.1 end to end: un-rotated q_R and new rows in, y out.  The cache before the step
    holds the oracle's rotated keys (rounded to the storage type); the step's keys are rotated on the GPU."""
    cfg = S.CONFIGS[key].with_(B=len(lens), s_q=s_q, L=0, paged=True, page_size=page_size, seed=577)
    case = Case(cfg, lens=lens)
    dec = case.dec
    try:
        # raw (un-rotated) k_R of every token are the generator's rows; rotate the whole cache on the host with the oracle
        raw_rows = [r.copy() for r in case.rows]
        for b in range(cfg.B):
            L = int(case.lens[b])
            case.rows[b][:, cfg.r_kv:] = S.quantize(O.rope(raw_rows[b][:, cfg.r_kv:], np.arange(L), ROPE_BASE).astype(np.float32), cfg.dtype)
        w_o = S.output_weights(cfg, d_model)
        d_w_o = case.to_device(w_o, cfg.dtype)
        full_lens = dec.d_lens
        dec.latent_pool, before = _prefix_pool(case, s_q)
        dec.d_lens = torch.from_numpy(before).cuda()
        dec.alloc_expanded()
        dec.expand(case.d_w_uk, case.d_w_uv)
        dec.d_lens = full_lens
        # the step
        new_raw = np.stack([raw_rows[b][int(case.lens[b]) - s_q:] for b in range(cfg.B)])
        d_rows = case.to_device(new_raw, cfg.dtype)
        d_q_r = case.to_device(case.q_r, cfg.dtype)                      # case.q_r serves as the un-rotated q_R
        dec.rope_step(ROPE_BASE, d_q_r, d_rows)
        dec.append_latent(d_rows)
        dec.expand_tail(case.d_w_uk, case.d_w_uv, s_q)
        out_g, _ = dec.decode_gqa(case.d_q_c, d_q_r)
        y_g = dec.output_projection(out_g, d_w_o)
        q_hat = dec.absorb_query(case.d_q_c, case.d_w_uk)
        out_a, _ = dec.decode_absorb(q_hat, d_q_r, case.d_w_uv)
        y_a = dec.output_projection(out_a, d_w_o)
        torch.cuda.synchronize()
        ref = []
        for b in range(cfg.B):
            L = int(case.lens[b])
            qR, _ = O.rope_step(case.q_r[b], raw_rows[b][L - s_q:, cfg.r_kv:], L, ROPE_BASE)
            kR = O.rope(raw_rows[b][:, cfg.r_kv:], np.arange(L), ROPE_BASE)
            KC, V = O.expand_latent(case.c(b), case.w_uk, case.w_uv)
            ref.append(O.output_projection(O.decode_gqa(case.q_c[b], qR, KC, V, kR)[0], w_o))
        ref = np.stack(ref)
        check("step y, GQA path", host(y_g), ref, cfg.dtype)
        check("step y, absorb path", host(y_a), ref, cfg.dtype)
    finally:
        case.close()
