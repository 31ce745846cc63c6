"""The decode step (rotary step, cache updates, both decode paths, output projection) recorded into a HIP graph and
replayed: the library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset nodes),
so a captured step must reproduce the eager step bit for bit on every replay, also after the inputs have been rewritten
in place."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from test_gpu_parity import Case

pytestmark = pytest.mark.gpu


def test_captured_step_replays_bit_identically():
    cfg = S.CONFIGS["C3"].with_(B=3, L=0, paged=True, seed=4711)
    case = Case(cfg, lens=[700, 130, 65])
    dec = case.dec
    try:
        dt = torch.bfloat16
        W = cfg.r_kv + cfg.d_r
        q_c, q_r = case.d_q_c.clone(), case.d_q_r.clone()
        rows = torch.stack([torch.from_numpy(case.rows[b][int(case.lens[b]) - cfg.s_q:]) for b in range(cfg.B)]).to(dt).cuda().contiguous()
        q_hat = torch.empty((cfg.B, cfg.s_q, cfg.h_q, cfg.r_kv), dtype=dt, device="cuda")
        out_a = torch.empty((cfg.B, cfg.s_q, cfg.h_q, cfg.d_h), dtype=dt, device="cuda")
        out_g = torch.empty_like(out_a)
        lse_a = torch.empty((cfg.B, cfg.s_q, cfg.h_q), dtype=torch.float32, device="cuda")
        lse_g = torch.empty_like(lse_a)
        dec.alloc_expanded(fill=0.0)
        dec.expand(case.d_w_uk, case.d_w_uv)          # the context, expanded once, outside the step
        d_model = 256
        w_o = case.to_device(S.output_weights(cfg, d_model), cfg.dtype)
        y_a = torch.empty((cfg.B, cfg.s_q, d_model), dtype=dt, device="cuda")
        y_g = torch.empty_like(y_a)
        q_r_src, rows_src = q_r.clone(), rows.clone()  # un-rotated inputs: the step rotates q_r and rows in place

        def reset_inputs():
            q_r.copy_(q_r_src)
            rows.copy_(rows_src)

        def step():
            dec.rope_step(10000.0, q_r, rows)
            dec.append_latent(rows)
            dec.expand_tail(case.d_w_uk, case.d_w_uv, cfg.s_q)
            dec.absorb_query(q_c, case.d_w_uk, q_hat)
            dec.decode_absorb(q_hat, q_r, case.d_w_uv, out_a, lse_a)
            dec.decode_gqa(q_c, q_r, out_g, lse_g)
            dec.output_projection(out_a, w_o, y_a)
            dec.output_projection(out_g, w_o, y_g)

        def snapshot():
            torch.cuda.synchronize()
            return [t.clone() for t in (out_a, lse_a, out_g, lse_g, dec.latent_pool, dec.expanded_pool, y_a, y_g, q_r, rows)]

        step()                                          # eager: also does every first-call set-up of the library
        ref0 = snapshot()
        reset_inputs()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        gen = torch.Generator(device="cuda").manual_seed(99)
        for replay in range(4):
            if replay:                                  # new queries and new step rows, written in place by eager work
                q_c.copy_(torch.randn(q_c.shape, generator=gen, device="cuda").to(dt))
                q_r_src.copy_(torch.randn(q_r.shape, generator=gen, device="cuda").to(dt))
                rows_src.copy_(torch.randn(rows.shape, generator=gen, device="cuda").to(dt))
            reset_inputs()
            for t in (out_a, lse_a, out_g, lse_g, y_a, y_g):
                t.zero_()
            torch.cuda.synchronize()
            graph.replay()
            got = snapshot()
            reset_inputs()
            for t in (out_a, lse_a, out_g, lse_g, y_a, y_g):
                t.zero_()
            step()                                      # the same inputs, eagerly
            ref = snapshot() if replay else ref0
            if not replay:
                torch.cuda.synchronize()
            for name, a, b in zip(("out absorb", "lse absorb", "out gqa", "lse gqa", "latent pool", "expanded pool", "y absorb", "y gqa",
                                   "rotated q_R", "rotated rows"), got, ref):
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), "replay %d: %s differs from the eager step" % (replay, name)
            assert torch.isfinite(got[0].float()).all() and torch.isfinite(got[2].float()).all()
    finally:
        case.close()
