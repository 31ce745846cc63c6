"""Pins for the CPU oracle: each test checks it against something other than itself
(brute force, closed forms, library attention, invariants, the paper's printed numbers)."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import gqla_oracle as O
from oracle import roofline as R
import synth_inputs as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_problem(seed, h_q=8, g=2, d_h=16, r_kv=32, d_r=8, L=64, s_q=1):
    r = np.random.default_rng(seed)
    c = r.standard_normal((L, r_kv))
    kR = r.standard_normal((L, d_r))
    qC = r.standard_normal((s_q, h_q, d_h))
    qR = r.standard_normal((s_q, h_q, d_r))
    W_UK = r.standard_normal((g, r_kv, d_h)) / math.sqrt(r_kv)
    W_UV = r.standard_normal((g, r_kv, d_h)) / math.sqrt(r_kv)
    return c, kR, qC, qR, W_UK, W_UV


def both_paths(c, kR, qC, qR, W_UK, W_UV):
    KC, V = O.expand_latent(c, W_UK, W_UV)
    o_g, lse_g = O.decode_gqa(qC, qR, KC, V, kR)
    o_a, lse_a = O.decode_absorb(O.absorb_query(qC, W_UK), qR, c, kR, W_UV)
    return o_g, lse_g, o_a, lse_a


# ---- P1: the two paths and the fully materialised per-head attention agree (Sec. 3.1) ----------
def test_c0_two_paths_and_bruteforce_agree():
    cfg = S.CONFIGS["C0"]
    w_uk, w_uv = S.weights(cfg)
    q_c, q_r = S.queries(cfg)
    rows = S.sequence_rows(cfg, 0, cfg.L)
    c, kR = rows[:, :cfg.r_kv], rows[:, cfg.r_kv:]
    o_g, lse_g, o_a, lse_a = both_paths(c, kR, q_c[0], q_r[0], w_uk, w_uv)
    o_m = O.decode_mha_bruteforce(q_c[0], q_r[0], c, kR, w_uk, w_uv)
    assert np.max(np.abs(o_g - o_a)) <= 1e-10
    assert np.max(np.abs(o_g - o_m)) <= 1e-10
    assert np.max(np.abs(lse_g - lse_a)) <= 1e-10


@pytest.mark.parametrize("h_q,g,d_h,r_kv,d_r,L,s_q", [
    (4, 4, 8, 8, 8, 5, 1),      # G = 1
    (6, 1, 8, 16, 8, 9, 2),     # one group (MQA), MTP
    (6, 3, 16, 8, 16, 7, 2),    # g*d_h > r_kv
    (12, 4, 8, 24, 8, 3, 2),    # L barely above s_q
    (2, 2, 8, 8, 8, 2, 2),      # L == s_q: first row sees one token
])
def test_random_tiny_shapes_agree(h_q, g, d_h, r_kv, d_r, L, s_q):
    p = tiny_problem(100 + h_q + L, h_q, g, d_h, r_kv, d_r, L, s_q)
    c, kR, qC, qR, W_UK, W_UV = p
    o_g, lse_g, o_a, lse_a = both_paths(*p)
    o_m = O.decode_mha_bruteforce(qC, qR, c, kR, W_UK, W_UV)
    assert np.max(np.abs(o_g - o_a)) <= 1e-10
    assert np.max(np.abs(o_g - o_m)) <= 1e-10
    assert np.max(np.abs(lse_g - lse_a)) <= 1e-10


# ---- P2: L = 1 -> softmax is 1 -> o_i = W_UV[j(i)]^T c_0, written with explicit indices ----------
def test_single_token_is_pure_value_projection():
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(7, h_q=6, g=3, d_h=8, r_kv=16, d_r=8, L=1)
    o_g, _, o_a, _ = both_paths(c, kR, qC, qR, W_UK, W_UV)
    for i in range(6):
        j = i // 2
        want = np.array([sum(W_UV[j, r, d] * c[0, r] for r in range(16)) for d in range(8)])
        assert np.max(np.abs(o_g[0, i] - want)) <= 1e-12
        assert np.max(np.abs(o_a[0, i] - want)) <= 1e-12


def test_group_routing_is_blockwise_not_strided():
    # heads 0,1 -> group 0; heads 2,3 -> group 1 (group-wise replication).
    assert [O.head_group(i, 4, 2) for i in range(4)] == [0, 0, 1, 1]
    assert [O.head_group(i, 128, 8) for i in (0, 15, 16, 127)] == [0, 0, 1, 7]
    with pytest.raises(ValueError):
        O.head_group(0, 10, 4)


# ---- P3: zero queries -> uniform softmax -> mean of V over the visible rows; lse = log |Vis| -------
@pytest.mark.parametrize("s_q", [1, 2])
def test_zero_query_gives_mean_value(s_q):
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(11, L=13, s_q=s_q)
    qC[:] = 0
    qR[:] = 0
    o_g, lse_g, o_a, lse_a = both_paths(c, kR, qC, qR, W_UK, W_UV)
    KC, V = O.expand_latent(c, W_UK, W_UV)
    for t in range(s_q):
        nv = 13 - s_q + t + 1
        for i in range(8):
            want = V[:nv, i // 4, :].mean(axis=0)
            assert np.max(np.abs(o_g[t, i] - want)) <= 1e-12
            assert np.max(np.abs(o_a[t, i] - want)) <= 1e-12
            assert abs(lse_g[t, i] - math.log(nv)) <= 1e-12
            assert abs(lse_a[t, i] - math.log(nv)) <= 1e-12


# ---- P4: selector weights (the "sparse identity" initialisation of Sec. 3.2.1) -> vanilla GQA -----
def test_selector_weights_reduce_to_plain_gqa():
    g, d_h, d_r, L, h_q = 3, 8, 8, 10, 6
    r_kv = g * d_h
    r = np.random.default_rng(5)
    c = r.standard_normal((L, r_kv))
    kR = r.standard_normal((L, d_r))
    qC = r.standard_normal((1, h_q, d_h))
    qR = r.standard_normal((1, h_q, d_r))
    W_UK = np.zeros((g, r_kv, d_h))
    W_UV = np.zeros((g, r_kv, d_h))
    for j in range(g):
        for d in range(d_h):
            W_UK[j, j * d_h + d, d] = 1.0        # K of group j = block j of the latent
            W_UV[j, (g - 1 - j) * d_h + d, d] = 1.0  # V of group j = block g-1-j
    KC, V = O.expand_latent(c, W_UK, W_UV)
    for j in range(g):
        assert np.array_equal(KC[:, j, :], c[:, j * d_h:(j + 1) * d_h])
        assert np.array_equal(V[:, j, :], c[:, (g - 1 - j) * d_h:(g - j) * d_h])
    o_g, _, o_a, _ = both_paths(c, kR, qC, qR, W_UK, W_UV)
    # plain GQA written directly on the latent blocks
    for i in range(h_q):
        j = i // 2
        Kb = np.concatenate([c[:, j * d_h:(j + 1) * d_h], kR], axis=1)
        z = Kb @ np.concatenate([qC[0, i], qR[0, i]]) / math.sqrt(d_h + d_r)
        p = np.exp(z - z.max())
        p /= p.sum()
        want = p @ c[:, (g - 1 - j) * d_h:(g - j) * d_h]
        assert np.max(np.abs(o_g[0, i] - want)) <= 1e-12
        assert np.max(np.abs(o_a[0, i] - want)) <= 1e-12


# ---- P5: library attention as a second opinion (g = h_q is MHA, g = 1 is MQA) ---------------------
@pytest.mark.parametrize("g", [6, 1, 3])
def test_against_torch_sdpa(g):
    h_q, d_h, d_r, r_kv, L = 6, 8, 8, 16, 33
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(23 + g, h_q, g, d_h, r_kv, d_r, L, 1)
    KC, V = O.expand_latent(c, W_UK, W_UV)
    o_g, _ = O.decode_gqa(qC, qR, KC, V, kR)
    G = h_q // g
    q = torch.from_numpy(np.concatenate([qC, qR], axis=2)).permute(1, 0, 2)[None]          # [1,h,1,D]
    K = np.concatenate([np.repeat(KC, G, axis=1), np.repeat(kR[:, None, :], h_q, axis=1)], axis=2)
    k = torch.from_numpy(K).permute(1, 0, 2)[None]                                          # [1,h,L,D]
    v = torch.from_numpy(np.repeat(V, G, axis=1)).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v)[0, :, 0, :].numpy()    # scale 1/sqrt(D)
    assert np.max(np.abs(o_g[0] - want)) <= 1e-12


def test_mtp_mask_against_torch_causal():
    # s_q = 2 with L == s_q is exactly a causal 2x2 problem.
    h_q, g, d_h, d_r, r_kv = 4, 2, 8, 8, 8
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(31, h_q, g, d_h, r_kv, d_r, 2, 2)
    KC, V = O.expand_latent(c, W_UK, W_UV)
    o_g, _ = O.decode_gqa(qC, qR, KC, V, kR)
    q = torch.from_numpy(np.concatenate([qC, qR], axis=2)).permute(1, 0, 2)[None]
    K = np.concatenate([np.repeat(KC, 2, axis=1), np.repeat(kR[:, None, :], h_q, axis=1)], axis=2)
    k = torch.from_numpy(K).permute(1, 0, 2)[None]
    v = torch.from_numpy(np.repeat(V, 2, axis=1)).permute(1, 0, 2)[None]
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.max(np.abs(o_g - want)) <= 1e-12


# ---- P6: adding a constant to every logit of a row leaves o unchanged and shifts lse ---------------
def test_logit_shift_invariance():
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(41, L=20)
    kR[:, 0] = 1.0
    o0, lse0, oa0, lsea0 = both_paths(c, kR, qC, qR, W_UK, W_UV)
    qR2 = qR.copy()
    qR2[:, :, 0] += 700.0                    # would overflow exp() without max subtraction
    o1, lse1, oa1, lsea1 = both_paths(c, kR, qC, qR2, W_UK, W_UV)
    shift = 700.0 / math.sqrt(16 + 8)
    assert np.max(np.abs(o0 - o1)) <= 1e-10
    assert np.max(np.abs(oa0 - oa1)) <= 1e-10
    assert np.max(np.abs(lse1 - lse0 - shift)) <= 1e-9
    assert np.max(np.abs(lsea1 - lsea0 - shift)) <= 1e-9


# ---- P7: MTP rows are plain decodes at lengths L-1 and L ---------------------------------------
def test_mtp_rows_equal_plain_decodes():
    L = 17
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(51, L=L, s_q=2)
    o2, lse2, oa2, lsea2 = both_paths(c, kR, qC, qR, W_UK, W_UV)
    o_last, lse_last, oa_last, _ = both_paths(c, kR, qC[1:2], qR[1:2], W_UK, W_UV)
    o_first, lse_first, oa_first, _ = both_paths(c[:L - 1], kR[:L - 1], qC[0:1], qR[0:1], W_UK, W_UV)
    assert np.max(np.abs(o2[1] - o_last[0])) <= 1e-12
    assert np.max(np.abs(o2[0] - o_first[0])) <= 1e-12
    assert np.max(np.abs(oa2[1] - oa_last[0])) <= 1e-12
    assert np.max(np.abs(oa2[0] - oa_first[0])) <= 1e-12
    assert np.max(np.abs(lse2[1] - lse_last[0])) <= 1e-12
    assert np.max(np.abs(lse2[0] - lse_first[0])) <= 1e-12
    # the last token must matter for row 1 and not for row 0
    c2 = c.copy()
    c2[L - 1] += 1.0
    o3, _, _, _ = both_paths(c2, kR, qC, qR, W_UK, W_UV)
    assert np.max(np.abs(o3[0] - o2[0])) == 0.0
    assert np.max(np.abs(o3[1] - o2[1])) > 1e-3


# ---- P8: split invariance of the log-sum-exp combine -------------------------------------------
@pytest.mark.parametrize("bounds", [
    [(0, 29)],
    [(0, 1), (1, 29)],
    [(0, 16), (16, 28), (28, 29)],            # last chunk holds only the token invisible to row 0
    [(k, k + 1) for k in range(29)],
])
def test_split_invariance(bounds):
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(61, L=29, s_q=2)
    KC, V = O.expand_latent(c, W_UK, W_UV)
    o, lse = O.decode_gqa(qC, qR, KC, V, kR)
    o_s, lse_s = O.decode_gqa_split(qC, qR, KC, V, kR, bounds)
    assert np.max(np.abs(o - o_s)) <= 1e-12
    assert np.max(np.abs(lse - lse_s)) <= 1e-12


def test_combine_matches_direct_formula_on_two_chunks():
    # two chunks with known local softmaxes: o = (e^{l1} o1 + e^{l2} o2) / (e^{l1} + e^{l2})
    o1, o2 = np.array([1.0, 2.0]), np.array([3.0, -1.0])
    l1, l2 = 0.3, -1.2
    o, lse = O.combine_partials([o1, o2], [l1, l2])
    w1, w2 = math.exp(l1), math.exp(l2)
    assert np.allclose(o, (w1 * o1 + w2 * o2) / (w1 + w2), atol=1e-15)
    assert abs(lse - math.log(w1 + w2)) <= 1e-15
    o, lse = O.combine_partials([o1, np.zeros(2)], [l1, -math.inf])   # an empty chunk has weight 0
    assert np.array_equal(o, o1) and lse == l1


# ---- P9 / P10: page permutation and token permutation invariance -----------------------------------
def test_page_permutation_invariance_exact():
    cfg = S.CONFIGS["C0"].with_(B=3, L=0, L_min=5, L_max=40, page_size=8, paged=True, seed=99)
    lens = S.seq_lens(cfg)
    table, num_pages = S.page_table(cfg, lens)
    ident, num_ident = S.page_table(cfg.with_(paged=False), lens)
    assert sorted(table[table >= 0].tolist()) == list(range(num_pages))
    from oracle import layout as Lay
    seqs = [S.sequence_rows(cfg, b, lens[b]) for b in range(cfg.B)]
    W = cfg.r_kv + cfg.d_r
    pool_p = Lay.pack_latent_pool(seqs, table, num_pages, cfg.page_size, W)
    pool_i = Lay.pack_latent_pool(seqs, ident, num_ident, cfg.page_size, W)
    for b in range(cfg.B):
        a = O.gather_rows(pool_p, table[b], lens[b], cfg.page_size)
        i = O.gather_rows(pool_i, ident[b], lens[b], cfg.page_size)
        assert np.array_equal(a, seqs[b]) and np.array_equal(i, seqs[b])
        assert not np.isnan(a).any()           # the NaN-filled tail slots are never gathered


def test_token_permutation_invariance():
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(71, L=21)
    o0, lse0, oa0, _ = both_paths(c, kR, qC, qR, W_UK, W_UV)
    perm = np.random.default_rng(1).permutation(21)
    o1, lse1, oa1, _ = both_paths(c[perm], kR[perm], qC, qR, W_UK, W_UV)
    assert np.max(np.abs(o0 - o1)) <= 1e-12
    assert np.max(np.abs(oa0 - oa1)) <= 1e-12
    assert np.max(np.abs(lse0 - lse1)) <= 1e-12


# ---- orientation pins: a transposed or swapped weight would fail these ------------------------------
def test_expand_orientation_explicit():
    r = np.random.default_rng(3)
    c = r.standard_normal((2, 5))
    W_UK = r.standard_normal((2, 5, 3))
    W_UV = r.standard_normal((2, 5, 3))
    KC, V = O.expand_latent(c, W_UK, W_UV)
    for s in range(2):
        for j in range(2):
            for d in range(3):
                assert abs(KC[s, j, d] - sum(W_UK[j, rr, d] * c[s, rr] for rr in range(5))) <= 1e-14
                assert abs(V[s, j, d] - sum(W_UV[j, rr, d] * c[s, rr] for rr in range(5))) <= 1e-14


def test_absorb_query_orientation_explicit():
    r = np.random.default_rng(4)
    qC = r.standard_normal((2, 4, 3))
    W_UK = r.standard_normal((2, 5, 3))
    qh = O.absorb_query(qC, W_UK)
    for t in range(2):
        for i in range(4):
            for rr in range(5):
                assert abs(qh[t, i, rr] - sum(W_UK[i // 2, rr, d] * qC[t, i, d] for d in range(3))) <= 1e-14


def test_scale_is_sqrt_of_total_key_dim():
    assert O.softmax_scale(128, 64) == 1.0 / math.sqrt(192)
    # doubling the scale must change the output (the scale is not silently dropped)
    c, kR, qC, qR, W_UK, W_UV = tiny_problem(81, L=9)
    KC, V = O.expand_latent(c, W_UK, W_UV)
    a, _ = O.decode_gqa(qC, qR, KC, V, kR)
    b, _ = O.decode_gqa(qC, qR, KC, V, kR, scale=2.0 / math.sqrt(24))
    assert np.max(np.abs(a - b)) > 1e-3


# ---- P11 / P12: the paper's printed numbers ---------------------------------------------------------
def _constants():
    out = {}
    for line in open(os.path.join(GOLDEN, "paper_constants.txt")):
        if line.strip() and not line.startswith("#"):
            name, value = line.split()[:2]
            out[name] = float(value)
    return out


def test_paper_size_and_intensity_constants():
    k = _constants()
    assert R.absorb_bytes_per_token(512, 64) == k["absorb_bytes_per_token"]
    assert R.gqa_bytes_per_token(8, 128, 64) == k["gqa_bytes_per_token_g8"]
    assert R.gqa_bytes_per_token(4, 128, 64) == k["gqa_bytes_per_token_g4"]
    assert round(R.absorb_intensity(128, 1, 512, 64)) == k["absorb_intensity_sq1"]
    assert round(R.absorb_intensity(128, 2, 512, 64)) == k["absorb_intensity_sq2"]
    assert round(R.gqa_intensity(128, 8, 2, 128, 64), 1) == k["gqa_intensity_g8_sq2"]
    assert round(R.gqa_intensity(128, 4, 1, 128, 64), 1) == k["gqa_intensity_g4_sq1"]
    assert round(R.ridge(989e12, 3.35e12)) == k["ridge_h100"]
    assert round(R.ridge(148e12, 4.0e12)) == k["ridge_h20"]
    from oracle import layout as Lay
    lat = Lay.latent_elems_per_token(512, 64)
    assert lat == 576
    assert 100.0 * lat / (2 * 8 * 128) == k["latent_vs_llama3_gqa_pct"]
    assert 100.0 * lat / (2 * 4 * 128) == k["latent_vs_qwen25_gqa_pct"]
    assert Lay.expanded_elems_per_token(8, 128, 64) == 2112


def test_paper_operating_point_table():
    hw = {"H100": (989e12, 3.35e12), "H20": (148e12, 4.0e12)}
    n = 0
    for line in open(os.path.join(GOLDEN, "roofline_table.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        gpu, path, g, s_q, bpt, inten, mem, cmp_, step, ktok = line.split()
        g, s_q = int(g), int(s_q)
        peak, bw = hw[gpu]
        if path == "absorb":
            nbytes = R.absorb_bytes(8192, 512, 64)
            flops = R.absorb_flops(8192, 128, s_q, 512, 64)
            inten_calc = R.absorb_intensity(128, s_q, 512, 64)
            assert R.absorb_bytes_per_token(512, 64) == int(bpt)
        else:
            nbytes = R.gqa_bytes(8192, g, 128, 64)
            flops = R.gqa_flops(8192, 128, s_q, 128, 64)
            inten_calc = R.gqa_intensity(128, g, s_q, 128, 64)
            assert R.gqa_bytes_per_token(g, 128, 64) == int(bpt)
        op = R.operating_point(nbytes, flops, s_q, peak, bw)
        assert abs(inten_calc - float(inten)) <= 0.5
        assert abs(inten_calc - flops / nbytes) <= 1e-9
        # two printed decimals; the s_q = 2 rows print twice the rounded s_q = 1 figure
        # (30.84 = 2 x 15.42 where the formula gives 30.834), hence one unit of the last digit.
        assert abs(op["mem_s"] * 1e6 - float(mem)) <= 0.01
        assert abs(op["cmp_s"] * 1e6 - float(cmp_)) <= 0.01
        assert abs(op["step_s"] * 1e6 - float(step)) <= 0.01
        # printed in thousands; the first row prints 354 where its own formula gives 354.98
        # (1 / 2.82 us = 354.6), so the pin allows one unit in the last printed digit.
        assert abs(op["tok_per_s"] / 1e3 - float(ktok)) <= 1.0
        n += 1
    assert n == 8


# ---- input generator sanity ---------------------------------------------------------------------
def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(4096).astype(np.float32) * 3
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]        # exact ties -> even
    bits = S.round_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    assert np.array_equal(S.bf16_bits_to_f32(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_generators_are_reproducible_and_per_sequence():
    cfg = S.CONFIGS["C4"].with_(B=4)
    lens = S.seq_lens(cfg)
    assert lens.min() >= 1024 and lens.max() <= 32768
    a = S.sequence_rows(cfg, 2, 100)
    b = S.sequence_rows(cfg, 2, 100)
    assert np.array_equal(a, b) and a.shape == (100, 576)
    w1, _ = S.weights(cfg)
    assert abs(float(w1.std()) - 512 ** -0.5) < 2e-3


def test_compress_is_the_inverse_of_expand_and_the_least_squares_solution():
    """Sec. 3.1 (the cache is converted once, in either direction): compressing an exact expansion returns the latent (g d_h >= r_kv),
    and on perturbed keys the result is numpy's least-squares solution of A c = k^C, token by token."""
    rng = np.random.default_rng(5)
    g, r_kv, d_h, L = 3, 10, 4, 7                     # g d_h = 12 >= r_kv = 10
    W_UK = rng.normal(size=(g, r_kv, d_h))
    W_UV = rng.normal(size=(g, r_kv, d_h))
    c = rng.normal(size=(L, r_kv))
    KC, _ = O.expand_latent(c, W_UK, W_UV)
    assert np.max(np.abs(O.compress_expanded(KC, W_UK) - c)) < 1e-10
    Linv = O.left_inverse_uk(W_UK)
    A = np.concatenate([W_UK[j].T for j in range(g)], axis=0)
    assert np.max(np.abs(Linv @ A - np.eye(r_kv))) < 1e-10           # a left inverse
    assert np.max(np.abs(Linv - np.linalg.pinv(A))) < 1e-9            # the Moore-Penrose one
    noisy = KC + 0.1 * rng.normal(size=KC.shape)
    want = np.stack([np.linalg.lstsq(A, noisy[s].reshape(-1), rcond=None)[0] for s in range(L)])
    assert np.max(np.abs(O.compress_expanded(noisy, W_UK) - want)) < 1e-9
    # column order: group-major, dim-minor -- compressing keys that live in one group only uses that group's block
    only1 = np.zeros_like(KC)
    only1[:, 1, :] = KC[:, 1, :]
    assert np.max(np.abs(O.compress_expanded(only1, W_UK) - KC[:, 1, :] @ Linv[:, d_h:2 * d_h].T)) < 1e-12


def test_rope_closed_forms_and_relative_position_property():
    """Sec. 3.1 ("Architecture"): rope_t.  Pins: identity at t = 0; a unit vector in pair 0 turns by exactly t
    radians, counter-clockwise; pair p turns base^(-2p/d) times as fast; the complex-number form of the same
    rotation; norm preservation; and what the method relies on: <rope_t q, rope_s k> depends on t - s only."""
    rng = np.random.default_rng(5)
    x = rng.normal(size=(3, 8))
    assert np.array_equal(O.rope(x, 0), x)
    # d = 2: the plane rotation by t radians, whatever the base
    for base in (10000.0, 7.0):
        got = O.rope(np.array([1.0, 0.0]), 1, base)
        assert np.allclose(got, [np.cos(1.0), np.sin(1.0)], atol=1e-15)
        got = O.rope(np.array([0.0, 1.0]), 2, base)
        assert np.allclose(got, [-np.sin(2.0), np.cos(2.0)], atol=1e-15)
    # d = 4, base 10000: pair 1 has frequency 10000^(-2/4) = 0.01, and it is the pair of elements 2 and 3
    got = O.rope(np.array([0.0, 0.0, 1.0, 0.0]), 50, 10000.0)
    assert np.allclose(got, [0.0, 0.0, np.cos(0.5), np.sin(0.5)], atol=1e-15)
    got = O.rope(np.array([1.0, 0.0, 0.0, 0.0]), 50, 10000.0)
    assert np.allclose(got, [np.cos(50.0), np.sin(50.0), 0.0, 0.0], atol=1e-13)
    # complex form: (x[2p] + i x[2p+1]) * exp(i t theta_p)
    d, t, base = 8, 37, 10000.0
    z = (x[:, 0::2] + 1j * x[:, 1::2]) * np.exp(1j * t * base ** (-np.arange(d // 2) * 2.0 / d))
    got = O.rope(x, t, base)
    assert np.allclose(got[:, 0::2], z.real, atol=1e-13) and np.allclose(got[:, 1::2], z.imag, atol=1e-13)
    # per-row positions broadcast
    pos = np.array([3, 11, 29])
    got = O.rope(x, pos)
    for r in range(3):
        assert np.allclose(got[r], O.rope(x[r], int(pos[r])), atol=1e-15)
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1), atol=1e-13)
    # relative positions
    q, k = rng.normal(size=64), rng.normal(size=64)
    for t, s in ((100, 90), (5000, 4990), (17, 7)):
        assert abs(O.rope(q, t) @ O.rope(k, s) - O.rope(q, t - s) @ k) < 1e-10
    assert abs(O.rope(q, 100) @ O.rope(k, 90) - O.rope(q, 100) @ O.rope(k, 91)) > 1e-3      # and on nothing less


def test_rope_step_positions_follow_the_in_step_mask():
    """Step token t sits at position L - s_q + t, the position n_visible uses; decoding with rotated inputs is
    invariant under shifting every position by the same amount (the logits see position differences only)."""
    rng = np.random.default_rng(6)
    s_q, h_q, g, d_h, d_r, r_kv, L = 2, 4, 2, 8, 4, 16, 9
    qR_raw, kR_raw_all = rng.normal(size=(s_q, h_q, d_r)), rng.normal(size=(L, d_r))
    qR, kR_new = O.rope_step(qR_raw, kR_raw_all[L - s_q:], L)
    assert np.allclose(qR[0], O.rope(qR_raw[0], L - 2)) and np.allclose(qR[1], O.rope(qR_raw[1], L - 1))
    assert np.allclose(kR_new[0], O.rope(kR_raw_all[L - 2], L - 2)) and np.allclose(kR_new[1], O.rope(kR_raw_all[L - 1], L - 1))
    qC = rng.normal(size=(s_q, h_q, d_h))
    c = rng.normal(size=(L, r_kv))
    W_UK, W_UV = rng.normal(size=(g, r_kv, d_h)), rng.normal(size=(g, r_kv, d_h))
    KC, V = O.expand_latent(c, W_UK, W_UV)
    outs = []
    for shift in (0, 1000):
        kR = O.rope(kR_raw_all, np.arange(L) + shift)
        qRs = O.rope(qR_raw, (L - s_q + np.arange(s_q) + shift)[:, None])
        outs.append(O.decode_gqa(qC, qRs, KC, V, kR)[0])
    assert np.max(np.abs(outs[0] - outs[1])) < 1e-10
    # the cache of shift 0 is what rope_step produces token by token
    kR0 = O.rope(kR_raw_all, np.arange(L))
    assert np.allclose(kR0[L - s_q:], kR_new, atol=1e-15)


def test_output_projection_is_the_sum_of_per_head_blocks():
    """Last line of both path equations: y = W^O [o_1; ...; o_hq] = sum_i W^O[:, i d_h:(i+1) d_h] o_i; the identity
    returns the concatenation; and the whole layer agrees between the two paths."""
    rng = np.random.default_rng(7)
    s_q, h_q, g, d_h, d_r, r_kv, L, D = 2, 4, 2, 8, 4, 16, 11, 12
    o = rng.normal(size=(s_q, h_q, d_h))
    W_O = rng.normal(size=(D, h_q * d_h))
    want = np.zeros((s_q, D))
    for t in range(s_q):
        for i in range(h_q):
            want[t] += W_O[:, i * d_h:(i + 1) * d_h] @ o[t, i]
    assert np.max(np.abs(O.output_projection(o, W_O) - want)) < 1e-12
    assert np.array_equal(O.output_projection(o, np.eye(h_q * d_h)), o.reshape(s_q, -1))
    qC, qR = rng.normal(size=(s_q, h_q, d_h)), rng.normal(size=(s_q, h_q, d_r))
    c, kR = rng.normal(size=(L, r_kv)), rng.normal(size=(L, d_r))
    W_UK, W_UV = rng.normal(size=(g, r_kv, d_h)), rng.normal(size=(g, r_kv, d_h))
    KC, V = O.expand_latent(c, W_UK, W_UV)
    y_g = O.output_projection(O.decode_gqa(qC, qR, KC, V, kR)[0], W_O)
    y_a = O.output_projection(O.decode_absorb(O.absorb_query(qC, W_UK), qR, c, kR, W_UV)[0], W_O)
    assert np.max(np.abs(y_g - y_a)) < 1e-10


def test_value_dim_may_differ_from_the_key_dim():
    """Sec. 3.2.2 (MLA checkpoints with d_h^V != d_h, e.g. 192 / 256): both paths against the scalar-loop brute force
    with d_v != d_h; the softmax scale keeps the key dim; the extra value dims are plain extra columns of W^UV."""
    rng = np.random.default_rng(11)
    s_q, h_q, g, d_h, d_v, d_r, r_kv, L = 2, 6, 3, 4, 6, 2, 5, 7
    qC, qR = rng.normal(size=(s_q, h_q, d_h)), rng.normal(size=(s_q, h_q, d_r))
    c, kR = rng.normal(size=(L, r_kv)), rng.normal(size=(L, d_r))
    W_UK, W_UV = rng.normal(size=(g, r_kv, d_h)), rng.normal(size=(g, r_kv, d_v))
    ref = O.decode_mha_bruteforce(qC, qR, c, kR, W_UK, W_UV)
    assert ref.shape == (s_q, h_q, d_v)
    KC, V = O.expand_latent(c, W_UK, W_UV)
    assert KC.shape == (L, g, d_h) and V.shape == (L, g, d_v)
    o_g, lse_g = O.decode_gqa(qC, qR, KC, V, kR)
    o_a, lse_a = O.decode_absorb(O.absorb_query(qC, W_UK), qR, c, kR, W_UV, d_h=d_h)
    assert np.max(np.abs(o_g - ref)) < 1e-10 and np.max(np.abs(o_a - ref)) < 1e-10 and np.max(np.abs(lse_g - lse_a)) < 1e-10
    # the scale is 1/sqrt(d_h + d_R) with the KEY dim: taking the value dim instead changes the result
    o_wrong, _ = O.decode_absorb(O.absorb_query(qC, W_UK), qR, c, kR, W_UV)         # default: W^UV's columns
    assert np.max(np.abs(o_wrong - ref)) > 1e-4
    # the first d_h value columns do not care about the others
    o_cut, _ = O.decode_gqa(qC, qR, KC, V[:, :, :d_h], kR)
    assert np.max(np.abs(o_cut - ref[:, :, :d_h])) < 1e-12
