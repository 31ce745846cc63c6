"""GPU parity: every entry point of the C-ABI library against the CPU oracle, element by element, on the
same seeded input bits.  bf16 bar: max abs 2e-2 and relative L2 1e-2; fp32 bar: max abs 1e-4, relative L2 1e-5
(the fp32 kernels accumulate a few hundred fp32 products of O(1) values)."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import gqla_oracle as O
from oracle import layout as Lay

pytestmark = pytest.mark.gpu

TOL = {"bf16": (2e-2, 1e-2), "f32": (1e-4, 1e-5)}


def rel_l2(a, ref):
    a = np.asarray(a, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(a - ref) / max(np.linalg.norm(ref), 1e-300))


def check(name, got, ref, dtype):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert np.isfinite(got).all(), name + ": non-finite output"
    ma, rl = TOL[dtype]
    err = float(np.max(np.abs(got - ref)))
    r = rel_l2(got, ref)
    print("%-34s max_abs %.3e  rel_l2 %.3e" % (name, err, r), flush=True)
    assert err <= ma, "%s: max abs %.3e" % (name, err)
    assert r <= rl, "%s: rel l2 %.3e" % (name, r)


def host(t):
    return t.float().cpu().numpy()


class Case:
    """Host copies of everything plus the device-side Decoder."""

    def __init__(self, cfg, lens=None, groups=None, group_begin=0, use_page_table=True, chunk_pages=(0, 0), num_cus=256):
        from paper_2605_15250_amd.harness import Decoder, to_device, build_latent_pool
        self.cfg = cfg
        self.lens = S.seq_lens(cfg) if lens is None else np.asarray(lens, np.int32)
        cfg_t = cfg.with_(L=0) if lens is not None else cfg
        self.table, self.num_pages = S.page_table(cfg_t, self.lens)
        self.w_uk, self.w_uv = S.weights(cfg)
        self.q_c, self.q_r = S.queries(cfg)
        self.rows = [S.sequence_rows(cfg, b, self.lens[b]) for b in range(cfg.B)]
        self.dec = Decoder(cfg, self.lens, self.table, self.num_pages, groups=groups, group_begin=group_begin,
                           use_page_table=use_page_table, chunk_pages_absorb=chunk_pages[0], chunk_pages_gqa=chunk_pages[1],
                           num_cus=num_cus)
        self.dec.latent_pool = build_latent_pool(cfg, self.lens, self.table, self.num_pages, lambda b, L: self.rows[b])
        self.d_w_uk = to_device(self.w_uk, cfg.dtype)
        self.d_w_uv = to_device(self.w_uv, cfg.dtype)
        self.d_q_c = to_device(self.q_c, cfg.dtype)
        self.d_q_r = to_device(self.q_r, cfg.dtype)
        self.to_device = to_device

    def c(self, b):
        return self.rows[b][:, : self.cfg.r_kv]

    def kR(self, b):
        return self.rows[b][:, self.cfg.r_kv:]

    def close(self):
        self.dec.close()


def run_absorb_path(case, seqs=None):
    cfg = case.cfg
    seqs = range(cfg.B) if seqs is None else seqs
    # a1: query absorption
    q_hat = case.dec.absorb_query(case.d_q_c, case.d_w_uk)
    torch.cuda.synchronize()
    q_hat_h = host(q_hat)
    ref_qh = np.stack([O.absorb_query(case.q_c[b], case.w_uk) for b in range(cfg.B)])
    check("absorb_query", q_hat_h, ref_qh, cfg.dtype)
    # a2-a4 in isolation: the oracle consumes exactly the q_hat bits the GPU consumes
    out, lse = case.dec.decode_absorb(q_hat, case.d_q_r, case.d_w_uv)
    torch.cuda.synchronize()
    out_h, lse_h = host(out), host(lse)
    ref_o = np.zeros_like(out_h, dtype=np.float64)
    ref_l = np.zeros_like(lse_h, dtype=np.float64)
    for b in seqs:
        ref_o[b], ref_l[b] = O.decode_absorb(q_hat_h[b], case.q_r[b], case.c(b), case.kR(b), case.w_uv, d_h=cfg.d_h)
    sel = list(seqs)
    check("decode_absorb (isolated)", out_h[sel], ref_o[sel], cfg.dtype)
    check("decode_absorb lse", lse_h[sel], ref_l[sel], cfg.dtype)
    # chained against the unrounded oracle
    ref_c = np.stack([O.decode_absorb(ref_qh[b], case.q_r[b], case.c(b), case.kR(b), case.w_uv, d_h=cfg.d_h)[0] for b in seqs])
    check("absorb path (chained)", out_h[sel], ref_c, cfg.dtype)
    return out_h


def run_gqa_path(case, seqs=None):
    cfg = case.cfg
    dec = case.dec
    seqs = range(cfg.B) if seqs is None else seqs
    sel = list(seqs)
    G = cfg.h_q // cfg.g
    j0, gc = dec.group_begin, dec.groups
    heads = slice(j0 * G, (j0 + gc) * G)
    # a5: expansion on the GPU into a NaN-filled pool
    dec.alloc_expanded()
    pool = dec.expand(case.d_w_uk, case.d_w_uv)
    torch.cuda.synchronize()
    pool_h = host(pool)
    exp_ref = {}
    for b in seqs:
        KC, V = O.expand_latent(case.c(b), case.w_uk[j0:j0 + gc], case.w_uv[j0:j0 + gc])
        exp_ref[b] = (KC, V)
        k2, v2, r2 = Lay.unpack_expanded_seq(pool_h, case.table[b], case.lens[b], cfg.page_size, gc, cfg.d_h, cfg.d_r, cfg.dv)
        check("expand K_C seq %d" % b, k2, KC, cfg.dtype)
        check("expand V seq %d" % b, v2, V, cfg.dtype)
        assert np.array_equal(r2, case.kR(b)), "k_R must be copied bit for bit"
    # slots no token owns were never written: still NaN, and their count is exact
    per_tok = gc * (cfg.d_h + cfg.dv) + cfg.d_r
    assert int(np.isnan(pool_h).sum()) == pool_h.size - int(case.lens.sum()) * per_tok
    # a6 in isolation: both sides consume the oracle's expansion rounded to the storage type
    q_c_s = np.ascontiguousarray(case.q_c[:, :, heads, :])
    q_r_s = np.ascontiguousarray(case.q_r[:, :, heads, :])
    d_q_c, d_q_r = case.to_device(q_c_s, cfg.dtype), case.to_device(q_r_s, cfg.dtype)
    KCq, Vq = {}, {}
    KC_all, V_all, kR_all = [], [], []
    for b in range(cfg.B):
        if b in exp_ref:
            KC, V = exp_ref[b]
        else:
            KC, V = O.expand_latent(case.c(b), case.w_uk[j0:j0 + gc], case.w_uv[j0:j0 + gc])
        KCq[b], Vq[b] = S.quantize(KC, cfg.dtype), S.quantize(V, cfg.dtype)
        KC_all.append(KCq[b]); V_all.append(Vq[b]); kR_all.append(case.kR(b))
    iso_pool = Lay.pack_expanded_pool(KC_all, V_all, kR_all, case.table, case.num_pages, cfg.page_size)
    gpu_pool = dec.expanded_pool
    dec.expanded_pool = case.to_device(iso_pool, cfg.dtype)
    out, lse = dec.decode_gqa(d_q_c, d_q_r)
    torch.cuda.synchronize()
    out_h, lse_h = host(out), host(lse)
    ref_o = np.zeros_like(out_h, dtype=np.float64)
    ref_l = np.zeros_like(lse_h, dtype=np.float64)
    for b in seqs:
        ref_o[b], ref_l[b] = O.decode_gqa(q_c_s[b], q_r_s[b], KCq[b], Vq[b], case.kR(b))
    check("decode_gqa (isolated)", out_h[sel], ref_o[sel], cfg.dtype)
    check("decode_gqa lse", lse_h[sel], ref_l[sel], cfg.dtype)
    # chained: GPU expansion -> GPU decode against the unrounded oracle
    dec.expanded_pool = gpu_pool
    out2, _ = dec.decode_gqa(d_q_c, d_q_r)
    torch.cuda.synchronize()
    out2_h = host(out2)
    ref_c = np.stack([O.decode_gqa(q_c_s[b], q_r_s[b], exp_ref[b][0], exp_ref[b][1], case.kR(b))[0] for b in seqs])
    check("gqa path (chained)", out2_h[sel], ref_c, cfg.dtype)
    return out2_h


# ---- C0: the tiny fp32 configuration, everything checked, including the brute-force per-head attention ---------
def test_c0_fp32_both_paths():
    cfg = S.CONFIGS["C0"]
    case = Case(cfg)
    try:
        oa = run_absorb_path(case)
        og = run_gqa_path(case)
        brute = O.decode_mha_bruteforce(case.q_c[0], case.q_r[0], case.c(0), case.kR(0), case.w_uk, case.w_uv)
        check("absorb vs brute-force MHA", oa[0], brute, "f32")
        check("gqa vs brute-force MHA", og[0], brute, "f32")
    finally:
        case.close()


@pytest.mark.parametrize("s_q,lens,paged,cp", [
    (1, [64], False, (0, 0)),
    (2, [40, 7, 2], True, (0, 0)),          # L == s_q, ragged tails, permuted pages
    (2, [100, 33], True, (2, 3)),           # forced multi-page chunks
])
def test_fp32_small_shapes(s_q, lens, paged, cp):
    cfg = S.CONFIGS["C0"].with_(B=len(lens), s_q=s_q, L=0, paged=paged, page_size=8, seed=77)
    case = Case(cfg, lens=lens, chunk_pages=cp)
    try:
        run_absorb_path(case)
        run_gqa_path(case)
    finally:
        case.close()


# ---- bf16 MFMA kernels at the paper's head dims, small batch: several tiles, ragged tails, permuted pages ----------
@pytest.mark.parametrize("h_q,g,s_q,lens,paged,cp", [
    (128, 8, 1, [300, 64, 129], True, (0, 0)),
    (128, 8, 2, [257, 2, 1000, 65], True, (0, 0)),       # L == s_q, a chunk whose only token is hidden from row 0
    (128, 8, 2, [1500, 700], True, (4, 5)),              # multi-page chunks with a ragged last chunk
    (32, 8, 1, [513, 100], False, (3, 2)),               # LLaMA-3-8B-converted heads: G = 4 (padded MFMA rows)
    (128, 8, 2, [640], False, (0, 0)),                   # contiguous cache, no page table
    (64, 4, 1, [900, 333], True, (0, 0)),                # g = 4 (2176 bytes per token, Sec. 4.2.3): 4-wave workgroups
    (32, 2, 2, [450, 64], True, (2, 2)),                 # g = 2: 2-wave workgroups, each wave stages two k_R slabs
    (48, 3, 1, [300], True, (0, 0)),                     # g = 3: no k_R sharing (direct loads)
    (128, 8, 1, [20000], True, (0, 0)),                  # one long sequence: the plan cuts it into a few dozen chunks
    (128, 8, 2, [6000, 70], True, (1, 1)),               # forced one-page chunks: 94 partials to merge for one sequence
    (16, 8, 1, [777, 40], True, (0, 0)),                 # one rank's heads under 8-way head parallelism: 16 query rows,
                                                         # four waves share them in the absorb kernel (half its rows padding)
    (16, 4, 2, [2, 300, 1029], True, (1, 2)),            # 32 rows shared by four waves, L == s_q, ragged chunks
    (8, 8, 1, [130, 64], False, (0, 0)),                 # G = 1 (multi-head limit of the grouping): 8 rows
    (128, 4, 2, [700, 65], True, (0, 0)),                # (g, s_q) = (4, 2) at 128 heads: G = 32, 64 rows per group
    (128, 4, 1, [321], False, (0, 0)),                   # (g, s_q) = (4, 1), the 2176-byte-per-token operating point
    (64, 1, 1, [300, 70], True, (0, 0)),                 # one group of 64 heads: a GQA wave takes both 32-row blocks, no k_R sharing
    (96, 2, 2, [513, 64, 2], True, (0, 1)),              # 96 rows per group: two waves of two row blocks, the last block all padding
    (16, 1, 2, [700, 2, 65, 300], True, (0, 0)),         # one group, 32 rows: the eight waves of a GQA workgroup share a chunk's tiles;
                                                         # chunks of 1 and 3 tiles leave most of the team without any
    (32, 1, 1, [1029, 40], False, (0, 3)),               # the same with 32 heads, forced 3-page chunks (6 tiles for 8 waves)
    (8, 1, 1, [130, 5000], True, (0, 0)),                # 8 rows (24 lanes of padding), one long sequence
])
@pytest.mark.parametrize("num_cus", [256, 2])   # planned for the whole chip, or for a sliver of it: with few chunks and
                                                # many compute units the absorb decode gives every 32 query rows a
                                                # workgroup of their own, otherwise 128 rows share one
def test_bf16_small_batches(h_q, g, s_q, lens, paged, cp, num_cus):
    cfg = S.CONFIGS["C2"].with_(B=len(lens), h_q=h_q, g=g, s_q=s_q, L=0, paged=paged, seed=4242 + h_q + s_q)
    case = Case(cfg, lens=lens, use_page_table=paged, chunk_pages=cp, num_cus=num_cus)
    try:
        run_absorb_path(case)
        run_gqa_path(case)
    finally:
        case.close()


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        g = int(rng.choice([1, 2, 3, 4, 5, 6, 8, 16]))
        G = int(rng.choice([1, 2, 3, 4, 6, 8, 16, 32]))
        if g * G > 128:
            continue
        s_q = int(rng.integers(1, 3))
        page_size = int(rng.choice([64, 128]))
        lens = [int(x) for x in rng.integers(s_q, 700, size=int(rng.integers(1, 4)))]
        cases.append((g * G, g, s_q, page_size, lens, bool(rng.integers(0, 2)), (int(rng.integers(0, 4)), int(rng.integers(0, 4)))))
    return cases


@pytest.mark.parametrize("h_q,g,s_q,page_size,lens,paged,cp", _random_cases(12, 20260515))
def test_bf16_random_shapes(h_q, g, s_q, page_size, lens, paged, cp):
    """Seeded random draws over what the bf16 kernels accept: group counts with and without k_R sharing, 1 to 32 heads
    per group (1 to 64 rows per group, 1 to 256 query rows per sequence), both page sizes, ragged lengths, forced
    chunk sizes, permuted or identity page tables."""
    cfg = S.CONFIGS["C2"].with_(B=len(lens), h_q=h_q, g=g, s_q=s_q, L=0, paged=paged, page_size=page_size, seed=9000 + h_q + g)
    case = Case(cfg, lens=lens, use_page_table=paged, chunk_pages=cp)
    try:
        run_absorb_path(case)
        run_gqa_path(case)
    finally:
        case.close()


@pytest.mark.parametrize("cp", [(0, 0), (1, 1)])
def test_bf16_length_sweep(cp):
    """Every length from s_q to s_q + 160 in one batch: one to six tiles per chunk in the absorb kernel's tile ring
    (fewer tiles than ring slots included), every tail length, lengths on and next to page boundaries; with one-page
    chunks every chunk has at most two tiles and most sequences are split."""
    s_q = 2
    lens = list(range(s_q, s_q + 161))
    cfg = S.CONFIGS["C2"].with_(B=len(lens), h_q=32, g=8, s_q=s_q, L=0, paged=True, seed=777)
    case = Case(cfg, lens=lens, chunk_pages=cp)
    try:
        run_absorb_path(case)
        run_gqa_path(case)
    finally:
        case.close()


@pytest.mark.parametrize("page_size,lens", [
    (1024, [1500, 70, 1024]),     # the largest page the MFMA kernels take; a sequence that ends exactly on a page boundary
    (192, [500, 193, 64]),        # a page size that is a multiple of 64 but not a power of two
])
def test_bf16_page_sizes(page_size, lens):
    cfg = S.CONFIGS["C3"].with_(B=len(lens), L=0, paged=True, page_size=page_size, seed=5150 + page_size)
    case = Case(cfg, lens=lens)
    try:
        run_absorb_path(case)
        run_gqa_path(case)
    finally:
        case.close()


@pytest.mark.parametrize("h_q,num_cus", [(128, 2), (128, 256), (16, 256)])   # absorb kernel: one wave per 32 query
                                                                              # rows, or four sharing them
def test_bf16_growing_logits(monkeypatch, h_q, num_cus):
    """Logits that keep growing along the sequence and reach far beyond the usual range: the reference maximum of the
    absorb kernel's online softmax has to move many times (it only moves in steps of more than 2^8), and both kernels
    must keep their exponentials in range.  The RoPE key of a cached token (which enters the logits only, so the outputs
    stay O(1)) is scaled by a factor that rises from 1 to 8 with the position, so late tokens dominate; the oracle sees
    exactly the same rows."""
    real_rows = S.sequence_rows

    def growing_rows(cfg, b, L_b):
        rows = real_rows(cfg, b, L_b).astype(np.float64)
        ramp = 1.0 + 7.0 * np.arange(int(L_b), dtype=np.float64) / max(int(L_b) - 1, 1)
        rows[:, cfg.r_kv:] *= ramp[:, None]
        return S.quantize(rows.astype(np.float32), cfg.dtype)

    monkeypatch.setattr(S, "sequence_rows", growing_rows)
    cfg = S.CONFIGS["C3"].with_(B=2, h_q=h_q, L=0, paged=True, seed=8128)
    case = Case(cfg, lens=[1500, 333], num_cus=num_cus)
    try:
        run_absorb_path(case)
        run_gqa_path(case)
    finally:
        case.close()


def test_bf16_single_group_slice():
    """One rank's share of 8-way head-axis tensor parallelism: 16 heads, one group, 320 elements per token."""
    cfg = S.CONFIGS["C3"].with_(B=2, L=0, paged=True, seed=909)
    case = Case(cfg, lens=[700, 130], groups=1, group_begin=5)
    try:
        run_gqa_path(case)
    finally:
        case.close()


def test_page_permutation_is_bit_identical():
    """Same logical data under an identity and a permuted page table, same plan: identical output bits."""
    lens = [400, 90]
    outs = []
    for paged in (False, True):
        cfg = S.CONFIGS["C3"].with_(B=2, L=0, paged=paged, seed=31337)
        case = Case(cfg, lens=lens, use_page_table=True)
        try:
            q_hat = case.dec.absorb_query(case.d_q_c, case.d_w_uk)
            oa, la = case.dec.decode_absorb(q_hat, case.d_q_r, case.d_w_uv)
            case.dec.alloc_expanded()
            case.dec.expand(case.d_w_uk, case.d_w_uv)
            og, lg = case.dec.decode_gqa(case.d_q_c, case.d_q_r)
            torch.cuda.synchronize()
            outs.append([x.clone().cpu() for x in (oa, la, og, lg)])
        finally:
            case.close()
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


@pytest.mark.parametrize("key,h_q,g,d_h,d_v,s_q,lens", [
    ("C2", 20, 4, 192, 256, 1, [300, 4000, 64]),     # the MLA checkpoint shape of Sec. 3.2.2 (h_q = 20, d_h = 192, d_h^V = 256), g = 4
    ("C2", 20, 5, 192, 256, 2, [129, 1000]),         # the same with g = 5 and two step tokens
    ("C2", 128, 8, 128, 256, 2, [700, 65]),          # only the value dim differs; 256 query rows
    ("C2", 32, 8, 192, 128, 1, [513]),               # only the key dim differs
    ("C0", 8, 2, 16, 24, 2, [40, 7, 2]),             # fp32 kernels
])
def test_absorb_path_with_a_value_dim_of_its_own(key, h_q, g, d_h, d_v, s_q, lens):
    """d_h^V != d_h (Sec. 3.2.2) on the absorb path: query absorption over d_h key dims, the latent decode with the scale
    1/sqrt(d_h + d_R), W_UV with d_v columns, and W^O over h_q d_v columns, against the oracle."""
    cfg = S.CONFIGS[key].with_(B=len(lens), h_q=h_q, g=g, d_h=d_h, d_v=d_v, s_q=s_q, L=0, paged=True,
                               page_size=64 if key != "C0" else 8, seed=6006 + d_h + d_v)
    case = Case(cfg, lens=lens)
    try:
        out = run_absorb_path(case)
        assert out.shape == (cfg.B, s_q, h_q, d_v)
        d_model = 256 if cfg.dtype == "bf16" else 24
        w_o = S.output_weights(cfg, d_model)
        assert w_o.shape == (d_model, h_q * d_v)
        if cfg.dtype == "bf16" and (h_q * d_v) % 256:
            return
        o_dev = case.to_device(out, cfg.dtype)                       # the GPU's own (storage-rounded) outputs
        y = case.dec.output_projection(o_dev, case.to_device(w_o, cfg.dtype))
        torch.cuda.synchronize()
        ref = np.stack([O.output_projection(S.quantize(out[b], cfg.dtype), w_o) for b in range(cfg.B)])
        check("W^O over h_q * d_v columns", host(y), ref, cfg.dtype)
    finally:
        case.close()


@pytest.mark.parametrize("key,h_q,g,d_h,d_v,s_q,lens,paged,cp", [
    ("C2", 20, 4, 192, 256, 1, [300, 4000, 64], True, (0, 0)),    # the MLA checkpoint shape of Sec. 3.2.2, g = 4 (G = 5)
    ("C2", 20, 5, 192, 256, 2, [129, 1000], True, (0, 1)),        # g = 5 (G = 4, no k_R sharing between waves), two step tokens
    ("C2", 128, 8, 192, 256, 2, [700, 65, 2], False, (0, 0)),     # 8 groups of 16 heads, contiguous pages, L == s_q
    ("C2", 32, 2, 192, 256, 1, [513], True, (0, 2)),              # 2 groups of 16 heads
    ("C0", 8, 2, 16, 24, 2, [40, 7, 2], True, (0, 0)),            # fp32 kernels, value dim larger than the key dim
    ("C0", 6, 3, 24, 8, 1, [33], True, (0, 0)),                   # fp32 kernels, value dim smaller than the key dim
])
def test_both_paths_with_a_value_dim_of_its_own(key, h_q, g, d_h, d_v, s_q, lens, paged, cp):
    """d_h^V != d_h (Sec. 3.2.2) through the expanded cache: the one-shot expansion (K plane with d_h dims, V plane with
    d_v dims), the GQA-path decode over it, the absorb path on the same weights, each against the oracle, and the
    paper's statement that the two paths give the same attention output (Sec. 3.1) between the two GPU paths."""
    cfg = S.CONFIGS[key].with_(B=len(lens), h_q=h_q, g=g, d_h=d_h, d_v=d_v, s_q=s_q, L=0, paged=paged,
                               page_size=64 if key != "C0" else 8, seed=7007 + d_h + d_v + h_q)
    case = Case(cfg, lens=lens, use_page_table=paged, chunk_pages=cp)
    try:
        out_a = run_absorb_path(case)
        out_g = run_gqa_path(case)
        assert out_a.shape == out_g.shape == (cfg.B, s_q, h_q, d_v)
        check("absorb path vs gqa path", out_a, out_g, cfg.dtype)
    finally:
        case.close()


@pytest.mark.parametrize("h_q,g,lens", [(20, 4, [200, 2, 65, 1000]), (128, 8, [300, 64])])
def test_step_updates_with_a_value_dim_of_its_own(h_q, g, lens):
    """(d_h, d_v) = (192, 256): the step's positions expanded by the tail variant hold bit for bit what the one-shot
    expansion writes there, nothing else is written, and the reverse cache switch recovers the latent."""
    from paper_2605_15250_amd import binding as B_
    cfg = S.CONFIGS["C2"].with_(B=len(lens), h_q=h_q, g=g, d_h=192, d_v=256, s_q=2, L=0, paged=True, seed=7100 + h_q)
    case = Case(cfg, lens=lens)
    dec = case.dec
    try:
        dec.alloc_expanded(fill=0.0)
        dec.expand(case.d_w_uk, case.d_w_uv)
        torch.cuda.synchronize()
        one_shot = dec.expanded_pool.clone()
        dec.alloc_expanded()                          # NaN everywhere
        dec.expand_tail(case.d_w_uk, case.d_w_uv, cfg.s_q)
        torch.cuda.synchronize()
        got = dec.expanded_pool
        written = ~torch.isnan(got.float())
        per_tok = cfg.g * (cfg.d_h + cfg.dv) + cfg.d_r
        assert int(written.sum()) == cfg.B * cfg.s_q * per_tok
        assert torch.equal(got[written].view(torch.int16), one_shot[written].view(torch.int16))
        pool_h = host(got)
        for b in range(cfg.B):
            L = int(case.lens[b])
            k2, v2, r2 = Lay.unpack_expanded_seq(pool_h, case.table[b], L, cfg.page_size, cfg.g, cfg.d_h, cfg.d_r, cfg.dv)
            assert np.isfinite(k2[L - cfg.s_q:]).all() and np.isfinite(v2[L - cfg.s_q:]).all() and np.isfinite(r2[L - cfg.s_q:]).all()
            assert np.isnan(k2[:L - cfg.s_q]).all() and np.isnan(v2[:L - cfg.s_q]).all()
        # reverse switch: latent from the expanded keys through the left inverse of the stacked key up-projection
        dec.expanded_pool = one_shot
        w_inv = B_.gqla_left_inverse(dec.shape, case.w_uk)
        truth = dec.latent_pool
        dec.latent_pool = torch.zeros_like(truth)
        dec.compress(case.to_device(S.quantize(w_inv, cfg.dtype), cfg.dtype))
        torch.cuda.synchronize()
        W = cfg.r_kv + cfg.d_r
        rec_h, tru_h = host(dec.latent_pool).reshape(-1, W), host(truth).reshape(-1, W)
        for b in range(cfg.B):
            t = np.arange(int(case.lens[b]))
            rows = case.table[b][t // cfg.page_size].astype(np.int64) * cfg.page_size + t % cfg.page_size
            assert np.array_equal(rec_h[rows, cfg.r_kv:], tru_h[rows, cfg.r_kv:]), "k_R is copied"
            r = rel_l2(rec_h[rows, :cfg.r_kv], tru_h[rows, :cfg.r_kv])
            print("recovered latent, sequence %d: rel_l2 %.3e" % (b, r), flush=True)
            assert r <= 2e-2      # what the 16-bit roundings of the keys and of the left inverse cost
        dec.latent_pool = truth
    finally:
        case.close()
