"""Pins for the oracle's integer bookkeeping: offsets are bijections onto the page, the packers
restate the scalar offset functions, and the split plan partitions every sequence."""
import numpy as np
import pytest

from oracle import layout as Lay


@pytest.mark.parametrize("P,g_c,d_h,d_r", [(16, 2, 16, 8), (64, 8, 128, 64), (32, 1, 128, 64), (8, 3, 24, 16)])
def test_expanded_offsets_tile_each_page_exactly_once(P, g_c, d_h, d_r):
    pe = Lay.expanded_page_elems(P, g_c, d_h, d_r)
    assert pe == P * Lay.expanded_elems_per_token(g_c, d_h, d_r)
    for page in (0, 3):
        seen = np.zeros(pe, dtype=np.int32)
        for s in range(P):
            for j in range(g_c):
                for d in range(d_h):
                    seen[Lay.expanded_k_offset(page, j, s, d, P, g_c, d_h, d_r) - page * pe] += 1
                    seen[Lay.expanded_v_offset(page, j, s, d, P, g_c, d_h, d_r) - page * pe] += 1
            for d in range(d_r):
                seen[Lay.expanded_kr_offset(page, s, d, P, g_c, d_h, d_r) - page * pe] += 1
        assert (seen == 1).all()


def test_expanded_layout_vector_contiguity():
    P, g_c, d_h, d_r = 64, 8, 128, 64
    # 8 consecutive dims of one token are adjacent in the K and k_R planes
    for d in range(7):
        assert Lay.expanded_k_offset(1, 3, 17, 8 + d + 1, P, g_c, d_h, d_r) == Lay.expanded_k_offset(1, 3, 17, 8 + d, P, g_c, d_h, d_r) + 1
        assert Lay.expanded_kr_offset(1, 17, 8 + d + 1, P, g_c, d_h, d_r) == Lay.expanded_kr_offset(1, 17, 8 + d, P, g_c, d_h, d_r) + 1
    # 8 consecutive tokens of one dim are adjacent in the V plane
    for s in range(7):
        assert Lay.expanded_v_offset(1, 3, 16 + s + 1, 5, P, g_c, d_h, d_r) == Lay.expanded_v_offset(1, 3, 16 + s, 5, P, g_c, d_h, d_r) + 1
    # consecutive tokens are 8 elements apart inside a K vector column
    assert Lay.expanded_k_offset(0, 0, 1, 0, P, g_c, d_h, d_r) - Lay.expanded_k_offset(0, 0, 0, 0, P, g_c, d_h, d_r) == 8


def test_packers_restate_scalar_offsets():
    P, g_c, d_h, d_r = 8, 2, 16, 8
    r = np.random.default_rng(0)
    lens = [5, 19]
    table = np.array([[4, -1, -1], [2, 0, 3]], dtype=np.int32)
    KC = [r.standard_normal((L, g_c, d_h)).astype(np.float32) for L in lens]
    V = [r.standard_normal((L, g_c, d_h)).astype(np.float32) for L in lens]
    kR = [r.standard_normal((L, d_r)).astype(np.float32) for L in lens]
    pool = Lay.pack_expanded_pool(KC, V, kR, table, 5, P)
    for b, L in enumerate(lens):
        for t in range(L):
            page, slot = Lay.phys_token(table[b], t, P)
            for j in range(g_c):
                for d in range(d_h):
                    assert pool[Lay.expanded_k_offset(page, j, slot, d, P, g_c, d_h, d_r)] == KC[b][t, j, d]
                    assert pool[Lay.expanded_v_offset(page, j, slot, d, P, g_c, d_h, d_r)] == V[b][t, j, d]
            for d in range(d_r):
                assert pool[Lay.expanded_kr_offset(page, slot, d, P, g_c, d_h, d_r)] == kR[b][t, d]
        k2, v2, r2 = Lay.unpack_expanded_seq(pool, table[b], L, P, g_c, d_h, d_r)
        assert np.array_equal(k2, KC[b]) and np.array_equal(v2, V[b]) and np.array_equal(r2, kR[b])
    # every slot not owned by a token keeps the fill value
    assert np.isnan(pool).sum() == 5 * Lay.expanded_page_elems(P, g_c, d_h, d_r) - sum(lens) * (2 * g_c * d_h + d_r)


@pytest.mark.parametrize("P,g_c,d_h,d_v,d_r", [(16, 2, 16, 24, 8), (64, 4, 192, 256, 64), (8, 3, 24, 8, 16)])
def test_expanded_offsets_with_a_value_dim_of_its_own(P, g_c, d_h, d_v, d_r):
    """d_h^V != d_h (Sec. 3.2.2): a token takes g (d_h + d_v) + d_R elements, the three planes still tile the page
    exactly once, V vectors still hold 8 consecutive tokens of one dim, and d_v = d_h gives the equal-dims offsets."""
    pe = Lay.expanded_page_elems(P, g_c, d_h, d_r, d_v)
    assert pe == P * (g_c * (d_h + d_v) + d_r)
    page = 2
    seen = np.zeros(pe, dtype=np.int32)
    for s in range(P):
        for j in range(g_c):
            for d in range(d_h):
                seen[Lay.expanded_k_offset(page, j, s, d, P, g_c, d_h, d_r, d_v) - page * pe] += 1
            for d in range(d_v):
                seen[Lay.expanded_v_offset(page, j, s, d, P, g_c, d_h, d_r, d_v) - page * pe] += 1
        for d in range(d_r):
            seen[Lay.expanded_kr_offset(page, s, d, P, g_c, d_h, d_r, d_v) - page * pe] += 1
    assert (seen == 1).all()
    for s in range(7):
        assert (Lay.expanded_v_offset(1, g_c - 1, s + 1, d_v - 1, P, g_c, d_h, d_r, d_v)
                == Lay.expanded_v_offset(1, g_c - 1, s, d_v - 1, P, g_c, d_h, d_r, d_v) + 1)
    # the planes come in the order K, V, k_R: the first V element sits right behind the last K element
    assert Lay.expanded_v_offset(0, 0, 0, 0, P, g_c, d_h, d_r, d_v) == g_c * P * d_h
    assert Lay.expanded_kr_offset(0, 0, 0, P, g_c, d_h, d_r, d_v) == g_c * P * (d_h + d_v)
    for args in ((1, 1, 3, 5), (0, 0, 7, 0)):
        assert Lay.expanded_v_offset(*args, P, g_c, d_h, d_r, d_h) == Lay.expanded_v_offset(*args, P, g_c, d_h, d_r)
        assert Lay.expanded_k_offset(*args, P, g_c, d_h, d_r, d_h) == Lay.expanded_k_offset(*args, P, g_c, d_h, d_r)
    # packer and unpacker restate the scalar offsets
    r = np.random.default_rng(1)
    lens = [P + 3, 2]
    table = np.array([[1, 3], [0, -1]], dtype=np.int32)
    KC = [r.standard_normal((L, g_c, d_h)).astype(np.float32) for L in lens]
    V = [r.standard_normal((L, g_c, d_v)).astype(np.float32) for L in lens]
    kR = [r.standard_normal((L, d_r)).astype(np.float32) for L in lens]
    pool = Lay.pack_expanded_pool(KC, V, kR, table, 4, P)
    assert pool.size == 4 * pe and np.isnan(pool).sum() == 4 * pe - sum(lens) * (g_c * (d_h + d_v) + d_r)
    for b, L in enumerate(lens):
        for t in (0, L - 1):
            pg, slot = Lay.phys_token(table[b], t, P)
            for j in (0, g_c - 1):
                for d in range(d_h):
                    assert pool[Lay.expanded_k_offset(pg, j, slot, d, P, g_c, d_h, d_r, d_v)] == KC[b][t, j, d]
                for d in range(d_v):
                    assert pool[Lay.expanded_v_offset(pg, j, slot, d, P, g_c, d_h, d_r, d_v)] == V[b][t, j, d]
            for d in range(d_r):
                assert pool[Lay.expanded_kr_offset(pg, slot, d, P, g_c, d_h, d_r, d_v)] == kR[b][t, d]
        k2, v2, r2 = Lay.unpack_expanded_seq(pool, table[b], L, P, g_c, d_h, d_r, d_v)
        assert np.array_equal(k2, KC[b]) and np.array_equal(v2, V[b]) and np.array_equal(r2, kR[b])


def test_latent_offsets_and_phys_token():
    P, r_kv, d_r = 64, 512, 64
    assert Lay.latent_offset(0, 0, 0, P, r_kv, d_r) == 0
    assert Lay.latent_offset(0, 1, 0, P, r_kv, d_r) == 576
    assert Lay.latent_offset(2, 3, 512, P, r_kv, d_r) == (2 * 64 + 3) * 576 + 512
    assert Lay.phys_token([7, 9, 4], 0, 64) == (7, 0)
    assert Lay.phys_token([7, 9, 4], 64, 64) == (9, 0)
    assert Lay.phys_token([7, 9, 4], 191, 64) == (4, 63)
    assert Lay.contiguous_page(3, 5, 128) == 389
    assert Lay.pages_needed(1, 64) == 1 and Lay.pages_needed(64, 64) == 1 and Lay.pages_needed(65, 64) == 2


@pytest.mark.parametrize("path", [Lay.PATH_ABSORB, Lay.PATH_GQA])
@pytest.mark.parametrize("lens", [[8192] * 64, [4096] * 32, [1], [64, 65, 63, 128, 1000], list(range(1024, 32768, 997))])
def test_plan_partitions_every_sequence(lens, path):
    P = 64
    cp = Lay.plan_chunk_pages(lens, P, 256, path, 128, 8, 2)
    assert 1 <= cp <= max(Lay.pages_needed(L, P) for L in lens)
    chunks, first = Lay.plan_chunks(lens, P, cp)
    assert len(first) == len(lens)
    at = 0
    for b, L in enumerate(lens):
        assert first[b] == at
        lo_expect = 0
        while at < len(chunks) and chunks[at][0] == b:
            _, lo, hi = chunks[at]
            assert lo == lo_expect and lo % P == 0 and lo < hi <= L
            assert hi - lo <= cp * P
            assert hi == L or hi % P == 0
            lo_expect = hi
            at += 1
        assert lo_expect == L
    assert at == len(chunks)


def test_plan_known_cases():
    # canonical uniform cases: one chunk per compute unit
    assert Lay.plan_chunk_pages([8192] * 64, 64, 256, Lay.PATH_ABSORB, 128, 8, 1) == 32
    assert Lay.plan_chunk_pages([4096] * 32, 64, 256, Lay.PATH_GQA, 32, 8, 1) == 8
    # one 8192-token sequence (128 pages) on 256 compute units, costs by hand in eightieths of a page time
    # (weight * rounds * (cp + overhead) + merge * chunks of the sequence):
    #   absorb (overhead 4, merge 16; every cp >= 2 gives at most 64 chunks, i.e. 64 * 4 row blocks <= 256 workgroups, so
    #   the shared-row launch applies and a page weighs 53): cp 5 -> 53*9 + 16*26 = 893, cp 6 -> 53*10 + 16*22 = 882,
    #   cp 7 -> 53*11 + 16*19 = 887, cp 8 -> 53*12 + 16*16 = 892
    assert Lay.plan_chunk_pages([8192], 64, 256, Lay.PATH_ABSORB, 128, 8, 1) == 6
    #   gqa (overhead 2, merge 5, weight 80): cp 2 -> 320 + 320 = 640, cp 3 -> 400 + 215 = 615, cp 4 -> 480 + 160 = 640
    assert Lay.plan_chunk_pages([8192], 64, 256, Lay.PATH_GQA, 128, 8, 1) == 3
    # without the merge term both would be cut into one-page chunks: a longer chain of partials costs more than it saves
    #   1024 pages: cp 18 -> 57 chunks: 53*22 + 16*57 = 2078; cp 19 -> 54: 53*23 + 16*54 = 2083; cp 17 -> 61: 53*21 + 16*61 = 2089
    assert Lay.plan_chunk_pages([65536], 64, 256, Lay.PATH_ABSORB, 128, 8, 1) == 18
    # four such sequences: with cp 8 there are 64 chunks, the last count at which every 32 rows get a workgroup of their
    # own (64 * 4 = 256): 53*12 + 16*16 = 892; cp 6 (88 chunks, ordinary launch) would cost 80*10 + 16*22 = 1152
    assert Lay.plan_chunk_pages([8192] * 4, 64, 256, Lay.PATH_ABSORB, 128, 8, 1) == 8
    # and four sequences of 32768 tokens: the shared-row launch needs cp >= 32 (53*36 + 16*16 = 2164), the ordinary one
    # gets by with cp 11 or 12 (80*15 + 16*47 = 1952, 80*16 + 16*43 = 1968)
    assert Lay.plan_chunk_pages([32768] * 4, 64, 256, Lay.PATH_ABSORB, 128, 8, 1) == 11
    assert Lay.plan_page_weight(Lay.PATH_ABSORB, 64, 256, 128, 1) == 53 and Lay.plan_page_weight(Lay.PATH_ABSORB, 65, 256, 128, 1) == 80
    assert Lay.plan_page_weight(Lay.PATH_ABSORB, 10**6, 256, 32, 1) == 53 and Lay.plan_page_weight(Lay.PATH_GQA, 1, 256, 128, 1) == 80
    #   s_q = 2 halves the chunk count at which that launch applies (256 rows = 8 row blocks)
    assert Lay.plan_page_weight(Lay.PATH_ABSORB, 32, 256, 128, 2) == 53 and Lay.plan_page_weight(Lay.PATH_ABSORB, 33, 256, 128, 2) == 80
    chunks, first = Lay.plan_chunks([130, 64], 64, 2)
    assert chunks == [(0, 0, 128), (0, 128, 130), (1, 0, 64)] and first == [0, 2]
    chunks, _ = Lay.plan_chunks([64 * 5], 64, 2)              # 5 pages, cp 2 -> 3 chunks of 2,2,1
    assert chunks == [(0, 0, 128), (0, 128, 256), (0, 256, 320)]
    chunks, _ = Lay.plan_chunks([64 * 9], 64, 4)              # 9 pages, cp 4 -> 3 chunks of 3 pages
    assert chunks == [(0, 0, 192), (0, 192, 384), (0, 384, 576)]
