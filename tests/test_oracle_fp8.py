"""Pins of the 8-bit cache oracle (oracle/fp8_cache.py): the E4M3 code table against the format's definition,
the quantiser against a brute-force nearest-code search with ties to even, and the page format's offsets."""
import numpy as np

from oracle import fp8_cache as F8


def test_code_table_matches_the_format_definition():
    # landmarks of the OCP E4M3 ("FN") format: largest finite 448 = S.1111.110, smallest normal 2^-6, smallest
    # subnormal 2^-9, one NaN code per sign, no infinities, 1.0 = 0.0111.000
    t = F8.E4M3_TABLE
    assert t[0x7E] == 448.0 and t[0xFE] == -448.0
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isfinite(np.delete(t, [0x7F, 0xFF])).all()
    assert t[0x08] == 2.0 ** -6 and t[0x01] == 2.0 ** -9 and t[0x07] == 7 * 2.0 ** -9
    assert t[0x38] == 1.0 and t[0x3C] == 1.5 and t[0x40] == 2.0 and t[0x00] == 0.0
    pos = t[:0x7F]
    assert (np.diff(pos) > 0).all()                        # codes are ordered like their values
    assert np.array_equal(t[0x80:0xFF], -pos)


def _brute_force(x):
    """Nearest finite code by exhaustive search; on a tie the code with the even mantissa; saturating."""
    t = F8.E4M3_TABLE[:0x7F]
    a = min(abs(float(x)), 448.0)
    d = np.abs(t - a)
    best = np.flatnonzero(d == d.min())
    c = int(best[0]) if len(best) == 1 else int([b for b in best if b % 2 == 0][0])
    return c | (0x80 if np.signbit(np.float32(x)) else 0)


def test_quantiser_against_brute_force():
    t = F8.E4M3_TABLE[:0x7F]
    xs = [0.0, -0.0, 448.0, 449.0, 464.0, 480.0, 1e6, 1e-12, 2.0 ** -10, 3 * 2.0 ** -10]
    for c in range(0x7E):
        mid = 0.5 * (t[c] + t[c + 1])
        xs += [t[c], mid, np.nextafter(np.float32(mid), np.float32(0)), np.nextafter(np.float32(mid), np.float32(1e9))]
    rng = np.random.default_rng(8)
    xs += list(rng.normal(size=4000) * np.exp(rng.uniform(-8, 6, size=4000)))
    xs = np.array(xs, dtype=np.float32)
    xs = np.concatenate([xs, -xs])
    got = F8.quantize_e4m3(xs)
    want = np.array([_brute_force(x) for x in xs], dtype=np.uint8)
    assert np.array_equal(got, want)
    # every finite code survives a round trip
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], dtype=np.uint8)
    assert np.array_equal(F8.quantize_e4m3(F8.dequantize_e4m3(codes).astype(np.float32)), codes)


def test_quantisation_error_bound():
    # relative error at most 2^-4 (half of the 2^-3 mantissa step) for normal values, absolute 2^-10 below 2^-6
    rng = np.random.default_rng(3)
    x = (rng.normal(size=20000) * 3).astype(np.float32)
    q = F8.dequantize_e4m3(F8.quantize_e4m3(x))
    big = np.abs(x) >= 2.0 ** -6
    assert (np.abs(q[big] - x[big]) <= np.abs(x[big]) * 2.0 ** -4 + 1e-12).all()
    assert (np.abs(q[~big] - x[~big]) <= 2.0 ** -10 + 1e-12).all()


def test_scaled_quantisation_uses_the_fp32_product():
    x = np.array([3.3, -7.7, 100.0], dtype=np.float32)
    s = 0.3
    inv = np.float32(1.0) / np.float32(s)
    assert np.array_equal(F8.quantize_tensor(x, s), F8.quantize_e4m3(x * inv))


def test_page_format_is_a_bijection_and_matches_the_written_rule():
    P, g, d_h, d_r = 64, 2, 32, 16
    pb = F8.fp8_page_bytes(P, g, d_h, d_r)
    assert pb == P * (2 * g * d_h + 2 * d_r)
    seen = np.zeros(2 * pb, dtype=np.int32)
    for page in (0, 1):
        for s in range(P):
            for j in range(g):
                for d in range(d_h):
                    seen[F8.k8_offset(page, j, s, d, P, g, d_h, d_r)] += 1
                    seen[F8.v8_offset(page, j, s, d, P, g, d_h, d_r)] += 1
            for d in range(d_r):
                o = F8.kr16_offset(page, s, d, P, g, d_h, d_r)
                seen[o] += 1
                seen[o + 1] += 1
    assert (seen == 1).all()                               # every byte of both pages owned exactly once
    # spot values of the rule: dim 32 kp + 16 u + 8 h + i -> vector 2 kp + h, byte 8 u + i
    assert F8.k8_offset(0, 0, 5, 0, P, g, d_h, d_r) == 5 * 16
    assert F8.k8_offset(0, 0, 5, 8, P, g, d_h, d_r) == (1 * P + 5) * 16          # h = 1 -> vector 1
    assert F8.k8_offset(0, 0, 5, 16, P, g, d_h, d_r) == 5 * 16 + 8               # u = 1 -> second half of vector 0
    assert F8.k8_offset(0, 1, 0, 0, P, g, d_h, d_r) == (d_h // 16) * P * 16      # next group
    assert F8.v8_offset(0, 0, 0, 3, P, g, d_h, d_r) == g * P * d_h + 3 * 32
    assert F8.v8_offset(0, 0, 8, 3, P, g, d_h, d_r) == g * P * d_h + 3 * 32 + 16  # slot 8: h = 1
    assert F8.v8_offset(0, 0, 16, 3, P, g, d_h, d_r) == g * P * d_h + 3 * 32 + 8  # slot 16: u = 1
    assert F8.v8_offset(0, 0, 32, 0, P, g, d_h, d_r) == g * P * d_h + d_h * 32    # next 32-token tile
    # the whole-pool packer agrees with the element rule
    rng = np.random.default_rng(1)
    L = 70
    kc = rng.integers(0, 255, size=(L, g, d_h), dtype=np.uint8)
    vv = rng.integers(0, 255, size=(L, g, d_h), dtype=np.uint8)
    kr = rng.integers(0, 65535, size=(L, d_r), dtype=np.uint16)
    table = [np.array([1, 0])]
    pool = F8.pack_fp8_pool([kc], [vv], [kr], table, 2, P)
    for s in (0, 7, 33, 64, 69):
        page, slot = table[0][s // P], s % P
        for j in range(g):
            for d in (0, 9, 17, 31):
                assert pool[F8.k8_offset(page, j, slot, d, P, g, d_h, d_r)] == kc[s, j, d]
                assert pool[F8.v8_offset(page, j, slot, d, P, g, d_h, d_r)] == vv[s, j, d]
        for d in (0, 15):
            o = F8.kr16_offset(page, slot, d, P, g, d_h, d_r)
            assert int(pool[o]) | (int(pool[o + 1]) << 8) == int(kr[s, d])


def test_latent_page_format_is_a_bijection_and_matches_the_written_rule():
    """8-bit latent cache (absorb path): codes [P][r_kv] then k_R [P][d_R] in 16 bits; r_kv + 2 d_R bytes per token."""
    P, r_kv, d_r = 64, 32, 16
    pb = F8.latent_fp8_page_bytes(P, r_kv, d_r)
    assert pb == P * (r_kv + 2 * d_r)
    # the canonical shape: 512 code bytes + 128 bytes of 16-bit RoPE key against 2 (r_kv + d_R) = 1152 (Sec. 4.2.1)
    assert F8.latent_fp8_page_bytes(1, 512, 64) == 640 and 2 * (512 + 64) == 1152
    seen = np.zeros(2 * pb, dtype=np.int32)
    for page in (0, 1):
        for s in range(P):
            for d in range(r_kv):
                seen[F8.latent_code_offset(page, s, d, P, r_kv, d_r)] += 1
            for d in range(d_r):
                o = F8.latent_kr16_offset(page, s, d, P, r_kv, d_r)
                seen[o] += 1
                seen[o + 1] += 1
    assert (seen == 1).all()
    assert F8.latent_code_offset(0, 0, 0, P, r_kv, d_r) == 0
    assert F8.latent_code_offset(0, 3, 5, P, r_kv, d_r) == 3 * r_kv + 5           # token rows back to back
    assert F8.latent_code_offset(1, 0, 0, P, r_kv, d_r) == pb
    assert F8.latent_kr16_offset(0, 0, 0, P, r_kv, d_r) == P * r_kv                # the key plane starts behind all codes
    assert F8.latent_kr16_offset(0, 2, 1, P, r_kv, d_r) == P * r_kv + (2 * d_r + 1) * 2
    rng = np.random.default_rng(2)
    L = 70
    cc = rng.integers(0, 255, size=(L, r_kv), dtype=np.uint8)
    kr = rng.integers(0, 65535, size=(L, d_r), dtype=np.uint16)
    table = [np.array([1, 0])]
    pool = F8.pack_latent_fp8_pool([cc], [kr], table, 2, P, fill=0x55)
    for s in (0, 7, 63, 64, 69):
        page, slot = table[0][s // P], s % P
        for d in (0, 9, 31):
            assert pool[F8.latent_code_offset(page, slot, d, P, r_kv, d_r)] == cc[s, d]
        for d in (0, 15):
            o = F8.latent_kr16_offset(page, slot, d, P, r_kv, d_r)
            assert int(pool[o]) | (int(pool[o + 1]) << 8) == int(kr[s, d])
    # bytes of slots no token owns keep the fill pattern: 2 * 64 - 70 = 58 empty slots
    assert int((pool == 0x55).sum()) >= 58 * (r_kv + 2 * d_r) - 58 * 4   # (a few data bytes may equal the pattern)


def test_absorb_decode_on_a_dequantised_latent_is_the_plain_decode_on_those_values():
    """The 8-bit latent decode is defined as the MQA-absorb equation on c' = value(code) * scale.  Two consequences that
    do not depend on the decode routine's inner workings: the scale can be pulled out of both uses of c' (logits
    linear in c', output linear in c'), and with codes that represent the latent exactly the result is the 16-bit one."""
    from oracle import gqla_oracle as O
    rng = np.random.default_rng(11)
    h_q, g, d_h, r_kv, d_r, L = 4, 2, 8, 16, 8, 40
    w_uk = rng.normal(size=(g, r_kv, d_h)); w_uv = rng.normal(size=(g, r_kv, d_h))
    q_c = rng.normal(size=(1, h_q, d_h)); q_r = rng.normal(size=(1, h_q, d_r))
    kR = rng.normal(size=(L, d_r))
    # latents that E4M3 holds exactly at scale 0.25: multiples of 0.25 * 2^-3 in [-1, 1] ... take code values directly
    codes = rng.integers(0x20, 0x48, size=(L, r_kv)).astype(np.uint8) | (rng.integers(0, 2, size=(L, r_kv)).astype(np.uint8) << 7)
    scale = 0.25
    c = F8.dequantize_e4m3(codes) * scale
    assert np.array_equal(F8.quantize_tensor(c.astype(np.float32), scale), codes)          # exact round trip
    q_hat = O.absorb_query(q_c, w_uk)
    o1, l1 = O.decode_absorb(q_hat, q_r, c, kR, w_uv)
    # scale pulled out by hand: logits with (scale * q_hat) on unscaled values, output scaled afterwards
    o2, l2 = O.decode_absorb(q_hat * scale, q_r, F8.dequantize_e4m3(codes), kR, w_uv)
    assert np.allclose(o1, o2 * scale, rtol=1e-12, atol=1e-12) and np.allclose(l1, l2, rtol=1e-12, atol=1e-12)
