"""Quantised (8-bit floating point) expanded cache for the GQA path, written out independently of the library.
TEST INFRASTRUCTURE ONLY (same rule as gqla_oracle.py).

The paper names quantised KV caches as complementary to its method and leaves them out of its model
(Sec. 2 "Related work"; Sec. 5.1 "Limitations", item (i)); it fixes neither a format nor scales.  What this build
takes (its own reading, listed in the design notes): K_C and V are stored as E4M3 of the OCP 8-bit floating point
specification ("FN" variant: bias 7, 3 mantissa bits, subnormals, no infinities, the one NaN code S.1111.111,
largest finite value 448), one scale per tensor kind:
    code = E4M3( fp32(x) * fp32(1 / scale) ),  round to nearest, ties to even, saturating at +-448
    x'   = value(code) * scale
and k_R stays in the cache's 16-bit type.  The decode then is the GQA-path equation (Sec. 3.1) on K_C', V'.

Page format (P tokens, g_c groups; byte offsets inside a page of P * (2 g_c d_h + 2 d_R) bytes), every 16-byte vector
holding what one lane of a 32x32x16 matrix instruction consumes in two consecutive k-steps:
    K8 : [g_c][d_h/16][P][16]      dim d = 32 kp + 16 u + 8 h + i  ->  vector 2 kp + h, byte 8 u + i
    V8 : [g_c][P/32][d_h][2][16]   slot s = 32 T + 16 u + 8 h + i  ->  tile T, dim d, half h, byte 8 u + i
    k_R: [d_R/8][P][8] 16-bit elements, after the two planes
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_value(code):
    """Value of one code, from the format's definition (sign, 4-bit exponent with bias 7, 3-bit mantissa)."""
    code = int(code)
    s, e, m = code >> 7, (code >> 3) & 15, code & 7
    if e == 15 and m == 7:
        return float("nan")
    v = (m / 8.0) * 2.0 ** (-6) if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return -v if s else v


E4M3_TABLE = np.array([e4m3_value(c) for c in range(256)], dtype=np.float64)


def dequantize_e4m3(codes):
    return E4M3_TABLE[np.asarray(codes, dtype=np.uint8)]


def quantize_e4m3(x):
    """fp32 values -> codes: round to nearest (ties to the even mantissa), magnitudes above 448 saturate to 448,
    zero keeps its sign.  Written with the spacing of the format: in the binade [2^k, 2^(k+1)) (k >= -6) codes are
    2^(k-3) apart, below 2^-6 they are 2^-9 apart."""
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    assert np.isfinite(x).all()
    a = np.minimum(np.abs(x), E4M3_MAX)
    k = np.floor(np.log2(np.maximum(a, 2.0 ** -6)))          # exponent of the binade (clamped into the subnormal range)
    step = 2.0 ** (k - 3)
    q = np.rint(a / step) * step                              # numpy rounds halves to even
    # q may have carried into the next binade (e.g. 15.5 * step -> 16 * step): still a representable value
    e = np.floor(np.log2(np.maximum(q, 2.0 ** -6)))
    is_sub = q < 2.0 ** -6
    mant = np.where(is_sub, q / 2.0 ** -9, (q / 2.0 ** e - 1.0) * 8.0)
    expo = np.where(is_sub, 0, e + 7)
    code = (expo.astype(np.int64) << 3) | np.rint(mant).astype(np.int64)
    code = code | (np.signbit(x).astype(np.int64) << 7)
    return code.astype(np.uint8)


def inv_scale_f32(scale):
    return np.float32(1.0) / np.float32(scale)


def quantize_tensor(x, scale):
    """Codes of x / scale, with the product taken in fp32 as the format reading above says."""
    x32 = np.asarray(x, dtype=np.float32)
    return quantize_e4m3(x32 * inv_scale_f32(scale))


def fp8_page_bytes(P, g_c, d_h, d_r):
    return P * (2 * g_c * d_h + 2 * d_r)


def k8_offset(page, j, slot, d, P, g_c, d_h, d_r):
    kp, u, h, i = d // 32, (d // 16) % 2, (d // 8) % 2, d % 8
    return page * fp8_page_bytes(P, g_c, d_h, d_r) + ((j * (d_h // 16) + 2 * kp + h) * P + slot) * 16 + 8 * u + i


def v8_offset(page, j, slot, d, P, g_c, d_h, d_r):
    T, u, h, i = slot // 32, (slot // 16) % 2, (slot // 8) % 2, slot % 8
    return (page * fp8_page_bytes(P, g_c, d_h, d_r) + g_c * P * d_h
            + (((j * (P // 32) + T) * d_h + d) * 2 + h) * 16 + 8 * u + i)


def kr16_offset(page, slot, d, P, g_c, d_h, d_r):
    """Byte offset of the 16-bit element d of the token's shared RoPE key."""
    return page * fp8_page_bytes(P, g_c, d_h, d_r) + 2 * g_c * P * d_h + (((d // 8) * P + slot) * 8 + d % 8) * 2


def pack_fp8_pool(KC_codes, V_codes, kR_bits, table, num_pages, P, fill=0xAA):
    """KC_codes[b], V_codes[b] = uint8 [L_b, g_c, d_h]; kR_bits[b] = uint16 [L_b, d_r] (the 16-bit patterns of k_R).
    Returns the pool as uint8 [num_pages * page_bytes]; bytes no token owns = fill."""
    L0, g_c, d_h = KC_codes[0].shape
    d_r = kR_bits[0].shape[1]
    pb = fp8_page_bytes(P, g_c, d_h, d_r)
    pool = np.full((num_pages * pb,), fill, dtype=np.uint8)
    d = np.arange(d_h, dtype=np.int64)
    kp, du, dh, di = d // 32, (d // 16) % 2, (d // 8) % 2, d % 8
    for b in range(len(KC_codes)):
        L = KC_codes[b].shape[0]
        t = np.arange(L, dtype=np.int64)
        page = np.asarray(table[b])[t // P].astype(np.int64)
        slot = t % P
        base = page * pb
        T, su, sh, si = slot // 32, (slot // 16) % 2, (slot // 8) % 2, slot % 8
        for j in range(g_c):
            ko = base[:, None] + ((j * (d_h // 16) + 2 * kp[None, :] + dh[None, :]) * P + slot[:, None]) * 16 + 8 * du[None, :] + di[None, :]
            pool[ko] = KC_codes[b][:, j, :]
            vo = (base[:, None] + g_c * P * d_h
                  + (((j * (P // 32) + T[:, None]) * d_h + d[None, :]) * 2 + sh[:, None]) * 16 + 8 * su[:, None] + si[:, None])
            pool[vo] = V_codes[b][:, j, :]
        dr = np.arange(d_r, dtype=np.int64)
        ro = base[:, None] + 2 * g_c * P * d_h + (((dr[None, :] // 8) * P + slot[:, None]) * 8 + dr[None, :] % 8) * 2
        bits = np.asarray(kR_bits[b], dtype=np.uint16)
        pool[ro] = (bits & 0xFF).astype(np.uint8)
        pool[ro + 1] = (bits >> 8).astype(np.uint8)
    return pool


# ---- 8-bit LATENT cache for the MQA-absorb path -----------------------------------------------------------------------
# Same idea, other cache (the paper's Sec. 4.2.1 cache: r_kv latent elements plus the shared RoPE key per token): c_kv as
# E4M3 codes with one positive scale for the whole cache, k_R left in the 16-bit type.  A token then takes r_kv + 2 d_R
# bytes (640 at the canonical shape, against the 1152 of Sec. 4.2.1).  The decode is the MQA-absorb equation (Sec. 3.1) on
# the dequantised latent c' = value(code) * scale: keys [c'; k_R], values c'.
# Page format (P tokens; byte offsets inside a page of P * (r_kv + 2 d_R) bytes), this build's own reading:
#     codes : [P][r_kv]        one byte per latent element, token rows back to back
#     k_R   : [P][d_R] 16-bit  behind the codes


def latent_fp8_page_bytes(P, r_kv, d_r):
    return P * (r_kv + 2 * d_r)


def latent_code_offset(page, slot, d, P, r_kv, d_r):
    return page * latent_fp8_page_bytes(P, r_kv, d_r) + slot * r_kv + d


def latent_kr16_offset(page, slot, d, P, r_kv, d_r):
    """Byte offset of the 16-bit element d of the token's shared RoPE key."""
    return page * latent_fp8_page_bytes(P, r_kv, d_r) + P * r_kv + (slot * d_r + d) * 2


def pack_latent_fp8_pool(c_codes, kR_bits, table, num_pages, P, fill=0xAA):
    """c_codes[b] = uint8 [L_b, r_kv]; kR_bits[b] = uint16 [L_b, d_r].  Returns the pool as uint8; bytes no token owns = fill."""
    r_kv, d_r = c_codes[0].shape[1], kR_bits[0].shape[1]
    pb = latent_fp8_page_bytes(P, r_kv, d_r)
    pool = np.full((num_pages * pb,), fill, dtype=np.uint8)
    for b in range(len(c_codes)):
        for t in range(c_codes[b].shape[0]):
            page, slot = int(np.asarray(table[b])[t // P]), t % P
            o = page * pb + slot * r_kv
            pool[o: o + r_kv] = c_codes[b][t]
            o = page * pb + P * r_kv + slot * d_r * 2
            bits = np.asarray(kR_bits[b][t], dtype=np.uint16)
            pool[o: o + 2 * d_r: 2] = (bits & 0xFF).astype(np.uint8)
            pool[o + 1: o + 2 * d_r: 2] = (bits >> 8).astype(np.uint8)
    return pool
