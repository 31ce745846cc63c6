"""Integer bookkeeping of the GQLA caches, written out independently of the library.
TEST INFRASTRUCTURE ONLY (same rule as gqla_oracle.py: tests, smoke and the benchmark's
CPU-baseline leg may import it; the product path may not).

The paper does not model paging (Sec. 5.1 "Limitations", item (i)); what is fixed by it are the
per-token element counts of the two caches (Sec. 4.2.1 and 4.2.2: r_kv + d_R and 2 g d_h + d_R).
The page formats below are this library's documented formats; the functions here restate the
documentation, element by element, so that the library's own address arithmetic can be checked
against a second implementation.

Latent page  (P tokens):   row-major  [P][r_kv + d_R]  =  c_kv | k_R   per token.
Expanded page (P tokens, g_c groups), three planes of 8-element vectors:
    K_C : [g_c][d_h/8][P][8]     8 consecutive dims of one token are contiguous
    V   : [g_c][P/8][d_v][8]     8 consecutive tokens of one dim are contiguous
    k_R : [d_R/8][P][8]
d_v is the per-head value dim (d_h^V of Sec. 3.2.2); it defaults to d_h, and a token then takes the 2 g d_h + d_R
elements of Sec. 4.2.2, otherwise g (d_h + d_v) + d_R.
"""
from __future__ import annotations

import numpy as np


# ---- sizes (Sec. 4.2.1, 4.2.2) ---------------------------------------------------------
def latent_elems_per_token(r_kv, d_r):
    return r_kv + d_r


def expanded_elems_per_token(g, d_h, d_r, d_v=None):
    return g * (d_h + (d_h if d_v is None else d_v)) + d_r


def pages_needed(L, P):
    return -(-int(L) // P)


# ---- logical token -> physical slot ----------------------------------------------------
def phys_token(page_row, t, P):
    """(page id, slot) of logical token t of a sequence whose page-table row is page_row."""
    return int(page_row[t // P]), t % P


def contiguous_page(b, p, max_pages):
    """Page id used when no page table is given: sequence b owns pages b*max_pages ..."""
    return b * max_pages + p


# ---- element offsets inside the pools ---------------------------------------------------
def latent_offset(page, slot, col, P, r_kv, d_r):
    """col in [0, r_kv) addresses c_kv, col in [r_kv, r_kv + d_r) addresses k_R."""
    return (page * P + slot) * (r_kv + d_r) + col


def expanded_page_elems(P, g_c, d_h, d_r, d_v=None):
    return P * expanded_elems_per_token(g_c, d_h, d_r, d_v)


def expanded_k_offset(page, j, slot, d, P, g_c, d_h, d_r, d_v=None):
    base = page * expanded_page_elems(P, g_c, d_h, d_r, d_v)
    return base + ((j * (d_h // 8) + d // 8) * P + slot) * 8 + d % 8


def expanded_v_offset(page, j, slot, d, P, g_c, d_h, d_r, d_v=None):
    """d in [0, d_v)."""
    dv = d_h if d_v is None else d_v
    base = page * expanded_page_elems(P, g_c, d_h, d_r, d_v) + g_c * P * d_h
    return base + ((j * (P // 8) + slot // 8) * dv + d) * 8 + slot % 8


def expanded_kr_offset(page, slot, d, P, g_c, d_h, d_r, d_v=None):
    dv = d_h if d_v is None else d_v
    base = page * expanded_page_elems(P, g_c, d_h, d_r, d_v) + g_c * P * (d_h + dv)
    return base + ((d // 8) * P + slot) * 8 + d % 8


# ---- whole-pool packers (vectorised restatements of the offsets above) ---------------------
def pack_latent_pool(seq_rows, table, num_pages, P, width, fill=np.nan):
    """seq_rows[b] = [L_b, width] array.  Returns pool [num_pages, P, width]; unused slots = fill."""
    pool = np.full((num_pages, P, width), fill, dtype=np.float32)
    for b, rows in enumerate(seq_rows):
        L = rows.shape[0]
        t = np.arange(L)
        pool[table[b][t // P], t % P] = rows
    return pool


def pack_expanded_pool(KC_seqs, V_seqs, kR_seqs, table, num_pages, P, fill=np.nan):
    """KC_seqs[b] = [L_b, g_c, d_h], V_seqs[b] = [L_b, g_c, d_v]; kR_seqs[b] = [L_b, d_r].
    Returns a flat fp32 pool of num_pages * expanded_page_elems elements; unused slots = fill."""
    L0, g_c, d_h = KC_seqs[0].shape
    d_v = V_seqs[0].shape[2]
    d_r = kR_seqs[0].shape[1]
    pe = expanded_page_elems(P, g_c, d_h, d_r, d_v)
    pool = np.full((num_pages * pe,), fill, dtype=np.float32)
    for b in range(len(KC_seqs)):
        L = KC_seqs[b].shape[0]
        t = np.arange(L)
        page = np.asarray(table[b])[t // P].astype(np.int64)
        slot = (t % P).astype(np.int64)
        base = page * pe
        d = np.arange(d_h, dtype=np.int64)
        e = np.arange(d_v, dtype=np.int64)
        for j in range(g_c):
            ko = base[:, None] + ((j * (d_h // 8) + d[None, :] // 8) * P + slot[:, None]) * 8 + d[None, :] % 8
            pool[ko] = KC_seqs[b][:, j, :]
            vo = (base[:, None] + g_c * P * d_h
                  + ((j * (P // 8) + slot[:, None] // 8) * d_v + e[None, :]) * 8 + slot[:, None] % 8)
            pool[vo] = V_seqs[b][:, j, :]
        dr = np.arange(d_r, dtype=np.int64)
        ro = base[:, None] + g_c * P * (d_h + d_v) + ((dr[None, :] // 8) * P + slot[:, None]) * 8 + dr[None, :] % 8
        pool[ro] = kR_seqs[b]
    return pool


def unpack_expanded_seq(pool, page_row, L, P, g_c, d_h, d_r, d_v=None):
    """Inverse of pack_expanded_pool for one sequence: (KC [L,g_c,d_h], V [L,g_c,d_v], kR [L,d_r])."""
    d_v = d_h if d_v is None else d_v
    pe = expanded_page_elems(P, g_c, d_h, d_r, d_v)
    t = np.arange(int(L))
    page = np.asarray(page_row)[t // P].astype(np.int64)
    slot = (t % P).astype(np.int64)
    base = page * pe
    d = np.arange(d_h, dtype=np.int64)
    e = np.arange(d_v, dtype=np.int64)
    KC = np.empty((int(L), g_c, d_h), pool.dtype)
    V = np.empty((int(L), g_c, d_v), pool.dtype)
    for j in range(g_c):
        KC[:, j, :] = pool[base[:, None] + ((j * (d_h // 8) + d[None, :] // 8) * P + slot[:, None]) * 8 + d[None, :] % 8]
        V[:, j, :] = pool[base[:, None] + g_c * P * d_h
                          + ((j * (P // 8) + slot[:, None] // 8) * d_v + e[None, :]) * 8 + slot[:, None] % 8]
    dr = np.arange(d_r, dtype=np.int64)
    kR = pool[base[:, None] + g_c * P * (d_h + d_v) + ((dr[None, :] // 8) * P + slot[:, None]) * 8 + dr[None, :] % 8]
    return KC, V, kR


# ---- split plan ---------------------------------------------------------------------------
PATH_ABSORB = 0
PATH_GQA = 1


def gqa_token_team(h_q, g, s_q):
    """GQA path with one group of at most 32 query rows: the eight waves of a workgroup share one chunk."""
    return g == 1 and h_q * s_q <= 32


def plan_slots(num_cus, path, h_q, g, s_q):
    """How many chunks the device works on at once under the documented launch shapes:
    absorb  one 4-wave workgroup per CU covers 128 query rows  -> num_cus / ceil(h_q*s_q / 128)
    gqa     8 waves per CU, one wave per (chunk, group, 32-row block) -> num_cus*8 / (g * ceil(G*s_q / 32)),
            or one workgroup per chunk -> num_cus with a token team"""
    if path == PATH_ABSORB:
        rb = -(-(h_q * s_q) // 128)
        return max(1, num_cus // rb)
    if gqa_token_team(h_q, g, s_q):
        return max(1, num_cus)
    rb = -(-((h_q // g) * s_q) // 32)
    return max(1, (num_cus * 8) // (g * rb))


def plan_overhead_pages(path, h_q=0, g=0, s_q=0):
    if path == PATH_ABSORB:
        return 4
    return 16 if gqa_token_team(h_q, g, s_q) else 2


def plan_merge_cost(path):
    """Eightieths of a page time that each chunk partial of the longest sequence adds to the combine."""
    return 16 if path == PATH_ABSORB else 5


def plan_page_weight(path, n_chunks, num_cus, h_q, s_q, g=0):
    """Eightieths of the reference page time that one page costs a workgroup: 80, or 53 on the absorb path when the
    launch gives every 32 query rows a workgroup of their own -- at most 32 rows per sequence, or so few chunks
    (counted in eights) that one workgroup per chunk and 32 rows still fits the device in one round; 10 on the GQA
    path with a token team (eight waves share the chunk's pages)."""
    if path != PATH_ABSORB:
        return 10 if gqa_token_team(h_q, g, s_q) else 80
    M = h_q * s_q
    padded = -(-n_chunks // 8) * 8
    return 53 if (M <= 32 or padded * (-(-M // 32)) <= num_cus) else 80


def plan_chunk_pages(lens, P, num_cus, path, h_q, g, s_q):
    """Chunk size (in pages): the cp in 1..max_b npages_b minimising
    weight(cp) * ceil(n_chunks(cp) / slots) * (cp + overhead) + merge * ceil(max_b npages_b / cp),
    n_chunks(cp) = sum_b ceil(npages_b / cp); ties go to the larger cp."""
    npages = [pages_needed(L, P) for L in lens]
    slots = plan_slots(num_cus, path, h_q, g, s_q)
    ovh = plan_overhead_pages(path, h_q, g, s_q)
    longest = max(npages)
    best_cp, best_cost = 1, None
    for cp in range(1, longest + 1):
        n_chunks = sum(-(-n // cp) for n in npages)
        rounds = -(-n_chunks // slots)
        cost = (plan_page_weight(path, n_chunks, num_cus, h_q, s_q, g) * rounds * (cp + ovh)
                + plan_merge_cost(path) * (-(-longest // cp)))
        if best_cost is None or cost <= best_cost:
            best_cp, best_cost = cp, cost
    return best_cp


def plan_chunks(lens, P, chunk_pages):
    """Chunk list in slot order (sequence-major).  Sequence b is cut into n_b = ceil(npages_b / chunk_pages)
    chunks of ceil(npages_b / n_b) pages (the last one shorter); a chunk is (b, tok_begin, tok_end)
    with tok_end clipped to L_b.  Also returns first_slot[b]."""
    chunks, first = [], []
    for b, L in enumerate(lens):
        L = int(L)
        n_pages = pages_needed(L, P)
        n_b = -(-n_pages // chunk_pages)
        per = -(-n_pages // n_b)
        first.append(len(chunks))
        k = 0
        while k * per < n_pages:
            lo = k * per * P
            hi = min((k + 1) * per * P, L)
            chunks.append((b, lo, hi))
            k += 1
    return chunks, first
