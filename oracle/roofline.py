"""The paper's analytical Roofline accounting (Sec. 4), as plain arithmetic.
TEST / MEASUREMENT INFRASTRUCTURE: used by tests and by the benchmark's reporting only."""
from __future__ import annotations


def ridge(peak_flops, bw):
    """Sec. 4.1: I* = FLOPs_max / BW."""
    return peak_flops / bw


# ---- MQA-absorb path (Sec. 4.2.1) -------------------------------------------------------
def absorb_bytes_per_token(r_kv, d_r, elem_bytes=2):
    return elem_bytes * (r_kv + d_r)


def absorb_bytes(L, r_kv, d_r, elem_bytes=2):
    return L * absorb_bytes_per_token(r_kv, d_r, elem_bytes)


def absorb_flops(L, h_q, s_q, r_kv, d_r):
    return 2 * L * h_q * s_q * (2 * r_kv + d_r)


def absorb_intensity(h_q, s_q, r_kv, d_r):
    return h_q * s_q * (2 * r_kv + d_r) / (r_kv + d_r)


# ---- GQA path (Sec. 4.2.2) ----------------------------------------------------------------
def gqa_bytes_per_token(g, d_h, d_r, elem_bytes=2):
    return elem_bytes * (2 * g * d_h + d_r)


def gqa_bytes(L, g, d_h, d_r, elem_bytes=2):
    return L * gqa_bytes_per_token(g, d_h, d_r, elem_bytes)


def gqa_flops(L, h_q, s_q, d_h, d_r):
    return 2 * L * h_q * s_q * (2 * d_h + d_r)


def gqa_intensity(h_q, g, s_q, d_h, d_r):
    return h_q * s_q * (2 * d_h + d_r) / (2 * g * d_h + d_r)


# ---- operating point (Sec. 4.2.3, Table 2) --------------------------------------------------
def operating_point(nbytes, flops, s_q, peak_flops, bw):
    """time = max(F / peak, B / BW); throughput = s_q / time."""
    mem = nbytes / bw
    cmp_ = flops / peak_flops
    step = max(mem, cmp_)
    return {"mem_s": mem, "cmp_s": cmp_, "step_s": step, "tok_per_s": s_q / step}
