"""CPU oracle for GQLA decode attention (fp64, numpy).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
file; the product path never does.  It shares no code with the HIP kernels.

Every function is the paper's definition written out, in the paper's notation
(Sec. 3.1: "GQA path" and "MQA-absorb path" equations), 0-based:

  h_q query heads, g KV groups, G = h_q / g heads per group, head i -> group j(i) = i // G
  (the paper's 1-based ceil(i / (h_q/g)); "repeat" is group-wise replication, i.e. heads
  j*G .. j*G+G-1 share group j's up-projection slice),
  c[s]  in R^{r_kv}   latent of cached token s,      kR[s] in R^{d_R}  shared RoPE key,
  qC[t,i] in R^{d_h}, qR[t,i] in R^{d_R}             queries of step token t, head i,
  W_UK[j], W_UV[j] in R^{r_kv x d_h}                 stored transposed w.r.t. the paper's
                                                     d_h x r_kv head slice,
  sigma = 1 / sqrt(d_h + d_R)                        softmax scale of both paths.

Reading for s_q > 1 (the paper leaves the in-step mask open): the L cached rows include
the s_q step tokens as their last rows; query t sits at position L - s_q + t and sees
s <= L - s_q + t.

All array arguments are per sequence.  Nothing is rounded here.
"""
from __future__ import annotations

import math
import numpy as np

F64 = np.float64


def head_group(i: int, h_q: int, g: int) -> int:
    """Sec. 3.1, routing rule of the GQA path: j(i), 0-based."""
    if h_q % g:
        raise ValueError("g must divide h_q")
    return i // (h_q // g)


def softmax_scale(d_h: int, d_r: int) -> float:
    """Sec. 3.1: both paths divide the logits by sqrt(d_h + d_h^R)."""
    return 1.0 / math.sqrt(d_h + d_r)


def n_visible(L: int, s_q: int, t: int) -> int:
    """Number of cached rows query t may attend to (rows 0 .. L - s_q + t)."""
    return L - s_q + t + 1


# ----------------------------------------------------------------------------------------
# cache switch  (Sec. 3.1, "Two equivalent decoding paths": one-shot expand)
# ----------------------------------------------------------------------------------------
def expand_latent(c, W_UK, W_UV):
    """k^C_s = W^UK c_s and v^C_s = W^UV c_s for every cached token (Sec. 3.1, Eq. (1) and
    first line of the GQA-path equation).  c [L, r_kv]; W_UK [g, r_kv, d_h], W_UV [g, r_kv, d_v] -> KC [L, g, d_h],
    V [L, g, d_v] (the value dim may differ from the key dim: d_h^V of Sec. 3.2.2)."""
    c = np.asarray(c, F64)
    W_UK = np.asarray(W_UK, F64)
    W_UV = np.asarray(W_UV, F64)
    L = c.shape[0]
    g, r_kv, d_h = W_UK.shape
    d_v = W_UV.shape[2]
    KC = np.empty((L, g, d_h), F64)
    V = np.empty((L, g, d_v), F64)
    for j in range(g):
        KC[:, j, :] = c @ W_UK[j]          # (W_UK[j]^T c_s) for all s
        V[:, j, :] = c @ W_UV[j]
    return KC, V


def left_inverse_uk(W_UK):
    """The matrix that undoes the key half of the expansion (Sec. 3.1: the cache switch between the two paths is a
    one-shot "compress/expand"; compression exists when the stacked key up-projection has full column rank, which
    needs g d_h >= r_kv).  With A = [W_UK[0]^T; ...; W_UK[g-1]^T] in R^{g d_h x r_kv} (so that k^C = A c), the left
    inverse is A^+ = (A^T A)^{-1} A^T in R^{r_kv x g d_h}; columns are ordered group-major, dim-minor like k^C."""
    W_UK = np.asarray(W_UK, F64)
    g, r_kv, d_h = W_UK.shape
    A = np.concatenate([W_UK[j].T for j in range(g)], axis=0)       # [g d_h, r_kv]
    return np.linalg.solve(A.T @ A, A.T)


def compress_expanded(KC, W_UK):
    """c_s = A^+ k^C_s for every cached token: KC [L, g, d_h] -> c [L, r_kv].  On exact expansions this returns the
    latent exactly; on rounded ones it is the least-squares latent."""
    KC = np.asarray(KC, F64)
    L = KC.shape[0]
    return KC.reshape(L, -1) @ left_inverse_uk(W_UK).T


# ----------------------------------------------------------------------------------------
# softmax over the visible rows, with its log-sum-exp
# ----------------------------------------------------------------------------------------
def _softmax_lse(z):
    m = np.max(z)
    e = np.exp(z - m)
    ssum = np.sum(e)
    return e / ssum, m + math.log(ssum)


# ----------------------------------------------------------------------------------------
# GQA path (Sec. 3.1, GQA-path equation)
# ----------------------------------------------------------------------------------------
def decode_gqa(qC, qR, KC, V, kR, scale=None):
    """o[t,i] = sum_s softmax_s( (qC[t,i].KC[s,j(i)] + qR[t,i].kR[s]) * sigma ) V[s,j(i)].

    qC [s_q,h_q,d_h], qR [s_q,h_q,d_R], KC [L,g,d_h], V [L,g,d_v], kR [L,d_R] -> o [s_q,h_q,d_v], lse [s_q,h_q]."""
    qC, qR, KC, V, kR = (np.asarray(a, F64) for a in (qC, qR, KC, V, kR))
    s_q, h_q, d_h = qC.shape
    L, g, _ = KC.shape
    d_r = qR.shape[2]
    sigma = softmax_scale(d_h, d_r) if scale is None else float(scale)
    o = np.empty((s_q, h_q, V.shape[2]), F64)
    lse = np.empty((s_q, h_q), F64)
    for t in range(s_q):
        nv = n_visible(L, s_q, t)
        if nv < 1:
            raise ValueError("empty visible set")
        for i in range(h_q):
            j = head_group(i, h_q, g)
            z = (KC[:nv, j, :] @ qC[t, i] + kR[:nv] @ qR[t, i]) * sigma
            p, lse[t, i] = _softmax_lse(z)
            o[t, i] = p @ V[:nv, j, :]
    return o, lse


# ----------------------------------------------------------------------------------------
# MQA-absorb path (Sec. 3.1, MQA-absorb equation)
# ----------------------------------------------------------------------------------------
def absorb_query(qC, W_UK):
    """q_hat[t,i] = (W-hat^UK_i)^T qC[t,i]; with W_UK[j] stored [r_kv, d_h] that is W_UK[j(i)] @ qC[t,i]."""
    qC = np.asarray(qC, F64)
    W_UK = np.asarray(W_UK, F64)
    s_q, h_q, d_h = qC.shape
    g, r_kv, _ = W_UK.shape
    q_hat = np.empty((s_q, h_q, r_kv), F64)
    for t in range(s_q):
        for i in range(h_q):
            q_hat[t, i] = W_UK[head_group(i, h_q, g)] @ qC[t, i]
    return q_hat


def decode_absorb_latent(q_hat, qR, c, kR, d_h, scale=None):
    """o_hat[t,i] = sum_s softmax_s( (q_hat[t,i].c[s] + qR[t,i].kR[s]) * sigma ) c[s]   (latent space)."""
    q_hat, qR, c, kR = (np.asarray(a, F64) for a in (q_hat, qR, c, kR))
    s_q, h_q, r_kv = q_hat.shape
    L = c.shape[0]
    d_r = qR.shape[2]
    sigma = softmax_scale(d_h, d_r) if scale is None else float(scale)
    o_hat = np.empty((s_q, h_q, r_kv), F64)
    lse = np.empty((s_q, h_q), F64)
    for t in range(s_q):
        nv = n_visible(L, s_q, t)
        if nv < 1:
            raise ValueError("empty visible set")
        for i in range(h_q):
            z = (c[:nv] @ q_hat[t, i] + kR[:nv] @ qR[t, i]) * sigma
            p, lse[t, i] = _softmax_lse(z)
            o_hat[t, i] = p @ c[:nv]
    return o_hat, lse


def project_latent_output(o_hat, W_UV):
    """o[t,i] = W-hat^UV_i o_hat[t,i]; with W_UV[j] stored [r_kv, d_h] that is W_UV[j(i)]^T o_hat[t,i]."""
    o_hat = np.asarray(o_hat, F64)
    W_UV = np.asarray(W_UV, F64)
    s_q, h_q, r_kv = o_hat.shape
    g, _, d_h = W_UV.shape
    o = np.empty((s_q, h_q, d_h), F64)
    for t in range(s_q):
        for i in range(h_q):
            o[t, i] = o_hat[t, i] @ W_UV[head_group(i, h_q, g)]
    return o


def decode_absorb(q_hat, qR, c, kR, W_UV, scale=None, d_h=None):
    """The whole MQA-absorb decode after query absorption: latent attention, then W^UV.  d_h is the key dim that
    enters the softmax scale; it defaults to W^UV's column count, i.e. to equal key and value dims."""
    if d_h is None:
        d_h = np.asarray(W_UV).shape[2]
    o_hat, lse = decode_absorb_latent(q_hat, qR, c, kR, d_h, scale)
    return project_latent_output(o_hat, W_UV), lse


# ----------------------------------------------------------------------------------------
# brute force: h_q fully materialised heads, textbook attention, python loops (tiny inputs)
# ----------------------------------------------------------------------------------------
def decode_mha_bruteforce(qC, qR, c, kR, W_UK, W_UV, scale=None):
    """Builds k_{s,i} = [k^C_{s,j(i)}; k^R_s] and v_{s,i} = v^C_{s,j(i)} element by element for
    every head (second line of the GQA-path equation) and evaluates the attention sum with
    scalar loops.  No matmul, no shared helper: an independent second opinion."""
    s_q, h_q, d_h = np.shape(qC)
    d_r = np.shape(qR)[2]
    L, r_kv = np.shape(c)
    g = np.shape(W_UK)[0]
    d_v = np.shape(W_UV)[2]
    G = h_q // g
    sigma = 1.0 / math.sqrt(d_h + d_r) if scale is None else float(scale)
    o = np.zeros((s_q, h_q, d_v), F64)
    for i in range(h_q):
        j = i // G
        K_i = [[0.0] * (d_h + d_r) for _ in range(L)]
        V_i = [[0.0] * d_v for _ in range(L)]
        for s in range(L):
            for d in range(d_h):
                ak = 0.0
                for r in range(r_kv):
                    ak += float(W_UK[j][r][d]) * float(c[s][r])
                K_i[s][d] = ak
            for d in range(d_v):
                av = 0.0
                for r in range(r_kv):
                    av += float(W_UV[j][r][d]) * float(c[s][r])
                V_i[s][d] = av
            for d in range(d_r):
                K_i[s][d_h + d] = float(kR[s][d])
        for t in range(s_q):
            q = [float(x) for x in qC[t][i]] + [float(x) for x in qR[t][i]]
            last = L - s_q + t                     # position of query t
            logits = []
            for s in range(last + 1):
                acc = 0.0
                for d in range(d_h + d_r):
                    acc += q[d] * K_i[s][d]
                logits.append(acc * sigma)
            mx = max(logits)
            w = [math.exp(x - mx) for x in logits]
            den = sum(w)
            for d in range(d_v):
                acc = 0.0
                for s in range(last + 1):
                    acc += w[s] * V_i[s][d]
                o[t, i, d] = acc / den
    return o


# ----------------------------------------------------------------------------------------
# split-L partials and their log-sum-exp combine
# ----------------------------------------------------------------------------------------
def partial_attention(z_row, values, lo, hi, nv):
    """Attention of one query row restricted to cached rows [lo, min(hi, nv)): returns the
    locally normalised output and the local log-sum-exp (-inf and zeros when the range is empty)."""
    hi = min(hi, nv)
    if hi <= lo:
        return np.zeros(values.shape[1], F64), -math.inf
    p, lse = _softmax_lse(z_row[lo:hi])
    return p @ values[lo:hi], lse


def combine_partials(o_k, lse_k):
    """lse = log sum_k exp(lse_k);  o = sum_k exp(lse_k - lse) o_k.   o_k [n, d], lse_k [n]."""
    o_k = np.asarray(o_k, F64)
    lse_k = np.asarray(lse_k, F64)
    m = np.max(lse_k)
    if m == -math.inf:
        raise ValueError("all partials empty")
    w = np.exp(lse_k - m)
    lse = m + math.log(np.sum(w))
    return (np.exp(lse_k - lse)[:, None] * o_k).sum(axis=0), lse


def decode_gqa_split(qC, qR, KC, V, kR, bounds, scale=None):
    """decode_gqa evaluated chunk by chunk (bounds = [(lo, hi), ...] covering [0, L)) and combined."""
    qC, qR, KC, V, kR = (np.asarray(a, F64) for a in (qC, qR, KC, V, kR))
    s_q, h_q, d_h = qC.shape
    L, g, _ = KC.shape
    sigma = softmax_scale(d_h, qR.shape[2]) if scale is None else float(scale)
    o = np.empty((s_q, h_q, d_h), F64)
    lse = np.empty((s_q, h_q), F64)
    for t in range(s_q):
        nv = n_visible(L, s_q, t)
        for i in range(h_q):
            j = head_group(i, h_q, g)
            z = (KC[:, j, :] @ qC[t, i] + kR @ qR[t, i]) * sigma
            parts = [partial_attention(z, V[:, j, :], lo, hi, nv) for lo, hi in bounds]
            o[t, i], lse[t, i] = combine_partials([p[0] for p in parts], [p[1] for p in parts])
    return o, lse


# ----------------------------------------------------------------------------------------
# whole-batch drivers over a paged pool (gather rows through the page table, then the above)
# ----------------------------------------------------------------------------------------
def gather_rows(pool_rows, page_row, L_b, page_size):
    """Logical rows 0..L_b-1 of one sequence out of a [num_pages, page_size, width] pool:
    row t lives in page page_row[t // page_size] at slot t % page_size."""
    t = np.arange(int(L_b))
    return pool_rows[np.asarray(page_row)[t // page_size], t % page_size]


# ----------------------------------------------------------------------------------------
# the steps either side of the path: decoupled RoPE (Sec. 3.1, "Architecture") and W^O (last
# line of both path equations)
# ----------------------------------------------------------------------------------------
def rope(x, t, base=10000.0):
    """rope_t(x) of Sec. 3.1 ("Architecture": q^R and k^R carry the position).  The paper takes the rotary
    embedding over from MLA without restating it; the reading here is the rotary embedding as published:
    the vector is d/2 adjacent pairs (x[2p], x[2p+1]) and pair p turns by the angle t * base^(-2p/d).
    x [..., d] (d even), t an integer position (scalar or broadcastable to x[..., 0])."""
    x = np.asarray(x, F64)
    d = x.shape[-1]
    if d % 2:
        raise ValueError("rope needs an even dimension")
    p = np.arange(d // 2, dtype=F64)
    theta = float(base) ** (-2.0 * p / d)                    # one frequency per pair
    ang = np.asarray(t, F64)[..., None] * theta              # [..., d/2]
    cos, sin = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[..., 0::2] = x[..., 0::2] * cos - x[..., 1::2] * sin
    out[..., 1::2] = x[..., 0::2] * sin + x[..., 1::2] * cos
    return out


def rope_step(qR_raw, kR_raw, L, base=10000.0):
    """The step's rotated inputs: q^R_{t,i} = rope_t(.) for every head and k^R_t = rope_t(.) of the new tokens
    (Sec. 3.1, "Architecture"), with step token t at position L - s_q + t (L counts the step's own tokens, as in
    n_visible).  qR_raw [s_q, h_q, d_R], kR_raw [s_q, d_R]."""
    qR_raw = np.asarray(qR_raw, F64)
    kR_raw = np.asarray(kR_raw, F64)
    s_q = qR_raw.shape[0]
    pos = L - s_q + np.arange(s_q)
    return rope(qR_raw, pos[:, None], base), rope(kR_raw, pos, base)


def output_projection(o, W_O):
    """y_t = W^O [o_{t,1}; ...; o_{t,h_q}] (last line of the GQA-path and of the MQA-absorb equation).
    o [s_q, h_q, d_h]; W_O [D, h_q * d_h] -> y [s_q, D]."""
    o = np.asarray(o, F64)
    W_O = np.asarray(W_O, F64)
    s_q = o.shape[0]
    return o.reshape(s_q, -1) @ W_O.T
