"""Residual resampling of the marked positions (Sec. 3.1, Eq. 2).
Test infrastructure.

A marked position u draws its token from p'_u = norm(max(0, p_u - q_u)).
To make the draw independent of floating-point summation order the weights are
turned into integers first:
    w(x)     = max(0, fl32(p_u(x) - q_u(x)))          float32 subtraction
    W(x)     = floor(w(x) * 2^40)                      exact for float32 w
    tot      = sum_x W(x)                              integer, order-free
    (tot == 0: fall back to w = p_u)
    T        = (word * tot) >> 32                      word = raw 32-bit Philox output
    token    = smallest x with sum_{x' <= x} W(x') > T
so token x is drawn for W(x)/tot of the 2^32 words up to rounding by one word.

mode 0 (default): every marked position draws from the residual.
mode 1: positions that were themselves rejected draw from the residual, the
        neighbours marked only by expansion draw from p_u (the paper re-samples
        expanded positions from the target model, Sec. 3.3 after Eq. 7).
mode 2: every marked position draws from p_u: the paper's own Step 6 (Alg. 1),
        which samples rejected tokens from the target model; no draft
        distribution is needed.
"""
import numpy as np

SCALE_BITS = 40


def integer_weights(w32):
    """floor(w * 2^40) as uint64 for float32 w in [0, 1]."""
    w32 = np.asarray(w32, dtype=np.float32)
    return np.floor(w32.astype(np.float64) * float(1 << SCALE_BITS)).astype(np.uint64)


def residual_weights(p_row, q_row):
    """Integer residual weights of one position; falls back to p when the residual is empty."""
    p_row = np.asarray(p_row, dtype=np.float32)
    q_row = np.asarray(q_row, dtype=np.float32)
    w = np.maximum(np.float32(0), (p_row - q_row).astype(np.float32))
    Wi = integer_weights(w)
    if int(Wi.sum(dtype=np.uint64)) == 0:
        Wi = integer_weights(p_row)
    return Wi


def threshold(word, tot):
    """T = (word * tot) >> 32 with python integers (no overflow)."""
    return (int(word) * int(tot)) >> 32


def draw(Wi, word):
    """Smallest x whose inclusive prefix sum of Wi exceeds T."""
    cdf = np.cumsum(Wi, dtype=np.uint64)
    tot = int(cdf[-1])
    T = threshold(word, tot)
    return int(np.searchsorted(cdf, np.uint64(T), side="right"))


def boundary_distance(Wi, word):
    """min |T - boundary| / tot over the two CDF boundaries that bracket T; used
    to list draws that a last-ulp difference in p could move."""
    cdf = np.cumsum(Wi, dtype=np.uint64)
    tot = int(cdf[-1])
    T = threshold(word, tot)
    x = int(np.searchsorted(cdf, np.uint64(T), side="right"))
    lo = int(cdf[x - 1]) if x > 0 else 0
    hi = int(cdf[x])
    d = min(T - lo, hi - T) if x > 0 else hi - T
    return d / tot


def resample_block(p, q_rows, q_row_index, draft_tokens, mask, accept, words, mode=0):
    """p: float32 [L, V]; q_rows: float32 [n_q, V]; q_row_index: int [L] (row of
    q_rows that belongs to position u); mask/accept: [L]; words: uint32 [L].
    Returns tokens_out int32 [L]."""
    L = p.shape[0]
    out = np.asarray(draft_tokens).astype(np.int32).copy()
    for u in range(L):
        if not mask[u]:
            continue
        if mode == 2 or (mode == 1 and accept[u]):
            Wi = integer_weights(p[u])
        else:
            Wi = residual_weights(p[u], q_rows[q_row_index[u]])
        out[u] = draw(Wi, words[u])
    return out
