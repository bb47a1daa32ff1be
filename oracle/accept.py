"""Step 4 of the method in its speculative-sampling form (Sec. 3.1, Eq. 1 and
Eq. 3).  Test infrastructure.

Target distribution: the target model is sampled at temperature 1 with no
top-k / top-p truncation (supplement, "Sampling"), so p_i = softmax(z_i) over
the whole codebook.

Accept test: draft token x~_i is kept with probability
min(1, pbar_i / q_i(x~_i)), where pbar_i = sum of p_i over the k nearest
codebook entries of x~_i (Eq. 3); k = 1 gives Eq. 1.  With a uniform u in
[0, 1) that is "accept iff u * q < pbar", the division-free form of
"u < min(1, pbar/q)"; it is also defined at q = 0 (accept iff pbar > 0) and,
because u <= 1 - 2^-24, accepts every position when q and p hold the same
bits.  The three quantities are float32 and the product is rounded to float32
before the comparison (the precision the decision is taken in).

Threshold form (Sec. 3.3, Eq. 5; the rule the paper itself runs): the draft
token is kept iff its pooled target mass reaches a threshold,
pbar_i >= tau, with no draft probability and no random number.  Eq. 5 writes
">=" and the listing of Alg. 1 writes ">"; the equation is taken (the two
differ only when pbar equals tau bit for bit).  pbar and tau are float32.
"""
import numpy as np

from .upsample import softmax_rows

NEAR_TIE = 1e-4


def guided_logits(z_cond, z_uncond, scale):
    """Classifier-free guidance (supplement, "Sampling": scale 4.0, empty negative prompt).  The paper names
    the technique and the scale, not the formula; the standard one is taken:
    z = z_u + s (z_c - z_u), in float64 (s = 1 gives the conditional logits, s = 0 the unconditional)."""
    zc = np.asarray(z_cond, dtype=np.float64)
    zu = np.asarray(z_uncond, dtype=np.float64)
    return zu + float(scale) * (zc - zu)


def target_probs(logits):
    """p = softmax(logits) over the last axis: float64 inside, rounded once to float32."""
    return softmax_rows(logits).astype(np.float32)


def pooled_mass(p, tokens, nbr=None):
    """pbar[..] = sum_m p[.., nbr[token, m]]  (Eq. 3 numerator); nbr None => p[.., token].

    p: float32 [..., V]; tokens: int [...]; nbr: int [V, k] with nbr[x, 0] == x.
    Summed in float64, rounded to float32.
    """
    p = np.asarray(p, dtype=np.float32)
    tok = np.asarray(tokens).astype(np.int64)
    if nbr is None:
        return np.take_along_axis(p, tok[..., None], axis=-1)[..., 0]
    cols = np.asarray(nbr)[tok]                       # [..., k]
    vals = np.take_along_axis(p, cols.astype(np.int64), axis=-1).astype(np.float64)
    return vals.sum(axis=-1).astype(np.float32)


def accept_test(pbar, q_tok, u):
    """accept iff fl32(u * q) < pbar; all float32 (Eq. 1 / Eq. 3)."""
    pbar = np.asarray(pbar, dtype=np.float32)
    q_tok = np.asarray(q_tok, dtype=np.float32)
    u = np.asarray(u, dtype=np.float32)
    return (u * q_tok).astype(np.float32) < pbar


def near_tie(pbar, q_tok, u, width=NEAR_TIE):
    """|pbar/q - u| < width, written without the division: |pbar - u q| < width q."""
    pbar = np.asarray(pbar, dtype=np.float64)
    q_tok = np.asarray(q_tok, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    return np.abs(pbar - u * q_tok) < width * q_tok


def accept_test_tau(pbar, tau):
    """accept iff pbar >= tau, both float32 (Eq. 5)."""
    return np.asarray(pbar, dtype=np.float32) >= np.float32(tau)


def near_tie_tau(pbar, tau, width=NEAR_TIE):
    """|pbar - tau| < width * tau: decisions that a last-ulp difference in pbar could flip."""
    return np.abs(np.asarray(pbar, dtype=np.float64) - float(np.float32(tau))) < width * float(np.float32(tau))
