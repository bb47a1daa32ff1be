"""Step 2 of the method (Sec. 3.2; Alg. 1 Step 2): bring the low-resolution
draft onto the target grid.  Test infrastructure.

The paper's up-sampler U_r is a trained network or a pixel-space
super-resolution pipeline, neither of which has a closed form; it states only
that the sequence grows by r^2 (Sec. 3.2).  The weight-free reading taken here
is replication (what a pixel-shuffle up-sampler with constant filters does):
every low-resolution cell (I, J) emits its r x r children, and the draft
distribution of a child is its parent's, which is then exactly the marginal law
of the replicated token, so the accept test of Eq. 1 stays valid per position.
"""
import numpy as np


def softmax_rows(logits):
    """softmax over the last axis, float64 inside (max-subtracted)."""
    z = np.asarray(logits, dtype=np.float64)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def parent_rows(h, w, r):
    """q_row[u] for u on the (r*h) x (r*w) target grid, raster order:
    parent(u) = (i_u // r) * w + (j_u // r)."""
    H, W = r * h, r * w
    i = np.arange(H)[:, None]
    j = np.arange(W)[None, :]
    return ((i // r) * w + (j // r)).reshape(H * W).astype(np.int32)


def upsample_draft(draft, draft_tokens, h, w, r, input_is_probs=False, materialise=False):
    """draft: [B, h*w, V] logits (or probabilities); draft_tokens: [B, h*w].

    Returns (tokens_hi int32 [B, H*W], q_lo float32 [B, h*w, V],
             q_row int32 [H*W], q_hi float32 [B, H*W, V] or None).
    q_lo = softmax(draft logits) rounded once to float32 (copied if the input
    already holds probabilities).
    """
    draft = np.asarray(draft)
    B = draft.shape[0]
    assert draft.shape[1] == h * w
    if input_is_probs:
        q_lo = draft.astype(np.float32)
    else:
        q_lo = softmax_rows(draft).astype(np.float32)
    q_row = parent_rows(h, w, r)
    toks = np.asarray(draft_tokens).reshape(B, h * w)
    tokens_hi = toks[:, q_row].astype(np.int32)
    q_hi = q_lo[:, q_row, :] if materialise else None
    return tokens_hi, q_lo, q_row, q_hi
