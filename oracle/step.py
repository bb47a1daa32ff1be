"""The whole verification step (Alg. 1 Steps 2-5, plus the one-shot residual
resampling of the marked positions that stands in for Step 6).  Test
infrastructure; composes the other oracle modules in the order of the paper.
"""
import numpy as np

from . import accept as A
from . import local as LOC
from . import philox as PH
from . import resample as RS
from . import upsample as UP


def decide(logits, q_rows, q_row_index, draft_tokens, *, W, n0, radius, expand=1,
           seed=0, rng_counter=0, nbr=None, mode=0, accept_mode=0, tau=0.0, logits_uncond=None,
           cfg_scale=1.0):
    """Decision stage on given logits (Sec. 3.1 Eq. 1-3, Sec. 3.3 Eq. 5-7).

    accept_mode 0: speculative test u q < pbar (Eq. 1 / Eq. 3); accept_mode 1:
    threshold test pbar >= tau (Eq. 5), where q_rows may be None if mode == 2.
    logits_uncond: float [B, L, V] or None; with it the target distribution is the softmax of the
    guided logits z_u + cfg_scale (z_c - z_u) (classifier-free guidance, supplement "Sampling").

    logits: float [B, L, V]; q_rows: float32 [B, n_q, V]; q_row_index: int [L]
    or None (identity); draft_tokens: int [B, L].
    Returns a dict of arrays: p, pbar, q_tok, u, accept, near_tie, mask, t0,
    tokens_out, stats [B, 4] = (accepted, rejected, marked, near ties).
    """
    logits = np.asarray(logits)
    if logits_uncond is not None:
        logits = A.guided_logits(logits, logits_uncond, cfg_scale)
    B, L, V = logits.shape
    qi = np.arange(L) if q_row_index is None else np.asarray(q_row_index).astype(np.int64)
    toks = np.asarray(draft_tokens).astype(np.int64).reshape(B, L)
    u = PH.uniform24(PH.step_words(seed, rng_counter, PH.STREAM_ACCEPT, B, L))
    words = PH.step_words(seed, rng_counter, PH.STREAM_SAMPLE, B, L)
    out = dict(p=np.empty((B, L, V), np.float32), pbar=np.empty((B, L), np.float32),
               q_tok=np.empty((B, L), np.float32), u=u, words=words,
               accept=np.empty((B, L), np.uint8), near_tie=np.empty((B, L), bool),
               mask=np.empty((B, L), np.uint8), t0=np.empty(B, np.int32),
               tokens_out=np.empty((B, L), np.int32), stats=np.zeros((B, 4), np.int32))
    for b in range(B):
        p = A.target_probs(logits[b])                                   # Step 3 -> p_i
        pbar = A.pooled_mass(p, toks[b], nbr)                           # Eq. 3 numerator
        qb = None if q_rows is None else np.asarray(q_rows[b], dtype=np.float32)
        q_tok = np.zeros(L, np.float32) if qb is None else qb[qi, toks[b]]   # q_i(x~_i)
        if accept_mode == 1:
            acc = A.accept_test_tau(pbar, tau)                          # Eq. 5
            nt = A.near_tie_tau(pbar, tau)
        else:
            acc = A.accept_test(pbar, q_tok, u[b])                      # Eq. 1
            nt = A.near_tie(pbar, q_tok, u[b])
        mask, t0 = LOC.local_mask(acc, W, n0, radius, expand)           # Eq. 6-7
        tok_out = RS.resample_block(p, qb, qi, toks[b], mask, acc, words[b], mode)  # Eq. 2 / Step 6
        out["p"][b], out["pbar"][b], out["q_tok"][b] = p, pbar, q_tok
        out["accept"][b], out["near_tie"][b] = acc, nt
        out["mask"][b], out["t0"][b], out["tokens_out"][b] = mask, t0, tok_out
        out["stats"][b] = (int(acc.sum()), int(L - acc.sum()), int(mask.sum()), int(nt.sum()))
    return out


def verify_step(decoder, P, draft_lo, draft_tokens_lo, prev_tokens, *, h_blk, w, r, W, n0,
                radius, expand=1, seed=0, rng_counter=0, nbr=None, mode=0,
                input_is_probs=False, accept_mode=0, tau=0.0):
    """Steps 2-5 + resampling for one block of L = (r*h_blk)*(r*w) positions.

    decoder: oracle.decoder.DecoderOracle whose cache holds P valid rows;
    draft_lo: [B, h_blk*w, V] draft logits (or probabilities) of the low-res rows
    behind this block; draft_tokens_lo: [B, h_blk*w]; prev_tokens: [B] the last
    committed (or last prefix) token.  Target inputs are [prev, x~_0 .. x~_{L-2}],
    so logit row j is p for draft position j (Alg. 1 Step 3).
    """
    tokens_hi, q_lo, q_row, _ = UP.upsample_draft(draft_lo, draft_tokens_lo, h_blk, w, r,
                                                  input_is_probs=input_is_probs)
    B, L = tokens_hi.shape
    inp = np.concatenate([np.asarray(prev_tokens).reshape(B, 1).astype(np.int32),
                          tokens_hi[:, :L - 1]], axis=1)
    logits = decoder.forward(inp, P).numpy()
    out = decide(logits, q_lo, q_row, tokens_hi, W=W, n0=n0, radius=radius, expand=expand,
                 seed=seed, rng_counter=rng_counter, nbr=nbr, mode=mode, accept_mode=accept_mode, tau=tau)
    out.update(tokens_hi=tokens_hi, q_lo=q_lo, q_row=q_row, logits=logits)
    return out


def resample_sequential(decoder, P, tokens, mask, t0, prev_tokens, *, seed=0, rng_counter=0):
    """Alg. 1 Step 6: the marked positions R_X are visited in increasing order and each gets a
    sample of the target model given the prefix and ALL earlier positions of the block as they
    stand after the earlier re-draws:  x_k ~ M_p(x | x_0 .. x_{k-1}).

    decoder: oracle decoder whose cache rows [0, P) are valid (rows of the block may hold anything:
    every row from the first marked position on is recomputed here, one token at a time, because
    its input or its context has changed).  tokens: int [B, L] block after the parallel step (draft
    tokens; marked positions are overwritten); mask: [B, L]; t0: [B] first rejected position (L if
    none); prev_tokens: [B].  The draw uses the integer inverse CDF of p (float32 probabilities)
    with the Philox word of stream 2 at (position, batch element).
    Returns (tokens_out int32 [B, L], logits float64 [B, L, V] with rows before min(t0) left at 0).
    """
    tok = np.asarray(tokens).astype(np.int32).copy()
    mask = np.asarray(mask).astype(bool)
    B, L = tok.shape
    words = PH.step_words(seed, rng_counter, PH.STREAM_SEQUENTIAL, B, L)
    start = int(np.min(t0))
    logits = None
    for u in range(start, L):
        inp = np.asarray(prev_tokens).reshape(B, 1) if u == 0 else tok[:, u - 1:u]
        z = decoder.forward(inp.astype(np.int32), P + u).numpy()[:, 0]       # [B, V]; rewrites cache row P + u
        if logits is None:
            logits = np.zeros((B, L, z.shape[-1]))
        logits[:, u] = z
        for b in range(B):
            if mask[b, u]:
                tok[b, u] = RS.draw(RS.integer_weights(A.target_probs(z[b])), words[b, u])
    if logits is None:
        logits = np.zeros((B, L, 0))
    return tok, logits


def resample_islands(decoder, P, tokens, mask, rank, prev_tokens, *, seed=0, rng_counter=0):
    """Island-parallel re-sampling (Sec. 3.4): the rejection islands of Eq. 8 are re-sampled concurrently,
    the positions inside an island one after the other in raster order.  Pass r evaluates, in ONE target
    call, the position of rank r of every island that has one, and draws its token from the target model.

    The paper does not spell out the context of such a concurrent evaluation; the reading taken here (Sec. 3.4:
    only settled positions are context): the query at block position u
    attends to the prefix and to those earlier block positions that are settled -- accepted ones (their cache
    rows are the verification pass's) and marked ones re-drawn in an earlier pass (rows rewritten then) --
    and to itself; marked positions not yet re-drawn are hidden.  Its input is the current token at u - 1.
    Its k, v replace cache row P + u; no other row is touched, so the row P + u + 1 of an unmarked successor keeps
    the k, v of the draft token that stood at u during verification (the caller commits the block afterwards).  Draws use the integer inverse CDF of p with the Philox word of the
    sequential stream at (position, batch element), so one island covering everything from its first
    position on is exactly `resample_sequential`.

    decoder: oracle decoder whose rows [0, P) are valid and whose rows P .. P+L-1 hold the verification pass
    of the block; tokens: int [B, L]; mask: [B, L] = R_X; rank: int [B, L] from local.rejection_islands
    (-1 where unmarked); prev_tokens: [B].  Returns (tokens_out int32 [B, L], passes, logits {(b, u): row})."""
    tok = np.asarray(tokens).astype(np.int32).copy()
    mask = np.asarray(mask).astype(bool)
    rank = np.asarray(rank)
    B, L = tok.shape
    words = PH.step_words(seed, rng_counter, PH.STREAM_SEQUENTIAL, B, L)
    settled = ~mask                                   # positions whose token and cache row are final
    passes = 0
    rows = {}
    while not settled.all():
        sel = [(b, u) for b in range(B) for u in range(L) if mask[b, u] and rank[b, u] == passes]
        assert sel, "ranks must be consecutive inside every island"
        inp = [int(np.asarray(prev_tokens)[b]) if u == 0 else int(tok[b, u - 1]) for b, u in sel]
        vis = np.zeros((len(sel), P + L), dtype=bool)
        for i, (b, u) in enumerate(sel):
            vis[i, :P] = True
            vis[i, P:P + u] = settled[b, :u]
            vis[i, P + u] = True
        z = decoder.forward_at(inp, [b for b, _ in sel], [P + u for _, u in sel], vis).numpy()
        for i, (b, u) in enumerate(sel):
            tok[b, u] = RS.draw(RS.integer_weights(A.target_probs(z[i])), words[b, u])
            rows[(b, u)] = z[i]
        for b, u in sel:
            settled[b, u] = True
        passes += 1
    return tok, passes, rows
