"""The oracle's whole verification step on the Tiny workload: invariants that
tie the stages together.  CPU only."""
import numpy as np
import torch

from oracle import accept as A
from oracle import decoder as D
from oracle import philox as PH
from oracle import resample as RS
from oracle import step as ST
from workloads import configs as C
from workloads import generators as G


def _tiny_step(seed=0, rng_counter=0):
    c = C.get("cfg1")
    m = c["model"]
    w = G.make_weights(m, seed=seed)
    cos, sin = G.rope_table(c["max_seq"], m["head_dim"])
    dec = D.DecoderOracle(m, w, cos, sin, c["B"], c["max_seq"], round_bf16=False)
    prefix = G.uniform_tokens((c["B"], c["prefix"]), m["vocab"], seed, tag=0)
    dec.forward(prefix, 0)
    dl = G.normal_logits((c["B"], c["h"] * c["w"], m["vocab"]), c["draft_std"], seed, tag=0)
    dt = G.sample_categorical(dl, seed, tag=0)
    out = ST.verify_step(dec, c["prefix"], dl, dt, prefix[:, -1], h_blk=c["h"], w=c["w"], r=c["r"],
                         W=c["W"], n0=0, radius=c["radius"], expand=c["expand"], seed=seed,
                         rng_counter=rng_counter)
    return c, dec, dt, out


def test_tiny_step_invariants():
    c, dec, dt, out = _tiny_step()
    B, L, V = c["B"], c["L"], c["model"]["vocab"]
    assert out["logits"].shape == (B, L, V) and out["tokens_out"].shape == (B, L)
    # draft tokens on the target grid are the replicated low-res tokens
    assert np.array_equal(out["tokens_hi"].reshape(B, c["h"], 2, c["w"], 2)[:, :, 0, :, 0].reshape(B, -1), dt)
    acc, mask = out["accept"].astype(bool), out["mask"].astype(bool)
    # random draft vs an unrelated target: partial acceptance, some positions marked
    assert 0 < acc.sum() < B * L and mask.sum() >= (~acc).sum()
    assert np.array_equal(out["tokens_out"][~mask], out["tokens_hi"][~mask])
    assert (out["tokens_out"] >= 0).all() and (out["tokens_out"] < V).all()
    assert np.abs(out["p"].astype(np.float64).sum(-1) - 1).max() < 1e-6
    # cache rows of the block were written, rows of the prefix kept
    assert dec.k[:, :, c["prefix"]:c["prefix"] + L].abs().min() > 0
    # the step is a pure function of (inputs, seed, counter)
    _, _, _, again = _tiny_step()
    assert np.array_equal(again["tokens_out"], out["tokens_out"])
    _, _, _, other = _tiny_step(rng_counter=1)
    assert not np.array_equal(other["accept"], out["accept"])


# ------------------------------------------------------------------ sequential re-sampling (Alg. 1 Step 6)
# Convention of the step: the cache holds rows [0, P) and `prev` is the token that FOLLOWS them (its own row
# is written by the step at row P).  So a context "prefix" of n tokens is prefilled as prefix[:, :-1]
# (P = n - 1) with prev = prefix[:, -1].
def _seq_setup(seed=4):
    from oracle import decoder as OD
    m = dict(n_layers=2, d_model=32, n_heads=2, head_dim=16, d_ffn=48, vocab=24, dtype="f32", rms_eps=1e-5)
    w = G.make_weights(m, seed=seed, std=0.35, threads=1)      # large enough for peaked, context-dependent distributions
    cos, sin = G.rope_table(64, m["head_dim"])
    mk = lambda: OD.DecoderOracle(m, w, cos, sin, 2, 64, round_bf16=False)
    return m, mk


def _teacher_forced(mk, prefix, out):
    """Logit rows of the conditionals of out[:, u] given prefix and out[:, :u], by one block pass."""
    ref = mk()
    z = ref.forward(np.concatenate([prefix, out], axis=1)[:, :-1], 0).numpy()
    return z[:, prefix.shape[1] - 1:]


def test_sequential_resampling_is_ancestral_sampling_of_the_target():
    """With every position marked, Step 6 is plain autoregressive sampling: position u is the inverse-CDF
    draw from the target's next-token distribution given the prefix and the tokens drawn before it.  Checked
    against a from-scratch recomputation (a fresh decoder run over the whole final sequence)."""
    m, mk = _seq_setup()
    V, B, Pn, L = m["vocab"], 2, 5, 12
    prefix = G.uniform_tokens((B, Pn), V, 1, tag=0)
    dec = mk(); dec.forward(prefix[:, :-1], 0)
    draft = G.uniform_tokens((B, L), V, 2, tag=0)
    out, zs = ST.resample_sequential(dec, Pn - 1, draft, np.ones((B, L), bool), np.zeros(B, int), prefix[:, -1], seed=9, rng_counter=3)
    z = _teacher_forced(mk, prefix, out)
    assert np.abs(zs - z).max() < 1e-9                    # the rows it sampled from are those conditionals
    assert A.target_probs(z).max(-1).mean() > 0.2         # the distributions are far from uniform ...
    assert np.abs(z[:, 1:] - z[:, :-1]).max() > 1.0       # ... and depend on the context
    words = PH.step_words(9, 3, PH.STREAM_SEQUENTIAL, B, L)
    for b in range(B):
        for u in range(L):
            assert out[b, u] == RS.draw(RS.integer_weights(A.target_probs(z[b, u])), words[b, u])
    # a dropped context refresh would show: re-running with the stale draft as context gives other logits
    assert np.abs(_teacher_forced(mk, prefix, draft) - z)[:, 1:].max() > 0.1


def test_sequential_resampling_keeps_unmarked_tokens_and_refreshes_their_context():
    m, mk = _seq_setup()
    V, B, Pn, L = m["vocab"], 2, 4, 10
    prefix = G.uniform_tokens((B, Pn), V, 3, tag=0)
    draft = G.uniform_tokens((B, L), V, 4, tag=0)
    mask = np.zeros((B, L), bool); mask[0, [3, 4, 8]] = True; mask[1, [6]] = True
    t0 = np.array([3, 6])
    P = Pn - 1
    dec = mk(); dec.forward(prefix[:, :-1], 0)
    dec.forward(np.concatenate([prefix[:, -1:], draft[:, :-1]], axis=1), P)     # the verify pass filled the block rows
    out, zs = ST.resample_sequential(dec, P, draft, mask, t0, prefix[:, -1], seed=1, rng_counter=0)
    assert np.array_equal(out[~mask], draft[~mask])
    # the re-draws are samples of the conditionals of the FINAL sequence (later marked positions see the earlier re-draws)
    z = _teacher_forced(mk, prefix, out)
    lo = int(t0.min())
    assert np.abs(zs[:, lo:] - z[:, lo:]).max() < 1e-9
    words = PH.step_words(1, 0, PH.STREAM_SEQUENTIAL, B, L)
    for b, u in zip(*np.nonzero(mask)):
        assert out[b, u] == RS.draw(RS.integer_weights(A.target_probs(z[b, u])), words[b, u])
    # afterwards the block's cache rows equal those of a fresh pass over the final inputs [prev, out_0 .. out_{L-2}]
    fresh = mk(); fresh.forward(prefix[:, :-1], 0)
    fresh.forward(np.concatenate([prefix[:, -1:], out[:, :-1]], axis=1), P)
    assert np.allclose(dec.k[:, :B, :P + L].numpy(), fresh.k[:, :B, :P + L].numpy(), atol=1e-9)
    assert np.allclose(dec.v[:, :B, :P + L].numpy(), fresh.v[:, :B, :P + L].numpy(), atol=1e-9)
    stale = mk(); stale.forward(prefix[:, :-1], 0)
    stale.forward(np.concatenate([prefix[:, -1:], draft[:, :-1]], axis=1), P)
    assert np.abs(stale.k[:, :B, P + lo + 1:P + L].numpy() - fresh.k[:, :B, P + lo + 1:P + L].numpy()).max() > 1e-3


def test_sequential_resampling_with_nothing_marked_is_the_identity():
    m, mk = _seq_setup()
    V, B, Pn, L = m["vocab"], 2, 4, 6
    prefix = G.uniform_tokens((B, Pn), V, 5, tag=0)
    draft = G.uniform_tokens((B, L), V, 6, tag=0)
    dec = mk(); dec.forward(prefix[:, :-1], 0)
    out, _ = ST.resample_sequential(dec, Pn - 1, draft, np.zeros((B, L), bool), np.array([L, L]), prefix[:, -1])
    assert np.array_equal(out, draft)


# --------------------------------------------------------------- island-parallel re-sampling (Sec. 3.4)
def _island_setup(B, Pn, H, W, seed):
    """Prefix prefilled without its last token, then the verification pass over the drafted H x W block."""
    m, mk = _seq_setup()
    V, L = m["vocab"], H * W
    prefix = G.uniform_tokens((B, Pn), V, seed, tag=0)
    draft = G.uniform_tokens((B, L), V, seed + 1, tag=0)
    dec = mk(); dec.forward(prefix[:, :-1], 0)
    dec.forward(np.concatenate([prefix[:, -1:], draft[:, :-1]], axis=1), Pn - 1)
    return m, mk, prefix, draft, dec


def _ranks(mask, W):
    from oracle import local as LOC
    out = [LOC.rejection_islands(mk_, W, 0) for mk_ in mask]
    return np.stack([o[1] for o in out]), max(o[3] for o in out)


def test_forward_at_on_a_contiguous_causal_block_is_the_block_pass():
    """Scattered queries at consecutive rows with causal visibility are the ordinary pass over a block: the
    library-style batched forward and the per-query forward agree in logits and in the cache they leave."""
    m, mk = _seq_setup()
    B, Pn, L = 2, 5, 7
    toks = G.uniform_tokens((B, Pn + L), m["vocab"], 8, tag=0)
    a, b = mk(), mk()
    a.forward(toks[:, :Pn], 0); b.forward(toks[:, :Pn], 0)
    za = a.forward(toks[:, Pn:], Pn).numpy()
    # the same L rows per sequence as single-token queries (all written first, each sees rows <= its own)
    seq = [s for s in range(B) for _ in range(L)]
    pos = [Pn + j for _ in range(B) for j in range(L)]
    vis = np.zeros((B * L, Pn + L), bool)
    for i, r in enumerate(pos):
        vis[i, :r + 1] = True
    zb = b.forward_at(toks[:, Pn:].reshape(-1), seq, pos, vis).numpy().reshape(B, L, -1)
    assert np.abs(za - zb).max() < 1e-10
    assert np.allclose(a.k.numpy(), b.k.numpy(), atol=1e-12) and np.allclose(a.v.numpy(), b.v.numpy(), atol=1e-12)
    # hiding a row changes the result (the visibility argument is used)
    vis2 = vis.copy(); vis2[L - 1, Pn] = False
    assert np.abs(b.forward_at(toks[:, Pn:].reshape(-1), seq, pos, vis2).numpy()[L - 1] - za[0, L - 1]).max() > 1e-3


def test_one_island_from_t0_on_is_sequential_resampling():
    """Everything from t0 on marked = one island whose ranks are the raster order: the island-parallel scheme
    degenerates to Alg. 1 Step 6 (same tokens, same cache), which is pinned above as ancestral sampling."""
    B, Pn, H, W = 2, 4, 3, 4
    m, mk, prefix, draft, dec = _island_setup(B, Pn, H, W, seed=11)
    L = H * W
    t0 = np.array([2, 5])
    mask = np.arange(L)[None, :] >= t0[:, None]
    rank, largest = _ranks(mask, W)
    assert np.array_equal(rank[0, 2:], np.arange(L - 2)) and largest == L - 2
    out, passes, rows = ST.resample_islands(dec, Pn - 1, draft, mask, rank, prefix[:, -1], seed=3, rng_counter=2)
    m2, mk2, _, _, dec2 = _island_setup(B, Pn, H, W, seed=11)
    ref, zs = ST.resample_sequential(dec2, Pn - 1, draft, mask, t0, prefix[:, -1], seed=3, rng_counter=2)
    assert passes == largest and np.array_equal(out, ref)
    for b in range(B):      # cache rows from each sequence's t0 on were rewritten identically
        lo = Pn - 1 + t0[b]
        assert np.allclose(dec.k[:, b, lo:Pn - 1 + L].numpy(), dec2.k[:, b, lo:Pn - 1 + L].numpy(), atol=1e-9)
    for (b, u), z in rows.items():
        assert np.abs(z - zs[b, u]).max() < 1e-9


def test_islands_are_resampled_concurrently_and_see_only_settled_positions():
    B, Pn, H, W = 2, 4, 6, 6
    m, mk, prefix, draft, dec = _island_setup(B, Pn, H, W, seed=21)
    L, P = H * W, Pn - 1
    mask = np.zeros((B, L), bool)
    mask[0, [1, 2, 8]] = True          # island {1, 2, 8} (8 = row 1, col 2 touches 1 and 2 diagonally / vertically)
    mask[0, [22, 23, 29]] = True       # island {22, 23, 29}, far from the first
    mask[0, 33] = True                 # a single position
    mask[1, [6, 12, 18]] = True        # a vertical island in column 0
    mask[1, 11] = True                 # row 1, last column: raster neighbour of 12 but not a grid neighbour
    rank, largest = _ranks(mask, W)
    assert largest == 3 and rank[1, 11] == 0 and rank[1, 12] == 1
    calls = []
    orig = dec.forward_at
    dec.forward_at = lambda t, s, p, v: (calls.append((list(s), list(p), np.array(v))), orig(t, s, p, v))[1]
    out, passes, rows = ST.resample_islands(dec, P, draft, mask, rank, prefix[:, -1], seed=6, rng_counter=1)
    # one target call per rank, each holding one position of every island that still has one
    assert passes == 3 and [len(c[0]) for c in calls] == [5, 3, 3]
    assert np.array_equal(out[~mask], draft[~mask])
    # visibility, restated from the ranks: hidden = marked, not the query itself, rank >= pass
    for r, (seqs, rows_, vis) in enumerate(calls):
        for i, (b, row) in enumerate(zip(seqs, rows_)):
            u = row - P
            want = np.zeros(P + L, bool)
            want[:P] = True
            for v in range(u + 1):
                want[P + v] = v == u or not mask[b, v] or rank[b, v] < r
            assert np.array_equal(vis[i], want)
    # every draw is the inverse-CDF draw from the row the pass produced, with the sequential stream's word
    words = PH.step_words(6, 1, PH.STREAM_SEQUENTIAL, B, L)
    for (b, u), z in rows.items():
        assert out[b, u] == RS.draw(RS.integer_weights(A.target_probs(z)), words[b, u])
    # what the cache held at marked positions before the call never reaches a result: every such row is
    # rewritten before anything may attend to it
    m3, mk3, _, _, dec3 = _island_setup(B, Pn, H, W, seed=21)
    rng = np.random.default_rng(0)
    for b, u in zip(*np.nonzero(mask)):
        dec3.k[:, b, P + u] = torch.tensor(rng.normal(size=dec3.k[:, b, P + u].shape))
        dec3.v[:, b, P + u] = torch.tensor(rng.normal(size=dec3.v[:, b, P + u].shape))
    out3, _, rows3 = ST.resample_islands(dec3, P, draft, mask, rank, prefix[:, -1], seed=6, rng_counter=1)
    assert np.array_equal(out3, out) and max(np.abs(rows3[k] - rows[k]).max() for k in rows) < 1e-9
    # ... whereas an accepted position's row does (hiding too much would pass the line above)
    m4, mk4, _, _, dec4 = _island_setup(B, Pn, H, W, seed=21)
    dec4.k[:, 0, P + 0] += 1.0
    _, _, rows4 = ST.resample_islands(dec4, P, draft, mask, rank, prefix[:, -1], seed=6, rng_counter=1)
    assert np.abs(rows4[(0, 1)] - rows[(0, 1)]).max() > 1e-3
    # a later position of an island sees the earlier re-draw: its row is the conditional given the NEW token
    # (position 2 follows position 1 in island one: changing the word that drew 1 changes the row at 2)
    m5, mk5, _, _, dec5 = _island_setup(B, Pn, H, W, seed=21)
    out5, _, rows5 = ST.resample_islands(dec5, P, draft, mask, rank, prefix[:, -1], seed=7, rng_counter=1)
    if out5[0, 1] != out[0, 1]:
        assert np.abs(rows5[(0, 2)] - rows[(0, 2)]).max() > 1e-3


def test_island_resampling_with_nothing_marked_is_the_identity():
    B, Pn, H, W = 2, 4, 2, 3
    m, mk, prefix, draft, dec = _island_setup(B, Pn, H, W, seed=31)
    mask = np.zeros((B, H * W), bool)
    rank, largest = _ranks(mask, W)
    out, passes, rows = ST.resample_islands(dec, Pn - 1, draft, mask, rank, prefix[:, -1])
    assert passes == 0 and largest == 0 and not rows and np.array_equal(out, draft)
