"""The oracle's whole verification step on the Tiny workload: invariants that
tie the stages together.  CPU only."""
import numpy as np

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
