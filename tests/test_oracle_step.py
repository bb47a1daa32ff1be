"""The oracle's whole verification step on the Tiny workload: invariants that
tie the stages together.  CPU only."""
import numpy as np

from oracle import decoder as D
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
