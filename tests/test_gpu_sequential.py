"""Sequential re-sampling (Alg. 1 Step 6) through the C ABI against the CPU oracle.

The re-drawn tokens feed back into the context, so one differing draw changes everything after it in that
sequence.  Parity is therefore checked the way the step tests do it: position by position, the device's token
must equal the oracle's draw from the ORACLE's distribution given the DEVICE's own earlier tokens (teacher
forcing on the device's output), except where the draw's threshold lies within the logit tolerance of a CDF
boundary; the logit rows the device used must match the oracle's for the same context."""
import numpy as np
import pytest
import torch

import paper_2601_05149_amd as mulo
from oracle import accept as A
from oracle import decoder as OD
from oracle import philox as PH
from oracle import resample as RS
from oracle import step as ST
from tests.gpu_util import DEV, make_ctx, say
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _run(m, B, Pn, L, mask, t0, seed, ctr, round_bf16, logit_tol):
    V = m["vocab"]
    w = G.make_weights(m, seed=0, threads=4)
    max_seq = (Pn + L + 15) // 8 * 8
    ctx, cos, sin = make_ctx(m, w, B, max_seq, (max(Pn, L) + 3) // 4 * 4, stream_copy=m["dtype"] == "bf16")
    kv = mulo.alloc_kv(ctx, DEV)
    prefix = G.uniform_tokens((B, Pn), V, 0, tag=0)
    draft = G.uniform_tokens((B, L), V, 1, tag=0)
    # convention of the step: rows [0, P) are cached and `prev` is the token that follows them, so the
    # context prefix is prefilled without its last token (P = Pn - 1), which is passed as prev
    P = Pn - 1
    scratch = torch.empty(B, max(Pn, L), V, device=DEV)
    mulo.mulo_verify_forward(ctx, kv, B, P, 0, torch.tensor(np.ascontiguousarray(prefix[:, :-1]), device=DEV), None,
                             scratch[:, :P].contiguous())
    # the parallel pass over the block (fills the block's cache rows, as the verify step would)
    inp = np.concatenate([prefix[:, -1:], draft[:, :-1]], axis=1)
    mulo.mulo_verify_forward(ctx, kv, B, L, P, torch.tensor(np.ascontiguousarray(inp), device=DEV), None,
                             scratch[:, :L].contiguous())
    tokens = torch.tensor(draft, device=DEV)
    logits = torch.zeros(B, L, V, device=DEV)
    mulo.mulo_resample_sequential(ctx, kv, B, P, L, int(t0.min()), seed, ctr, torch.tensor(np.ascontiguousarray(prefix[:, -1]), device=DEV),
                                  torch.tensor(mask.astype(np.uint8), device=DEV), tokens, logits)
    torch.cuda.synchronize()
    got, zg = tokens.cpu().numpy(), logits.cpu().numpy()
    assert np.array_equal(got[~mask], draft[~mask])
    # oracle: every conditional of the device's final sequence in one teacher-forced pass
    dec = OD.DecoderOracle(m, w, cos, sin, B, max_seq, round_bf16=round_bf16)
    z = dec.forward(np.concatenate([prefix, got], axis=1)[:, :-1], 0).numpy()[:, Pn - 1:]      # [B, L, V]
    lo = int(t0.min())
    err = np.abs(zg[:, lo:] - z[:, lo:]).max()
    words = PH.step_words(seed, ctr, PH.STREAM_SEQUENTIAL, B, L)
    rel = np.expm1(2 * logit_tol) + 1e-4
    n_close = 0
    for b, u in zip(*np.nonzero(mask)):
        Wi = RS.integer_weights(A.target_probs(z[b, u]))
        want = RS.draw(Wi, words[b, u])
        if got[b, u] != want:
            assert RS.boundary_distance(Wi, words[b, u]) < 4 * rel, "token differs away from a CDF boundary (b=%d u=%d)" % (b, u)
            n_close += 1
    say("  sequential: %d marked, max|logit err| %.3g, %d draws at a boundary" % (mask.sum(), err, n_close))
    return err, got, draft


def test_sequential_tiny_f32():
    m = dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=688, vocab=1024, dtype="f32", rms_eps=1e-5)
    B, Pn, L = 2, 9, 24
    rng = np.random.default_rng(0)
    mask = rng.random((B, L)) < 0.4
    mask[:, :3] = False
    t0 = np.array([np.flatnonzero(mask[b])[0] for b in range(B)])
    err, got, draft = _run(m, B, Pn, L, mask, t0, seed=5, ctr=1, round_bf16=False, logit_tol=1e-4)
    assert err <= 1e-4
    assert (got[mask] != draft[mask]).mean() > 0.9      # V = 1024: a re-draw almost never repeats the draft


def test_sequential_small_bf16_all_marked_is_ancestral_sampling():
    m = dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=512, vocab=2048, dtype="bf16", rms_eps=1e-5)
    B, Pn, L = 3, 8, 16
    mask = np.ones((B, L), bool)
    err, got, draft = _run(m, B, Pn, L, mask, np.zeros(B, int), seed=11, ctr=(3 << 32) | 7, round_bf16=True, logit_tol=2e-2)
    assert err <= 2e-2


def test_sequential_nothing_marked_and_errors():
    m = dict(n_layers=1, d_model=128, n_heads=2, head_dim=64, d_ffn=128, vocab=256, dtype="bf16", rms_eps=1e-5)
    B, Pn, L = 2, 4, 8
    w = G.make_weights(m, seed=0, threads=2)
    ctx, cos, sin = make_ctx(m, w, B, 16, L)
    kv = mulo.alloc_kv(ctx, DEV)
    toks = torch.tensor(G.uniform_tokens((B, L), 256, 2, tag=0), device=DEV)
    before = toks.clone()
    prev = torch.zeros(B, dtype=torch.int32, device=DEV)
    none = torch.zeros(B, L, dtype=torch.uint8, device=DEV)
    mulo.mulo_resample_sequential(ctx, kv, B, Pn, L, L, 0, 0, prev, none, toks)      # u_start = L: nothing to do
    mulo.mulo_resample_sequential(ctx, kv, B, Pn, L, 0, 0, 0, prev, none, toks)      # all positions refreshed, none drawn
    torch.cuda.synchronize()
    assert torch.equal(toks, before)
    for bad in (dict(u_start=-1), dict(u_start=L + 1), dict(P=9)):       # 9 + 8 rows exceed the 16-row cache
        with pytest.raises(mulo.MuloError):
            mulo.mulo_resample_sequential(ctx, kv, B, bad.get("P", Pn), L, bad.get("u_start", 0), 0, 0, prev, none, toks)
