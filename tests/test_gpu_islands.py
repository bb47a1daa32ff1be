"""Island-parallel re-sampling (Sec. 3.4) through the C ABI against the CPU oracle.

The device labels the islands itself (mulo_rejection_islands), then re-samples them pass by pass.  As for the
sequential re-sampler, a differing draw changes the context of everything settled after it, so the comparison is
teacher-forced on the device's own result: the oracle's `resample_islands` is re-run with every draw replaced by
the device's token, and each device token must equal the oracle's draw from the oracle's row for that context
(except within the logit tolerance of a CDF boundary); the logit rows must agree to the bf16 bar."""
import numpy as np
import pytest
import torch

import paper_2601_05149_amd as mulo
from oracle import accept as A
from oracle import decoder as OD
from oracle import local as LOC
from oracle import philox as PH
from oracle import resample as RS
from oracle import step as ST
from tests.gpu_util import DEV, make_ctx, say
from workloads import generators as G

pytestmark = pytest.mark.gpu


def _device_run(m, w, B, Pn, H, W, mask, seed, ctr, cap_extra=0, n_passes=None):
    V, L = m["vocab"], H * W
    max_seq = (Pn + L + 15) // 8 * 8
    ctx, cos, sin = make_ctx(m, w, B, max_seq, max(Pn, L), stream_copy=m["dtype"] == "bf16")
    kv = mulo.alloc_kv(ctx, DEV)
    prefix = G.uniform_tokens((B, Pn), V, 0, tag=0)
    draft = G.uniform_tokens((B, L), V, 1, tag=0)
    P = Pn - 1
    scratch = torch.empty(B, max(Pn, L), V, device=DEV)
    mulo.mulo_verify_forward(ctx, kv, B, P, 0, torch.tensor(np.ascontiguousarray(prefix[:, :-1]), device=DEV), None,
                             scratch[:, :P].contiguous())
    inp = np.concatenate([prefix[:, -1:], draft[:, :-1]], axis=1)
    mulo.mulo_verify_forward(ctx, kv, B, L, P, torch.tensor(np.ascontiguousarray(inp), device=DEV), None,
                             scratch[:, :L].contiguous())
    mask_d = torch.tensor(mask.astype(np.uint8), device=DEV)
    island = torch.empty(B, L, dtype=torch.int32, device=DEV)
    rank = torch.empty(B, L, dtype=torch.int32, device=DEV)
    counts = torch.empty(B, 2, dtype=torch.int32, device=DEV)
    mulo.mulo_rejection_islands(ctx, B, W, 0, L, mask_d, island, rank, counts)
    cn = counts.cpu().numpy()
    cap = max(1, int(cn[:, 0].max())) + cap_extra
    passes = int(cn[:, 1].max()) if n_passes is None else n_passes
    tokens = torch.tensor(draft, device=DEV)
    logits = torch.zeros(B, L, V, device=DEV)
    over = torch.zeros(1, dtype=torch.int32, device=DEV)
    mulo.mulo_resample_islands(ctx, kv, B, P, L, passes, cap, seed, ctr,
                               torch.tensor(np.ascontiguousarray(prefix[:, -1]), device=DEV), mask_d, rank, tokens, logits, over)
    torch.cuda.synchronize()
    return dict(ctx=ctx, kv=kv, cos=cos, sin=sin, prefix=prefix, draft=draft, P=P, max_seq=max_seq, rank=rank.cpu().numpy(),
                counts=cn, cap=cap, passes=passes, tokens=tokens.cpu().numpy(), logits=logits.cpu().numpy(),
                overflow=int(over.item()))


def _oracle_teacher_forced(m, w, r, mask, seed, ctr, round_bf16):
    """The oracle's passes with the device's tokens forced in: rows[(b, u)] is the oracle's logit row for position
    u given exactly the context the device had (its own earlier draws)."""
    B, L = mask.shape
    dec = OD.DecoderOracle(m, w, r["cos"], r["sin"], B, r["max_seq"], round_bf16=round_bf16)
    P = r["P"]
    dec.forward(r["prefix"][:, :-1], 0)
    dec.forward(np.concatenate([r["prefix"][:, -1:], r["draft"][:, :-1]], axis=1), P)
    got = r["tokens"]
    orig_draw = RS.draw
    order = []
    words = PH.step_words(seed, ctr, PH.STREAM_SEQUENTIAL, B, L)
    lookup = {int(words[b, u]): (b, u) for b, u in zip(*np.nonzero(mask))}
    assert len(lookup) == int(mask.sum())                      # the words identify the positions
    try:
        RS.draw = lambda Wi, word: (order.append(lookup[int(word)]), int(got[lookup[int(word)]]))[1]
        tok, passes, rows = ST.resample_islands(dec, P, r["draft"], mask, r["rank"], r["prefix"][:, -1], seed=seed, rng_counter=ctr)
    finally:
        RS.draw = orig_draw
    assert np.array_equal(tok, got)
    return rows, passes, words


def _compare(m, w, r, mask, seed, ctr, round_bf16, logit_tol):
    B, L = mask.shape
    got = r["tokens"]
    assert r["overflow"] == 0
    assert np.array_equal(got[~mask], r["draft"][~mask])
    ranks = np.stack([LOC.rejection_islands(mask[b], r["W"], 0)[1] for b in range(B)])
    assert np.array_equal(r["rank"], ranks)
    rows, passes, words = _oracle_teacher_forced(m, w, r, mask, seed, ctr, round_bf16)
    assert passes == r["counts"][:, 1].max()
    rel = np.expm1(2 * logit_tol) + 1e-4
    err, n_close = 0.0, 0
    for (b, u), z in rows.items():
        err = max(err, float(np.abs(r["logits"][b, u] - z).max()))
        Wi = RS.integer_weights(A.target_probs(z))
        want = RS.draw(Wi, words[b, u])
        if got[b, u] != want:
            assert RS.boundary_distance(Wi, words[b, u]) < 4 * rel, "token differs away from a CDF boundary (b=%d u=%d)" % (b, u)
            n_close += 1
    say("  islands: %d marked in %d passes, max|logit err| %.3g, %d draws at a boundary" % (mask.sum(), passes, err, n_close))
    return err


SMALL = dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=512, vocab=2048, dtype="bf16", rms_eps=1e-5)


WIDE_HEADS = dict(n_layers=2, d_model=256, n_heads=2, head_dim=128, d_ffn=512, vocab=2048, dtype="bf16", rms_eps=1e-5)


@pytest.mark.parametrize("m", [SMALL, WIDE_HEADS], ids=["dh64", "dh128"])
def test_islands_small_bf16_several_islands_vs_oracle(m):
    w = G.make_weights(m, seed=0, threads=4)
    B, Pn, H, W = 3, 9, 8, 8
    L = H * W
    mask = np.zeros((B, L), bool)
    mask[0, [1, 2, 10]] = True; mask[0, [30, 31, 39, 47]] = True; mask[0, 56] = True
    mask[1, [8, 16, 24]] = True; mask[1, 15] = True                      # 15 | 16: raster neighbours, not grid neighbours
    mask[2, 20:44] = True                                               # three full rows: one long island
    r = _device_run(m, w, B, Pn, H, W, mask, seed=5, ctr=(2 << 32) | 9)
    r["W"] = W
    assert r["counts"].tolist() == [[3, 4], [2, 3], [1, 24]]
    err = _compare(m, w, r, mask, 5, (2 << 32) | 9, True, 2e-2)
    assert err <= 2e-2
    assert (r["tokens"][mask] != r["draft"][mask]).mean() > 0.9


def test_islands_one_island_from_t0_equals_sequential_on_device():
    """Everything from t0 on marked: the device's island path and its sequential path give the same tokens."""
    m = SMALL
    w = G.make_weights(m, seed=0, threads=4)
    B, Pn, H, W = 2, 8, 4, 8
    L = H * W
    t0 = np.array([5, 11])
    mask = np.arange(L)[None, :] >= t0[:, None]
    r = _device_run(m, w, B, Pn, H, W, mask, seed=3, ctr=4, n_passes=L - 5)
    assert r["overflow"] == 0
    # sequential path on a fresh cache
    ctx, kv = r["ctx"], mulo.alloc_kv(r["ctx"], DEV)
    V, P = m["vocab"], r["P"]
    scratch = torch.empty(B, max(Pn, L), V, device=DEV)
    mulo.mulo_verify_forward(ctx, kv, B, P, 0, torch.tensor(np.ascontiguousarray(r["prefix"][:, :-1]), device=DEV), None,
                             scratch[:, :P].contiguous())
    inp = np.concatenate([r["prefix"][:, -1:], r["draft"][:, :-1]], axis=1)
    mulo.mulo_verify_forward(ctx, kv, B, L, P, torch.tensor(np.ascontiguousarray(inp), device=DEV), None, scratch[:, :L].contiguous())
    tokens = torch.tensor(r["draft"], device=DEV)
    mulo.mulo_resample_sequential(ctx, kv, B, P, L, 5, 3, 4, torch.tensor(np.ascontiguousarray(r["prefix"][:, -1]), device=DEV),
                                  torch.tensor(mask.astype(np.uint8), device=DEV), tokens)
    torch.cuda.synchronize()
    seq = tokens.cpu().numpy()
    # sequence 0 (t0 = 5 = u_start) sees identical contexts on both paths; sequence 1's unmarked rows 5 .. 10 are
    # refreshed by the sequential path only, with their unchanged inputs and context: the same values
    same = (seq == r["tokens"]).mean()
    say("  one island vs sequential: %.3f of the tokens equal" % same)
    assert np.array_equal(seq[0], r["tokens"][0])
    assert same > 0.9


def test_islands_slot_bound_too_small_is_reported_and_errors():
    m = dict(n_layers=1, d_model=128, n_heads=2, head_dim=64, d_ffn=128, vocab=256, dtype="bf16", rms_eps=1e-5)
    w = G.make_weights(m, seed=0, threads=2)
    B, Pn, H, W = 2, 4, 4, 4
    L = H * W
    mask = np.zeros((B, L), bool); mask[0, [0, 3, 12, 15]] = True; mask[1, 5] = True      # four single-position islands
    r = _device_run(m, w, B, Pn, H, W, mask, seed=1, ctr=0, cap_extra=-2)                 # room for two of them
    assert r["cap"] == 2 and r["overflow"] == 2
    assert (r["tokens"][0, [12, 15]] == r["draft"][0, [12, 15]]).all()                    # the surplus was not re-drawn
    ctx, kv = r["ctx"], r["kv"]
    i32 = lambda *s: torch.zeros(*s, dtype=torch.int32, device=DEV)
    u8 = torch.zeros(B, L, dtype=torch.uint8, device=DEV)
    for bad in (dict(n_passes=-1), dict(cap=0), dict(cap=10 ** 6), dict(P=100)):
        with pytest.raises(mulo.MuloError):
            mulo.mulo_resample_islands(ctx, kv, B, bad.get("P", 3), L, bad.get("n_passes", 1), bad.get("cap", 4), 0, 0, i32(B), u8,
                                       i32(B, L), i32(B, L))
    mt = dict(n_layers=1, d_model=64, n_heads=1, head_dim=64, d_ffn=64, vocab=64, dtype="f32", rms_eps=1e-5)
    ctx32, _, _ = make_ctx(mt, G.make_weights(mt, seed=0, threads=1), B, 32, L)
    with pytest.raises(mulo.MuloError) as e:
        mulo.mulo_resample_islands(ctx32, mulo.alloc_kv(ctx32, DEV), B, 3, L, 1, 4, 0, 0, i32(B), u8, i32(B, L), i32(B, L))
    assert e.value.status == 6


@pytest.mark.parametrize("B", [3, 5])
def test_islands_many_single_positions_in_one_pass(B):
    """16 isolated positions per sequence, one pass: 48 slots go through the weight-streaming kernel (three token
    groups), 80 slots are more than it takes, so the tiled GEMMs place their rows through the slot table (ragged
    tile, scattered cache rows)."""
    m = SMALL
    w = G.make_weights(m, seed=0, threads=4)
    Pn, H, W = 6, 8, 8
    L = H * W
    mask = np.zeros((B, H, W), bool)
    mask[:, ::2, ::2] = True
    mask[1, 0, 0] = False                                   # 15 islands in sequence 1: one unused slot
    mask = mask.reshape(B, L)
    r = _device_run(m, w, B, Pn, H, W, mask, seed=8, ctr=1)
    r["W"] = W
    assert r["counts"][:3].tolist() == [[16, 1], [15, 1], [16, 1]] and r["cap"] == 16
    err = _compare(m, w, r, mask, 8, 1, True, 2e-2)
    assert err <= 2e-2
