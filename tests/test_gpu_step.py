"""The whole verification step through the C ABI: it must equal the composition
of its three stages on the device bit for bit, and agree with the CPU oracle's
whole step wherever the oracle's decision margin exceeds what the logit
tolerance can move."""
import numpy as np
import pytest
import torch

import paper_2601_05149_amd as mulo
from oracle import decoder as OD
from oracle import resample as RS
from oracle import step as ST
from tests.gpu_util import DEV, check_bf16_logits, decide_buffers, make_ctx, say, to_np
from workloads import configs as WC
from workloads import generators as G

pytestmark = pytest.mark.gpu


def gpu_step(ctx, kv, c, P, n0, dl, dt, prev, rng_counter, seed=0, want_logits=True):
    B, L, V = dl.shape[0], c["L"], ctx.cfg.vocab
    out = decide_buffers(B, L)
    out["tokens_hi"] = torch.empty(B, L, dtype=torch.int32, device=DEV)
    out["logits"] = torch.empty(B, L, V, device=DEV) if want_logits else None
    params = mulo.make_params(c["H"], c["W"], n0, L, c["radius"], c["expand"], seed=seed, rng_counter=rng_counter)
    mulo.mulo_verify_step(ctx, kv, B, P, params, L // c["W"] // c["r"], c["w"], c["r"], torch.tensor(dl, device=DEV), 0,
                          torch.tensor(dt, device=DEV), torch.tensor(np.ascontiguousarray(prev), device=DEV),
                          out["tokens_out"], out["accept"], out["mask"], out["t0"], out["stats"], out["tokens_hi"],
                          out["logits"])
    torch.cuda.synchronize()
    return out


def gpu_composed(ctx, kv, c, P, n0, dl, dt, prev, rng_counter, seed=0):
    """The same step through the three stage entry points."""
    B, L, V = dl.shape[0], c["L"], ctx.cfg.vocab
    h_blk, w, r = L // c["W"] // c["r"], c["w"], c["r"]
    n_lo = h_blk * w
    thi = torch.empty(B, L, dtype=torch.int32, device=DEV)
    q_lo = torch.empty(B, n_lo, V, device=DEV)
    q_row = torch.empty(L, dtype=torch.int32, device=DEV)
    mulo.mulo_upsample_draft(ctx, B, h_blk, w, r, torch.tensor(dl, device=DEV), 0, torch.tensor(dt, device=DEV), thi,
                             q_lo, q_row, None)
    inp = torch.cat([torch.tensor(np.ascontiguousarray(prev), device=DEV).reshape(B, 1), thi[:, :L - 1]], dim=1).contiguous()
    logits = torch.empty(B, L, V, device=DEV)
    mulo.mulo_verify_forward(ctx, kv, B, L, P, inp, None, logits)
    out = decide_buffers(B, L)
    params = mulo.make_params(c["H"], c["W"], n0, L, c["radius"], c["expand"], seed=seed, rng_counter=rng_counter)
    mulo.mulo_accept_local_resample(ctx, B, params, logits, q_lo, q_row, n_lo * V, thi, out["tokens_out"],
                                    out["accept"], out["mask"], out["t0"], out["stats"], None)
    torch.cuda.synchronize()
    out["tokens_hi"], out["logits"] = thi, logits
    return out


def assert_same(a, b):
    for k in ("tokens_out", "accept", "mask", "t0", "stats", "tokens_hi", "logits"):
        assert torch.equal(a[k], b[k]), k


def compare_step_with_oracle(gpu, ref, logit_tol, label):
    """Accept flags may differ only where the oracle's margin |pbar - u q| is
    within what a logit error of logit_tol can move pbar (relative e^(2 tol) - 1)
    or at a near tie; sequences without a flip must match in mask / t0, and in the
    re-drawn tokens except draws whose threshold lies that close to a boundary."""
    rel = np.expm1(2 * logit_tol) + 1e-4
    acc_g, acc_r = gpu["accept"].astype(bool), ref["accept"].astype(bool)
    margin = np.abs(ref["pbar"].astype(np.float64) - ref["u"].astype(np.float64) * ref["q_tok"])
    movable = margin <= rel * np.maximum(ref["pbar"], ref["u"] * ref["q_tok"])
    diff = acc_g != acc_r
    assert not (diff & ~movable).any(), "%s: accept flag differs beyond the logit tolerance" % label
    assert np.array_equal(gpu["tokens_hi"], ref["tokens_hi"])
    n_tok = 0
    for b in range(acc_r.shape[0]):
        if diff[b].any():
            continue
        assert np.array_equal(gpu["mask"][b], ref["mask"][b]) and gpu["t0"][b] == ref["t0"][b]
        assert np.array_equal(gpu["stats"][b, :3], ref["stats"][b, :3])
        for u in np.flatnonzero(gpu["tokens_out"][b] != ref["tokens_out"][b]):
            assert ref["mask"][b, u]
            Wi = RS.residual_weights(ref["p"][b, u], ref["q_lo"][b][ref["q_row"][u]])
            assert RS.boundary_distance(Wi, ref["words"][b, u]) < 4 * rel, "%s: token differs away from a boundary" % label
            n_tok += 1
    return dict(flips=int(diff.sum()), movable=int(movable.sum()), tok_mismatch=n_tok)


@pytest.mark.parametrize("name", ["cfg1", "cfg1_r4"])
def test_step_tiny_f32_vs_oracle_and_composition(name):
    c = WC.get(name)
    m, B, L, Pn, V = c["model"], c["B"], c["L"], c["prefix"], c["model"]["vocab"]
    w = G.make_weights(m, seed=0)
    ctx, cos, sin = make_ctx(m, w, B, c["max_seq"], L)
    kv = mulo.alloc_kv(ctx, DEV)
    dec = OD.DecoderOracle(m, w, cos, sin, B, c["max_seq"], round_bf16=False)
    prefix = G.uniform_tokens((B, Pn), V, 0, tag=0)
    dec.forward(prefix, 0)
    mulo.mulo_verify_forward(ctx, kv, B, Pn, 0, torch.tensor(prefix, device=DEV), None, torch.empty(B, Pn, V, device=DEV))
    dl = G.normal_logits((B, c["h"] * c["w"], V), c["draft_std"], 0, tag=0)
    dt = G.sample_categorical(dl, 0, tag=0)
    ref = ST.verify_step(dec, Pn, dl, dt, prefix[:, -1], h_blk=c["h"], w=c["w"], r=c["r"], W=c["W"], n0=0,
                         radius=c["radius"], expand=c["expand"], seed=0, rng_counter=0)
    g = gpu_step(ctx, kv, c, Pn, 0, dl, dt, prefix[:, -1], 0)
    assert_same(g, gpu_composed(ctx, kv, c, Pn, 0, dl, dt, prefix[:, -1], 0))
    gn = to_np(g)
    err = np.abs(gn["logits"] - ref["logits"]).max()
    rep = compare_step_with_oracle(gn, ref, 1e-4, "tiny step")
    say("  tiny step %s (ratio %d, radius %d): max|logit err| %.3g acc %.3f marked %.3f %r"
        % (name, c["r"], c["radius"], err, ref["accept"].mean(), ref["mask"].mean(), rep))
    assert err <= 1e-4


def test_step_small_bf16_chained_blocks_vs_oracle():
    """Config 2: four 256-token blocks of a 32x32 grid, B = 4; after every block
    both sides commit the ORACLE's output tokens (so each block is compared on
    the same context) with an un-timed forward that rewrites the block's cache rows."""
    c = WC.get("cfg2")
    m, B, L, Pn, V = c["model"], c["B"], c["L"], c["prefix"], c["model"]["vocab"]
    w = G.make_weights(m, seed=0)
    ctx, cos, sin = make_ctx(m, w, B, c["max_seq"], L)
    kv = mulo.alloc_kv(ctx, DEV)
    dec = OD.DecoderOracle(m, w, cos, sin, B, c["max_seq"], round_bf16=True)
    exact = OD.DecoderOracle(m, w, cos, sin, B, c["max_seq"], round_bf16=False)   # for the rounding-noise floor
    prefix = G.uniform_tokens((B, Pn), V, 0, tag=0)
    dec.forward(prefix, 0)
    exact.forward(prefix, 0)
    scratch = torch.empty(B, L, V, device=DEV)
    mulo.mulo_verify_forward(ctx, kv, B, Pn, 0, torch.tensor(prefix, device=DEV), None, scratch[:, :Pn].contiguous())
    prev = prefix[:, -1].copy()
    rows_lo = L // c["W"] // c["r"]
    dl_all = G.normal_logits((B, c["h"] * c["w"], V), c["draft_std"], 0, tag=0)
    dt_all = G.sample_categorical(dl_all, 0, tag=0)
    P = Pn
    for blk in range(c["T"] // L):
        n0 = blk * L
        sl = slice(blk * rows_lo * c["w"], (blk + 1) * rows_lo * c["w"])
        dl, dt = np.ascontiguousarray(dl_all[:, sl]), np.ascontiguousarray(dt_all[:, sl])
        ref = ST.verify_step(dec, P, dl, dt, prev, h_blk=rows_lo, w=c["w"], r=c["r"], W=c["W"], n0=n0,
                             radius=c["radius"], expand=c["expand"], seed=0, rng_counter=blk)
        g = gpu_step(ctx, kv, c, P, n0, dl, dt, prev, blk)
        if blk == 0:
            assert_same(g, gpu_composed(ctx, kv, c, P, n0, dl, dt, prev, blk))
        gn = to_np(g)
        inp = np.concatenate([prev.reshape(B, 1), ref["tokens_hi"][:, :L - 1]], axis=1).astype(np.int32)
        err = check_bf16_logits("small step block %d" % blk, gn["logits"], ref["logits"], exact.forward(inp, P).numpy())
        rep = compare_step_with_oracle(gn, ref, err, "small step block %d" % blk)
        say("  small block %d: acc %.3f marked %.3f %r" % (blk, ref["accept"].mean(), ref["mask"].mean(), rep))
        # commit the oracle's tokens on both sides: inputs [prev, out_0 .. out_{L-2}] rewrite rows P .. P+L-1
        commit = np.concatenate([prev.reshape(B, 1), ref["tokens_out"][:, :L - 1]], axis=1).astype(np.int32)
        dec.forward(commit, P)
        exact.forward(commit, P)
        mulo.mulo_verify_forward(ctx, kv, B, L, P, torch.tensor(commit, device=DEV), None, scratch)
        prev = ref["tokens_out"][:, -1].copy()
        P += L


def test_step_expand_two_equals_double_radius_on_device():
    c = dict(WC.get("cfg2"))
    m, B, L, V = c["model"], 2, c["L"], c["model"]["vocab"]
    w = G.make_weights(m, seed=0)
    ctx, _, _ = make_ctx(m, w, 4, c["max_seq"], L)
    kv = mulo.alloc_kv(ctx, DEV)
    dl = G.normal_logits((B, L // 4, V), 2.0, 1)
    dt = G.sample_categorical(dl, 1)
    prev = np.zeros(B, np.int32)
    a = gpu_step(ctx, kv, {**c, "radius": 1, "expand": 2}, 0, 0, dl, dt, prev, 1, want_logits=False)
    b = gpu_step(ctx, kv, {**c, "radius": 2, "expand": 1}, 0, 0, dl, dt, prev, 1, want_logits=False)
    for k in ("tokens_out", "accept", "mask", "t0", "stats"):
        assert torch.equal(a[k], b[k])
    z = gpu_step(ctx, kv, {**c, "radius": 1, "expand": 1}, 0, 0, dl, dt, prev, 1, want_logits=False)
    assert (z["mask"] <= a["mask"]).all() and z["mask"].sum() < a["mask"].sum()


def test_step_argument_errors():
    c = WC.get("cfg1")
    m = c["model"]
    w = G.make_weights(m, seed=0)
    ctx, _, _ = make_ctx(m, w, 1, c["max_seq"], c["L"])
    kv = mulo.alloc_kv(ctx, DEV)
    dl = G.normal_logits((1, 64, m["vocab"]), 2.0, 0)
    dt = G.sample_categorical(dl, 0)
    with pytest.raises(mulo.MuloError) as e:       # h_blk * r * w * r != L
        out = decide_buffers(1, 256)
        params = mulo.make_params(16, 16, 0, 256, 1)
        mulo.mulo_verify_step(ctx, kv, 1, 32, params, 4, 8, 2, torch.tensor(dl, device=DEV), 0, torch.tensor(dt, device=DEV),
                              torch.zeros(1, dtype=torch.int32, device=DEV), out["tokens_out"], out["accept"],
                              out["mask"], out["t0"], out["stats"])
    assert e.value.status == 2
    with pytest.raises(mulo.MuloError) as e:       # block would run past the cache
        out = decide_buffers(1, 256)
        params = mulo.make_params(16, 16, 0, 256, 1)
        mulo.mulo_verify_step(ctx, kv, 1, 64, params, 8, 8, 2, torch.tensor(dl, device=DEV), 0, torch.tensor(dt, device=DEV),
                              torch.zeros(1, dtype=torch.int32, device=DEV), out["tokens_out"], out["accept"],
                              out["mask"], out["t0"], out["stats"])
    assert e.value.status == 2
    assert (out["tokens_out"] == -7).all()          # nothing was written


def test_step_tau_rule_without_draft_distribution_vs_oracle():
    """The paper's own rule through the whole step (Eq. 5 + Alg. 1 Step 6 as a one-shot re-draw from p):
    no draft logits are passed, only the draft tokens."""
    c = WC.get("cfg1")
    m, B, L, Pn, V = c["model"], c["B"], c["L"], c["prefix"], c["model"]["vocab"]
    w = G.make_weights(m, seed=0)
    ctx, cos, sin = make_ctx(m, w, B, c["max_seq"], L)
    kv = mulo.alloc_kv(ctx, DEV)
    dec = OD.DecoderOracle(m, w, cos, sin, B, c["max_seq"], round_bf16=False)
    prefix = G.uniform_tokens((B, Pn), V, 0, tag=0)
    dec.forward(prefix, 0)
    mulo.mulo_verify_forward(ctx, kv, B, Pn, 0, torch.tensor(prefix, device=DEV), None, torch.empty(B, Pn, V, device=DEV))
    dl = G.normal_logits((B, c["h"] * c["w"], V), c["draft_std"], 0, tag=0)
    dt = G.sample_categorical(dl, 0, tag=0)
    tau = 8e-4     # near the median of p(x~) for this random-weight model: both outcomes occur
    ref = ST.verify_step(dec, Pn, dl, dt, prefix[:, -1], h_blk=c["h"], w=c["w"], r=c["r"], W=c["W"], n0=0,
                         radius=c["radius"], expand=c["expand"], seed=0, rng_counter=3, accept_mode=1, tau=tau, mode=2)
    out = decide_buffers(B, L)
    out["tokens_hi"] = torch.empty(B, L, dtype=torch.int32, device=DEV)
    out["logits"] = torch.empty(B, L, V, device=DEV)
    params = mulo.make_params(c["H"], c["W"], 0, L, c["radius"], c["expand"], seed=0, rng_counter=3, resample_mode=2,
                              accept_mode=mulo.MULO_ACCEPT_TAU, tau=tau)
    mulo.mulo_verify_step(ctx, kv, B, Pn, params, c["h"], c["w"], c["r"], None, 0, torch.tensor(dt, device=DEV),
                          torch.tensor(np.ascontiguousarray(prefix[:, -1]), device=DEV), out["tokens_out"],
                          out["accept"], out["mask"], out["t0"], out["stats"], out["tokens_hi"], out["logits"])
    torch.cuda.synchronize()
    g = to_np(out)
    assert np.abs(g["logits"] - ref["logits"]).max() <= 1e-4
    assert np.array_equal(g["tokens_hi"], ref["tokens_hi"])
    # flags may differ only where a logit error of 1e-4 can carry pbar across tau
    rel = np.expm1(2e-4) + 1e-4
    movable = np.abs(ref["pbar"].astype(np.float64) - tau) <= rel * tau
    diff = g["accept"].astype(bool) != ref["accept"].astype(bool)
    assert not (diff & ~movable).any()
    say("  tau step: acc %.3f marked %.3f flips %d movable %d" % (ref["accept"].mean(), ref["mask"].mean(), diff.sum(), movable.sum()))
    assert 0.05 < ref["accept"].mean() < 0.95
    for b in range(B):
        if diff[b].any():
            continue
        assert np.array_equal(g["mask"][b], ref["mask"][b]) and g["t0"][b] == ref["t0"][b]
        assert np.array_equal(g["stats"][b, :3], ref["stats"][b, :3])
        for u in np.flatnonzero(g["tokens_out"][b] != ref["tokens_out"][b]):
            assert ref["mask"][b, u]
            assert RS.boundary_distance(RS.integer_weights(ref["p"][b, u]), ref["words"][b, u]) < 4 * rel
    # and the ratio rule still refuses to run without a draft distribution
    with pytest.raises(mulo.MuloError) as e:
        mulo.mulo_verify_step(ctx, kv, B, Pn, mulo.make_params(c["H"], c["W"], 0, L, c["radius"], c["expand"]), c["h"],
                              c["w"], c["r"], None, 0, torch.tensor(dt, device=DEV),
                              torch.tensor(np.ascontiguousarray(prefix[:, -1]), device=DEV), out["tokens_out"],
                              out["accept"], out["mask"], out["t0"], out["stats"], None, None)
    assert e.value.status == 1


def test_step_with_guidance_equals_its_composition_on_device():
    """Classifier-free guidance through the whole step: the forward runs on 2 B sequences (conditional and
    unconditional caches), the decision stage guides the logits.  The step must equal forward(2B) + decide."""
    c = WC.get("cfg1")
    m, B, L, Pn, V = c["model"], c["B"], c["L"], c["prefix"], c["model"]["vocab"]
    w = G.make_weights(m, seed=0)
    ctx, cos, sin = make_ctx(m, w, 2 * B, c["max_seq"], L)
    kv = mulo.alloc_kv(ctx, DEV)
    prefix = np.concatenate([G.uniform_tokens((B, Pn), V, 0, tag=0), G.uniform_tokens((B, Pn), V, 0, tag=7)], axis=0)   # cond, uncond
    mulo.mulo_verify_forward(ctx, kv, 2 * B, Pn, 0, torch.tensor(prefix, device=DEV), None, torch.empty(2 * B, Pn, V, device=DEV))
    dl = G.normal_logits((B, c["h"] * c["w"], V), c["draft_std"], 0, tag=0)
    dt = G.sample_categorical(dl, 0, tag=0)
    prev = torch.tensor(np.ascontiguousarray(prefix[:B, -1]), device=DEV)
    params = mulo.make_params(c["H"], c["W"], 0, L, c["radius"], c["expand"], seed=0, rng_counter=5, cfg_scale=4.0)
    out = decide_buffers(B, L)
    thi = torch.empty(B, L, dtype=torch.int32, device=DEV)
    lg = torch.empty(2 * B, L, V, device=DEV)
    mulo.mulo_verify_step(ctx, kv, B, Pn, params, c["h"], c["w"], c["r"], torch.tensor(dl, device=DEV), 0,
                          torch.tensor(dt, device=DEV), prev, out["tokens_out"], out["accept"], out["mask"], out["t0"],
                          out["stats"], thi, lg)
    # composition
    q_lo = torch.empty(B, c["h"] * c["w"], V, device=DEV)
    q_row = torch.empty(L, dtype=torch.int32, device=DEV)
    thi2 = torch.empty(B, L, dtype=torch.int32, device=DEV)
    mulo.mulo_upsample_draft(ctx, B, c["h"], c["w"], c["r"], torch.tensor(dl, device=DEV), 0, torch.tensor(dt, device=DEV), thi2, q_lo, q_row, None)
    inp = torch.cat([prev.reshape(B, 1), thi2[:, :L - 1]], dim=1)
    inp2 = torch.cat([inp, inp], dim=0).contiguous()
    lg2 = torch.empty(2 * B, L, V, device=DEV)
    mulo.mulo_verify_forward(ctx, kv, 2 * B, L, Pn, inp2, None, lg2)
    out2 = decide_buffers(B, L)
    mulo.mulo_accept_local_resample(ctx, B, params, lg2, q_lo, q_row, c["h"] * c["w"] * V, thi2, out2["tokens_out"],
                                    out2["accept"], out2["mask"], out2["t0"], out2["stats"], None)
    torch.cuda.synchronize()
    assert torch.equal(lg, lg2) and torch.equal(thi, thi2)
    for k in ("tokens_out", "accept", "mask", "t0", "stats"):
        assert torch.equal(out[k], out2[k]), k
    # and against the oracle's decision stage on the device's own logits
    z = lg.cpu().numpy()
    ref = ST.decide(z[:B], q_lo.cpu().numpy(), q_row.cpu().numpy(), thi.cpu().numpy(), W=c["W"], n0=0, radius=c["radius"],
                    expand=c["expand"], seed=0, rng_counter=5, logits_uncond=z[B:], cfg_scale=4.0)
    from tests.gpu_util import compare_decisions
    rep = compare_decisions(to_np(out), ref, thi.cpu().numpy(), q_lo.cpu().numpy(), q_row.cpu().numpy(), label="guided step")
    say("  guided step: acc %.3f marked %.3f %r" % (ref["accept"].mean(), ref["mask"].mean(), rep))
    assert not np.array_equal(z[:B], z[B:])
