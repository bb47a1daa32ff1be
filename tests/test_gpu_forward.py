"""GPU parity of the target forward (Alg. 1 Step 3) against the CPU oracle,
through the C ABI.

float32 configuration: max |logit error| <= 1e-4.
bf16 configurations: the oracle rounds to bf16 at the same tensor boundaries as
the device; every pass is held to the oracle's own rounding noise (see
tests.gpu_util.check_bf16_logits): bf16 rounding makes the forward chaotic, and
the stated max |logit error| <= 2e-2 lies below that noise except for shallow
models at the small width, where it is asserted as well."""
import numpy as np
import pytest
import torch

import paper_2601_05149_amd as mulo
from oracle import decoder as OD
from tests.gpu_util import (DEV, check_bf16_logits, dev, device_weights, make_ctx, make_ctx_from_device, say)
from workloads import configs as WC
from workloads import generators as G

pytestmark = pytest.mark.gpu

from tests.cases_7b import hires_case, seeded_cache_rows, weights_7b  # noqa: E402


def gpu_forward(ctx, kv, tokens, P, embeds=None):
    B, L = tokens.shape
    logits = torch.empty(B, L, ctx.cfg.vocab, device=DEV)
    mulo.mulo_verify_forward(ctx, kv, B, L, P, dev(tokens), embeds, logits)
    torch.cuda.synchronize()
    return logits.cpu().numpy()


def cache_error(dec, kv, B, rows):
    """|device cache - oracle cache| over rows [0, rows), in the oracle's layout."""
    k = kv[0].float().cpu().permute(0, 1, 3, 2, 4)[:, :B, :rows]      # -> [nl, B, S, nh, dh]
    v = kv[1].float().cpu().permute(0, 1, 4, 2, 3)[:, :B, :rows]
    ek = (k.double() - dec.k[:, :B, :rows].double()).abs()
    ev = (v.double() - dec.v[:, :B, :rows].double()).abs()
    return ek, ev


def pair(m, w, cos, sin, B, S):
    return (OD.DecoderOracle(m, w, cos, sin, B, S, round_bf16=True),
            OD.DecoderOracle(m, w, cos, sin, B, S, round_bf16=False))


def test_forward_tiny_f32():
    c = WC.get("cfg1")
    m, B, L, Pn = c["model"], c["B"], c["L"], c["prefix"]
    w = G.make_weights(m, seed=0)
    ctx, cos, sin = make_ctx(m, w, B, c["max_seq"] + 8, L)
    kv = mulo.alloc_kv(ctx, DEV)
    dec = OD.DecoderOracle(m, w, cos, sin, B, c["max_seq"] + 8, round_bf16=False)
    prefix = G.uniform_tokens((B, Pn), m["vocab"], 0, tag=0)
    block = G.uniform_tokens((B, L), m["vocab"], 0, tag=1)
    for tag, toks, P in (("tiny prefill", prefix, 0), ("tiny block", block, Pn)):
        err = np.abs(gpu_forward(ctx, kv, toks, P) - dec.forward(toks, P).numpy()).max()
        say("  %s: max|err| %.3g (tol 1e-4)" % (tag, err))
        assert err <= 1e-4
    ek, ev = cache_error(dec, kv, B, Pn + L)
    assert ek.max() < 1e-5 and ev.max() < 1e-5
    assert kv[0][:, :, :, Pn + L:].abs().max() == 0 and kv[1][:, :, :, :, Pn + L:].abs().max() == 0
    # token-by-token passes give the block pass (causality), on the device
    kv2 = mulo.alloc_kv(ctx, DEV)
    gpu_forward(ctx, kv2, prefix, 0)
    seq = np.concatenate([gpu_forward(ctx, kv2, block[:, j:j + 1], Pn + j) for j in range(24)], axis=1)
    blk = gpu_forward(ctx, kv, block, Pn)
    assert np.abs(seq - blk[:, :24]).max() < 1e-4


def test_forward_small_bf16_chained_blocks():
    c = WC.get("cfg2")
    m, B, L, Pn = c["model"], c["B"], c["L"], c["prefix"]
    w = G.make_weights(m, seed=0)
    ctx, cos, sin = make_ctx(m, w, B, c["max_seq"], L)
    kv = mulo.alloc_kv(ctx, DEV)
    dr, du = pair(m, w, cos, sin, B, c["max_seq"])
    prefix = G.uniform_tokens((B, Pn), m["vocab"], 0, tag=0)
    check_bf16_logits("small prefill", gpu_forward(ctx, kv, prefix, 0), dr.forward(prefix, 0).numpy(),
                      du.forward(prefix, 0).numpy())
    P = Pn
    for blk in range(3):                                    # cache append at n0 = 0, 256, 512
        toks = G.uniform_tokens((B, L), m["vocab"], 0, tag=10 + blk)
        check_bf16_logits("small block %d (P=%d)" % (blk, P), gpu_forward(ctx, kv, toks, P),
                          dr.forward(toks, P).numpy(), du.forward(toks, P).numpy())
        P += L
    ek, ev = cache_error(dr, kv, B, P)
    # layer 0 sees identical inputs on both sides: its cache rows agree up to rare one-ulp bf16 flips
    # (a flipped input element moves every output of its row by a little, hence the absolute part)
    tol_k = 2.0 ** -6 * (dr.k[0, :B, :P].double().abs() + 0.1)
    tol_v = 2.0 ** -6 * (dr.v[0, :B, :P].double().abs() + 0.1)
    say("  layer-0 cache: K mismatching %.4f%% (max %.3g, beyond tol %d)  V mismatching %.4f%% (max %.3g, beyond tol %d)" % (
        100 * (ek[0] > 0).double().mean(), ek[0].max(), int((ek[0] > tol_k).sum()),
        100 * (ev[0] > 0).double().mean(), ev[0].max(), int((ev[0] > tol_v).sum())))
    for name, e_, t_ in (("K", ek[0], tol_k), ("V", ev[0], tol_v)):
        bad = (e_ > t_).nonzero()
        if len(bad):
            say("  %s violations at [b, row, head, c]: %r" % (name, bad[:8].tolist()))
    assert (ek[0] <= tol_k).all() and (ev[0] <= tol_v).all()
    assert (ek[0] > 0).double().mean() < 0.01 and (ev[0] > 0).double().mean() < 0.01
    # deeper layers drift with the format's noise but stay close
    assert ek.max() < 0.25 and ev.max() < 0.25


def test_forward_single_layer_bf16():
    """One decoder layer + lm-head at the small and at the 7B-class width.  At
    the small width the stated 2e-2 holds; at the 7B width one layer's own
    rounding noise already exceeds it (logit std 1.28)."""
    for name, L, P in (("small", 256, 64), ("7b", 192, 64)):
        m = dict(WC.model(name), n_layers=1)
        w = G.make_weights(m, seed=3)
        S = P + L
        ctx, cos, sin = make_ctx(m, w, 2, S, L)
        kv = mulo.alloc_kv(ctx, DEV)
        dr, du = pair(m, w, cos, sin, 2, S)
        pre = G.uniform_tokens((2, P), m["vocab"], 3, tag=0)
        blk = G.uniform_tokens((2, L), m["vocab"], 3, tag=1)
        gpu_forward(ctx, kv, pre, 0)
        dr.forward(pre, 0)
        du.forward(pre, 0)
        check_bf16_logits("1-layer %s" % name, gpu_forward(ctx, kv, blk, P), dr.forward(blk, P).numpy(),
                          du.forward(blk, P).numpy(), strict=(name == "small"))


def test_forward_ragged_shapes_bf16():
    # M = 300 (not a tile multiple), vocabulary 1000 (ragged last column tile), odd prefix length
    m = dict(n_layers=2, d_model=256, n_heads=4, head_dim=64, d_ffn=320, vocab=1000, dtype="bf16", rms_eps=1e-5)
    B, L, Pn, S = 3, 100, 37, 144
    w = G.make_weights(m, seed=5, std=0.05)
    ctx, cos, sin = make_ctx(m, w, B, S, L)
    kv = mulo.alloc_kv(ctx, DEV, zero=False)
    kv[0].fill_(float("nan"))                               # rows not yet written must never be used
    kv[1].fill_(float("nan"))
    dr, du = pair(m, w, cos, sin, B, S)
    prefix = G.uniform_tokens((B, Pn), m["vocab"], 5, tag=0)
    block = G.uniform_tokens((B, L), m["vocab"], 5, tag=1)
    check_bf16_logits("ragged prefill", gpu_forward(ctx, kv, prefix, 0), dr.forward(prefix, 0).numpy(),
                      du.forward(prefix, 0).numpy())
    check_bf16_logits("ragged block", gpu_forward(ctx, kv, block, Pn), dr.forward(block, Pn).numpy(),
                      du.forward(block, Pn).numpy())
    # head_dim 128 variant with a single short block
    m2 = dict(n_layers=1, d_model=256, n_heads=2, head_dim=128, d_ffn=192, vocab=512, dtype="bf16", rms_eps=1e-5)
    w2 = G.make_weights(m2, seed=6, std=0.05)
    ctx2, cos2, sin2 = make_ctx(m2, w2, 2, 80, 72)
    kv2 = mulo.alloc_kv(ctx2, DEV)
    d2r, d2u = pair(m2, w2, cos2, sin2, 2, 80)
    t2 = G.uniform_tokens((2, 72), 512, 6)
    check_bf16_logits("dh128 block", gpu_forward(ctx2, kv2, t2, 0), d2r.forward(t2, 0).numpy(),
                      d2u.forward(t2, 0).numpy())


def test_forward_embeds_input_and_errors():
    m = dict(n_layers=1, d_model=128, n_heads=2, head_dim=64, d_ffn=128, vocab=256, dtype="bf16", rms_eps=1e-5)
    w = G.make_weights(m, seed=7, std=0.05)
    ctx, cos, sin = make_ctx(m, w, 2, 64, 32)
    kv = mulo.alloc_kv(ctx, DEV)
    toks = G.uniform_tokens((2, 32), 256, 7)
    a = gpu_forward(ctx, kv, toks, 0)
    emb = w["embed"][torch.as_tensor(toks).long()].to(DEV).contiguous()
    b = gpu_forward(ctx, kv, toks * 0, 0, embeds=emb)
    assert np.array_equal(a, b)
    for bad in [dict(B=3, L=32, P=0), dict(B=2, L=40, P=0), dict(B=2, L=32, P=40)]:
        with pytest.raises(mulo.MuloError) as e:
            mulo.mulo_verify_forward(ctx, kv, bad["B"], bad["L"], bad["P"], torch.zeros(3, 40, dtype=torch.int32, device=DEV),
                                     None, torch.empty(3, 40, 256, device=DEV))
        assert e.value.status == 2


@pytest.mark.timeout(900)
def test_forward_7b_first_block_and_teacher_forced_layers():
    """7B-class decoder, batch 1: real prefill of the 128-token prefix, then the
    first 576-token block (M = 576 is not a multiple of the 128/256 tiles); then
    layers 0, 15 and 31 alone, each fed the oracle's hidden state entering it."""
    c = WC.get("cfg3")
    m, B, L, Pn = c["model"], c["B"], c["L"], c["prefix"]
    w = weights_7b()
    ctx, cos, sin = make_ctx(m, w, B, c["max_seq"], L)
    kv = mulo.alloc_kv(ctx, DEV)
    dr, du = pair(m, w, cos, sin, B, Pn + L)
    prefix = G.uniform_tokens((B, Pn), m["vocab"], 0, tag=0)
    block = G.uniform_tokens((B, L), m["vocab"], 0, tag=1)
    say("7B prefill (oracle, rounded + exact) ...")
    check_bf16_logits("7B prefill", gpu_forward(ctx, kv, prefix, 0), dr.forward(prefix, 0).numpy(),
                      du.forward(prefix, 0).numpy())
    say("7B block (oracle, rounded + exact) ...")
    taps = []
    zr = dr.forward(block, Pn, taps=taps).numpy()
    check_bf16_logits("7B block", gpu_forward(ctx, kv, block, Pn), zr, du.forward(block, Pn).numpy())
    del ctx, kv
    wd = device_weights(w)
    m1 = dict(m, n_layers=1)
    for l in (0, 15, 31):
        sl = lambda t: t[l:l + 1] if t.dim() == 3 or (t.dim() == 2 and t.shape[0] == m["n_layers"]) else t
        w1 = {k: sl(v) for k, v in w.items()}
        wd1 = {k: sl(v) for k, v in wd.items()}
        x_in = taps[l].to(torch.bfloat16)                       # hidden state entering layer l, as the bf16 input
        ctx1, cos1, sin1 = make_ctx_from_device(m1, wd1, B, L, L)
        kv1 = mulo.alloc_kv(ctx1, DEV)
        d1r, d1u = pair(m1, w1, cos1, sin1, B, L)
        zg = gpu_forward(ctx1, kv1, block * 0, 0, embeds=x_in.to(DEV).contiguous())
        emb = x_in.double().numpy()
        check_bf16_logits("7B layer %d teacher-forced" % l, zg, d1r.forward(block * 0, 0, embeds=emb).numpy(),
                          d1u.forward(block * 0, 0, embeds=emb).numpy())
        del ctx1, kv1


def fill_device_cache(kv, m, P, B):
    """Seeded N(0, 1) rows [0, P) of every batch element, as tests.cases_7b.seeded_cache_rows makes them."""
    for b in range(B):
        kb, vb = seeded_cache_rows(m, P, b)                                  # [nl, nh, P, dh]
        kv[0][:, b, :, :P] = kb.to(DEV)
        kv[1][:, b, :, :, :P] = vb.permute(0, 1, 3, 2).to(DEV)


@pytest.mark.timeout(900)
def test_forward_7b_hires_full_launch_sampled_sequence():
    """Config-4 launch (B = 4, L = 1024, P = 3200: the largest cache) on the
    device; the oracle recomputes batch element 0 in full.  Cache rows [0, P) are
    seeded N(0, 1) values on both sides (a real prefill of 3200 rows is hours of
    CPU time); the inputs are the sigma recipe's provisional up-sampled draft."""
    h = hires_case()
    c, P, toks = h["c"], h["P"], h["inp"]
    m, B, L = c["model"], c["B"], c["L"]
    w = weights_7b()
    ctx, cos, sin = make_ctx(m, w, B, c["max_seq"], L)
    kv = mulo.alloc_kv(ctx, DEV)
    fill_device_cache(kv, m, P, B)
    zg = gpu_forward(ctx, kv, toks, P)
    check_bf16_logits("7B hi-res b=0", zg[:1], h["z_r"], h["z_u"])
    say("  logits above 2e-2 of the oracle's: %d of %d" % (int((np.abs(zg[:1] - h["z_r"]) > 2e-2).sum()), h["z_r"].size))
    # batch elements are independent: element 3 alone reproduces its rows of the batched launch
    kv1 = (kv[0][:, 3:4].contiguous(), kv[1][:, 3:4].contiguous())
    ctx1, _, _ = make_ctx(m, w, 1, c["max_seq"], L)
    z3 = gpu_forward(ctx1, kv1, toks[3:4], P)
    say("  batch element 3 alone vs in the batch: max diff %.3g" % np.abs(z3 - zg[3:4]).max())
    assert np.abs(z3 - zg[3:4]).max() <= 1e-3
    del ctx, ctx1


@pytest.mark.parametrize("dh,nh,copy", [(64, 4, False), (128, 2, False), (128, 2, True)])
def test_forward_single_token_steps_with_split_keys(dh, nh, copy):
    """Decode shape: one token per sequence against a cache of several key tiles, so that the keys are dealt
    to several workgroups per head and combined (and the projections run in the weight-streaming kernel).
    Cache lengths 199 .. 202 straddle a tile boundary (64-key tiles, the last one partly filled)."""
    m = dict(n_layers=2, d_model=dh * nh, n_heads=nh, head_dim=dh, d_ffn=512, vocab=1024, dtype="bf16", rms_eps=1e-5)
    B, Pn = 3, 199
    w = G.make_weights(m, seed=5)
    ctx, cos, sin = make_ctx(m, w, B, 208, 200, stream_copy=copy)   # copy: the weights once more in fragment order
    kv = mulo.alloc_kv(ctx, DEV)
    dr, du = pair(m, w, cos, sin, B, 208)
    pre = G.uniform_tokens((B, Pn), m["vocab"], 5, tag=0)
    gpu_forward(ctx, kv, pre, 0)
    dr.forward(pre, 0)
    du.forward(pre, 0)
    for step in range(4):
        t = G.uniform_tokens((B, 1), m["vocab"], 5, tag=10 + step)
        check_bf16_logits("single token, %d cached rows, dh %d" % (Pn + step, dh), gpu_forward(ctx, kv, t, Pn + step),
                          dr.forward(t, Pn + step).numpy(), du.forward(t, Pn + step).numpy(), strict=True)


def frag_to_rows(buf, M, K):
    """Undo the fragment order of a [M, K] token operand (include/mulo.h, mulo_workspace_read): element (m, k)
    sits at ((m / 16) * (K / 32) + k / 32) * 512 + ((k % 32) / 8 * 16 + m % 16) * 8 + k % 8."""
    m = np.arange(M)[:, None]
    k = np.arange(K)[None, :]
    idx = ((m // 16) * (K // 32) + k // 32) * 512 + ((k % 32) // 8 * 16 + m % 16) * 8 + k % 8
    return buf.reshape(-1)[idx]


@pytest.mark.parametrize("B,L,copy", [(3, 1, False), (4, 13, False), (2, 32, False), (3, 1, True), (4, 13, True),
                                      (4, 40, True), (2, 100, True)])
def test_forward_few_tokens_keeps_its_operands_in_fragment_order(B, L, copy):
    """Launches of at most 64 tokens (one, four and four token groups of 16; 3, 52 and 64 tokens) run every projection
    in the weight-streaming kernel, whose token operand the producing kernels leave in the matrix instruction's own
    order; with the context's weight copy in fragment order so do launches of up to 256 tokens (160 and 200 here: the
    kernel that shares the token operand through LDS and deals K to several workgroups).  One layer: the attention output and silu(gate) * up read back through mulo_workspace_read, put back in
    row order by the documented formula, are the oracle's stage tensors; the logits are held to the usual bound."""
    m = dict(n_layers=1, d_model=256, n_heads=2, head_dim=128, d_ffn=512, vocab=1024, dtype="bf16", rms_eps=1e-5)
    Pn, S, M = 70, 184, B * L
    w = G.make_weights(m, seed=11)
    ctx, cos, sin = make_ctx(m, w, B, S, 104, stream_copy=copy)
    kv = mulo.alloc_kv(ctx, DEV)
    dr, du = pair(m, w, cos, sin, B, S)
    pre = G.uniform_tokens((B, Pn), m["vocab"], 11, tag=0)
    gpu_forward(ctx, kv, pre, 0)
    dr.forward(pre, 0)
    du.forward(pre, 0)
    blk = G.uniform_tokens((B, L), m["vocab"], 11, tag=1)
    stages = {}
    z_r = dr.forward(blk, Pn, stages=stages).numpy()
    z = gpu_forward(ctx, kv, blk, Pn)
    check_bf16_logits("%d x %d tokens, weight-streaming projections" % (B, L), z, z_r, du.forward(blk, Pn).numpy(), strict=True)
    M16 = (M + 15) // 16 * 16
    for name, which, K in (("att", mulo.MULO_WS_ATTN, m["d_model"]), ("hmid", mulo.MULO_WS_FFN, m["d_ffn"])):
        buf = torch.empty(M16 * K, dtype=torch.bfloat16, device=DEV)
        mulo.mulo_workspace_read(ctx, which, buf)
        torch.cuda.synchronize()
        got = frag_to_rows(buf.float().cpu().numpy(), M, K)
        want = stages[name][0].reshape(M, K).double().numpy()
        err = np.abs(got - want)
        tol = 2.0 ** -5 * (np.abs(want) + np.sqrt((want ** 2).mean()))
        say("  %s in fragment order, %d tokens: max|err| %.3g, beyond tolerance %d of %d" % (name, M, err.max(), (err > tol).sum(), err.size))
        assert (err > tol).mean() <= 0.005 and err.max() <= 0.25 * np.abs(want).max()
