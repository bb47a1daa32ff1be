"""Shared, cached 7B-class reference cases of the GPU parity tests (the oracle's 32-layer float64 passes cost
minutes, so the tests that need the same pass share it).  Everything here is seeded input generation and calls of
`oracle/`; nothing comes from the device."""
import numpy as np
import torch

from oracle import decoder as OD
from oracle import upsample as UP
from tests.gpu_util import say
from workloads import configs as WC
from workloads import generators as G

_CACHE = {}


def weights_7b():
    if "w" not in _CACHE:
        say("generating 7B-class weights on the host ...")
        _CACHE["w"] = G.make_weights(WC.model("7b"), seed=0)
        say("... done")
    return _CACHE["w"]


def seeded_cache_rows(m, P, b):
    """K and V rows [0, P) of batch element b, [n_layers, n_heads, P, d_h] bf16 N(0, 1) (the stand-in for a prefill
    of thousands of rows, which is hours of oracle time)."""
    nl, nh, dh = m["n_layers"], m["n_heads"], m["head_dim"]
    return (G.random_kv((nl, nh, P, dh), seed=0, tag=2 * b), G.random_kv((nl, nh, P, dh), seed=0, tag=2 * b + 1))


def fill_oracle_cache(dec, b, kb, vb, P):
    dec.k[:, b, :P] = kb.permute(0, 2, 1, 3).to(dec.k.dtype)
    dec.v[:, b, :P] = vb.permute(0, 2, 1, 3).to(dec.v.dtype)


def provisional_inputs(c, B, tag):
    """The sigma recipe's first step: a uniform low-resolution draft of the block, up-sampled, and the target's
    inputs [prev, x~_0 .. x~_{L-2}] for it."""
    V, L = c["model"]["vocab"], c["L"]
    h_blk = L // c["W"] // c["r"]
    y = G.uniform_tokens((B, h_blk * c["w"]), V, 0, tag=tag)
    x_hi = UP.upsample_draft(np.zeros((B, h_blk * c["w"], 1)), y, h_blk, c["w"], c["r"], input_is_probs=True)[0]
    prev = G.uniform_tokens((B,), V, 0, tag=tag + 1)
    return np.concatenate([prev.reshape(B, 1), x_hi[:, :L - 1]], axis=1).astype(np.int32), prev


def draft_from_target_logits(c, z_p, sigma, tag):
    """The recipe's remaining steps on ORACLE logits z_p [B, L, V] of the provisional pass: draft logits of a
    low-resolution cell = target logits of its top-left child + sigma * N(0, 1); draft tokens ~ softmax."""
    B, L, V = z_p.shape
    r, h_blk = c["r"], L // c["W"] // c["r"]
    child0 = (np.arange(h_blk)[:, None] * r * c["W"] + np.arange(c["w"])[None, :] * r).reshape(-1)
    dl = (z_p[:, child0, :] + sigma * G.normal_logits((B, h_blk * c["w"], V), 1.0, 0, tag=tag)).astype(np.float32)
    return np.ascontiguousarray(dl), G.sample_categorical(dl, 0, tag=tag)


def hires_case():
    """Config-4 shape, batch element 0: L = 1024 provisional inputs against P = 3200 seeded cache rows; the
    oracle's rounded and exact logits, the residual stream entering every layer (rounded pass), and the inputs."""
    if "hires" in _CACHE:
        return _CACHE["hires"]
    c = WC.get("cfg4")
    m, B, L = c["model"], c["B"], c["L"]
    P = c["max_seq"] - L
    w = weights_7b()
    cos, sin = G.rope_table(c["max_seq"], m["head_dim"])
    inp, prev = provisional_inputs(c, B, tag=3)
    kb, vb = seeded_cache_rows(m, P, 0)
    dr = OD.DecoderOracle(m, w, cos, sin, 1, c["max_seq"], round_bf16=True)
    du = OD.DecoderOracle(m, w, cos, sin, 1, c["max_seq"], round_bf16=False)
    fill_oracle_cache(dr, 0, kb, vb, P)
    fill_oracle_cache(du, 0, kb, vb, P)
    say("7B hi-res block, oracle (rounded, then exact) on batch element 0 ...")
    taps = []
    z_r = dr.forward(inp[:1], P, taps=taps).numpy()
    z_u = du.forward(inp[:1], P).numpy()
    del du
    _CACHE["hires"] = dict(c=c, P=P, inp=inp, prev=prev, z_r=z_r, z_u=z_u, taps=taps, kb=kb, vb=vb, dr=dr, cos=cos, sin=sin)
    return _CACHE["hires"]
