"""Step 3 of the method (Sec. 3.2; Alg. 1 Step 3): one pass of the target model
M_p over the drafted block, against the cache of the prefix, giving the L
next-token logit vectors.  Test infrastructure; torch CPU ops in float64.

The paper only says the target (AR-DTok) is LlamaGen-based; the architecture is
the pre-norm Llama-style decoder of the workload configs: RMSNorm, multi-head
attention with rotary embedding on adjacent pairs, SwiGLU feed-forward, no
biases, untied lm-head over the image codebook.

    xh = rmsnorm(x, g_attn);  q, k, v = xh Wq^T, xh Wk^T, xh Wv^T
    q, k <- rotary(q), rotary(k) at absolute cache rows P + j;  cache[P + j] = (k, v)
    a_j = sum_{s <= P + j} softmax_s(q_j . k_s / sqrt(d_h)) v_s      per head
    x += a Wo^T
    xh = rmsnorm(x, g_ffn);  x += (silu(xh Wg^T) * (xh Wu^T)) Wd^T
    logits = rmsnorm(x, g_final) Wlm^T

Row j of the result is the distribution of the token that FOLLOWS input j.

Rounding contract of the bf16 configurations (round_bf16=True): weights hold
bf16 values; the tensors the device keeps in bf16 -- the normalised
activations xh, q and k after the rotation, v, the attention output a and the
SwiGLU product -- are rounded to bf16 (nearest-even) at those points, once.
Everything else (residual stream, GEMM accumulation, softmax, norms, logits) is
unrounded float64 here (>= float32 on the device).  With round_bf16=False
nothing is rounded (float32 configuration).
"""
import math

import numpy as np
import torch


def round_to_bf16(x):
    """Round a float64 tensor to the nearest bf16 value (ties to even), staying
    in float64.  Done on the bit pattern so there is a single rounding (not
    float64 -> float32 -> bf16).  Valid for magnitudes in bf16's normal range."""
    assert x.dtype == torch.float64
    bits = x.contiguous().view(torch.int64)
    drop = 45                                    # 52 - 7 mantissa bits kept
    lsb = (bits >> drop) & 1
    bits = bits + ((1 << (drop - 1)) - 1) + lsb
    bits = bits & ~((1 << drop) - 1)
    return bits.view(torch.float64)


def rmsnorm(x, g, eps):
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    ms = (x * x).mean(dim=-1, keepdim=True)
    return x / torch.sqrt(ms + eps) * g


def rotary(t, cos, sin):
    """Adjacent-pair rotation: (t[2m], t[2m+1]) <- (t[2m] c - t[2m+1] s, t[2m] s + t[2m+1] c).
    t: [B, L, n_h, d_h]; cos, sin: [L, d_h/2] for the L absolute positions."""
    te, to = t[..., 0::2], t[..., 1::2]
    c = cos[None, :, None, :]
    s = sin[None, :, None, :]
    out = torch.empty_like(t)
    out[..., 0::2] = te * c - to * s
    out[..., 1::2] = te * s + to * c
    return out


def silu(t):
    return t / (1.0 + torch.exp(-t))


class DecoderOracle:
    """Holds weights (torch tensors, any float dtype; converted to float64 per
    use), the rotary table and its own KV cache [n_layers, B, S, n_h, d_h]."""

    def __init__(self, cfg, weights, rope_cos, rope_sin, max_batch, max_seq, round_bf16):
        self.cfg = dict(cfg)
        self.w = weights
        self.rb = round_to_bf16 if round_bf16 else (lambda t: t)
        self.cos = torch.as_tensor(np.asarray(rope_cos)).to(torch.float64)
        self.sin = torch.as_tensor(np.asarray(rope_sin)).to(torch.float64)
        nl, nh, dh = cfg["n_layers"], cfg["n_heads"], cfg["head_dim"]
        cdt = torch.float32 if round_bf16 else torch.float64     # float32 holds bf16 values exactly
        self.k = torch.zeros(nl, max_batch, max_seq, nh, dh, dtype=cdt)
        self.v = torch.zeros(nl, max_batch, max_seq, nh, dh, dtype=cdt)

    def _w(self, name, layer=None):
        t = self.w[name]
        if layer is not None:
            t = t[layer]
        return t.to(torch.float64)

    @torch.no_grad()
    def forward(self, tokens, P, embeds=None, taps=None, stages=None):
        """tokens: int [B, L]; P: number of valid cache rows; writes cache rows
        P .. P+L-1; returns float64 logits [B, L, V].  taps: optional list that
        receives a copy of the residual stream entering every layer.  stages:
        optional dict that receives, per layer (appended to lists), the tensors
        the device keeps between its kernels: "q" rotated queries [B, L, n_h, d_h],
        "att" attention output [B, L, d], "hmid" SwiGLU product [B, L, f] (each after
        its rounding point) and "x_out" the residual stream leaving the layer."""
        cfg = self.cfg
        nl, d, nh, dh = cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["head_dim"]
        eps = cfg.get("rms_eps", 1e-5)
        tok = torch.as_tensor(np.asarray(tokens)).long()
        B, L = tok.shape
        S = P + L
        if embeds is None:
            x = self._w("embed")[tok]                               # [B, L, d]
        else:
            x = torch.as_tensor(np.asarray(embeds)).to(torch.float64).reshape(B, L, d).clone()
        cos, sin = self.cos[P:S], self.sin[P:S]
        pos_q = torch.arange(P, S)[:, None]
        visible = torch.arange(S)[None, :] <= pos_q                  # key s visible to query j iff s <= P + j
        for l in range(nl):
            if taps is not None:
                taps.append(x.clone())
            xh = self.rb(rmsnorm(x, self._w("attn_norm", l), eps))
            q = (xh @ self._w("wq", l).T).reshape(B, L, nh, dh)
            k = (xh @ self._w("wk", l).T).reshape(B, L, nh, dh)
            v = (xh @ self._w("wv", l).T).reshape(B, L, nh, dh)
            q = self.rb(rotary(q, cos, sin))
            k = self.rb(rotary(k, cos, sin))
            v = self.rb(v)
            self.k[l, :B, P:S] = k.to(self.k.dtype)
            self.v[l, :B, P:S] = v.to(self.v.dtype)
            K = self.k[l, :B, :S].to(torch.float64).permute(0, 2, 1, 3)   # [B, nh, S, dh]
            Vv = self.v[l, :B, :S].to(torch.float64).permute(0, 2, 1, 3)
            s = (q.permute(0, 2, 1, 3) @ K.transpose(-1, -2)) / math.sqrt(dh)   # [B, nh, L, S]
            s = s.masked_fill(~visible[None, None], float("-inf"))
            s = s - s.max(dim=-1, keepdim=True).values
            e = torch.exp(s)
            a = (e / e.sum(dim=-1, keepdim=True)) @ Vv                    # [B, nh, L, dh]
            a = self.rb(a.permute(0, 2, 1, 3).reshape(B, L, d))
            x = x + a @ self._w("wo", l).T
            xh = self.rb(rmsnorm(x, self._w("ffn_norm", l), eps))
            hmid = self.rb(silu(xh @ self._w("w_gate", l).T) * (xh @ self._w("w_up", l).T))
            x = x + hmid @ self._w("w_down", l).T
            if stages is not None:
                for name, t in (("q", q), ("att", a), ("hmid", hmid), ("x_out", x)):
                    stages.setdefault(name, []).append(t.clone())
        xh = self.rb(rmsnorm(x, self._w("final_norm"), eps))
        return xh @ self._w("lm_head").T

    @torch.no_grad()
    def forward_at(self, tokens, seq, pos, visible):
        """One pass of M_p over single-token queries at scattered cache rows (island-parallel re-sampling,
        Sec. 3.4: positions of different rejection islands are evaluated concurrently).

        tokens: int [n] input token of each query; seq: int [n] the cache sequence it belongs to; pos: int [n]
        its cache row (its rotary position); visible: bool [n, S], S > max(pos): the cache rows query i attends
        to (row pos[i] itself must be among them).  At every layer all queries first write their own k, v to
        cache row (seq[i], pos[i]), then each attends to its visible rows of its sequence.  Returns float64
        logits [n, V]: row i is the distribution of the token at block position pos[i] + 1 - (rows before the
        block), i.e. of the token that follows input i."""
        cfg = self.cfg
        nl, d, nh, dh = cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["head_dim"]
        eps = cfg.get("rms_eps", 1e-5)
        tok = torch.as_tensor(np.asarray(tokens)).long().reshape(-1)
        seq = [int(b) for b in np.asarray(seq).reshape(-1)]
        pos = [int(r) for r in np.asarray(pos).reshape(-1)]
        vis = torch.as_tensor(np.asarray(visible)).bool()
        n, S = vis.shape
        assert len(seq) == n and len(pos) == n and all(vis[i, pos[i]] for i in range(n))
        x = self._w("embed")[tok]                                           # [n, d]
        cos, sin = self.cos[pos], self.sin[pos]                             # [n, dh/2]
        for l in range(nl):
            xh = self.rb(rmsnorm(x, self._w("attn_norm", l), eps))
            q = (xh @ self._w("wq", l).T).reshape(1, n, nh, dh)
            k = (xh @ self._w("wk", l).T).reshape(1, n, nh, dh)
            v = (xh @ self._w("wv", l).T).reshape(n, nh, dh)
            q = self.rb(rotary(q, cos, sin))[0]
            k = self.rb(rotary(k, cos, sin))[0]
            v = self.rb(v)
            for i in range(n):
                self.k[l, seq[i], pos[i]] = k[i].to(self.k.dtype)
                self.v[l, seq[i], pos[i]] = v[i].to(self.v.dtype)
            a = torch.empty(n, nh, dh, dtype=torch.float64)
            for i in range(n):
                K = self.k[l, seq[i], :S].to(torch.float64)                 # [S, nh, dh]
                Vv = self.v[l, seq[i], :S].to(torch.float64)
                s = torch.einsum("hc,shc->hs", q[i], K) / math.sqrt(dh)     # [nh, S]
                s = s.masked_fill(~vis[i][None, :], float("-inf"))
                s = s - s.max(dim=-1, keepdim=True).values
                e = torch.exp(s)
                a[i] = torch.einsum("hs,shc->hc", e / e.sum(dim=-1, keepdim=True), Vv)
            a = self.rb(a.reshape(n, d))
            x = x + a @ self._w("wo", l).T
            xh = self.rb(rmsnorm(x, self._w("ffn_norm", l), eps))
            hmid = self.rb(silu(xh @ self._w("w_gate", l).T) * (xh @ self._w("w_up", l).T))
            x = x + hmid @ self._w("w_down", l).T
        xh = self.rb(rmsnorm(x, self._w("final_norm"), eps))
        return xh @ self._w("lm_head").T
