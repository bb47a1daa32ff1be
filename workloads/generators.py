"""Seeded synthetic inputs shared by the oracle-side and the device-side tests
and by the benchmark.  Pure input generation (numpy's Philox bit generator and
torch dtype casts): none of the method's arithmetic lives here.
"""
from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np
import torch

_TENSORS = ["embed", "wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down", "lm_head"]


def _rng(seed, *tags):
    key = int(seed) & 0xFFFFFFFF
    for t in tags:
        key = key * 1000003 + int(t) + 1
    return np.random.Generator(np.random.Philox(key=key & ((1 << 128) - 1)))


def _normal(shape, std, seed, *tags):
    return _rng(seed, *tags).standard_normal(shape, dtype=np.float32) * np.float32(std)


def make_weights(m, seed=0, std=0.02, threads=None):
    """Decoder weights: every matrix ~ N(0, std) (std, not variance), norm gains 1.
    m: model dict (n_layers, d_model, d_ffn, vocab, dtype).  Returns torch CPU
    tensors in the model dtype (bf16 values are the rounded float32 draws):
      embed [V,d], attn_norm/ffn_norm [nl,d], wq/wk/wv/wo [nl,d,d],
      w_gate/w_up [nl,f,d], w_down [nl,d,f], final_norm [d], lm_head [V,d]."""
    nl, d, f, V = m["n_layers"], m["d_model"], m["d_ffn"], m["vocab"]
    tdt = torch.bfloat16 if m["dtype"] == "bf16" else torch.float32
    shapes = dict(embed=(V, d), wq=(nl, d, d), wk=(nl, d, d), wv=(nl, d, d), wo=(nl, d, d),
                  w_gate=(nl, f, d), w_up=(nl, f, d), w_down=(nl, d, f), lm_head=(V, d))
    out = {k: torch.empty(s, dtype=tdt) for k, s in shapes.items()}
    jobs = []
    for ti, name in enumerate(_TENSORS):
        if len(shapes[name]) == 3:
            jobs += [(name, ti, l) for l in range(nl)]
        else:
            jobs.append((name, ti, None))

    def run(job):
        name, ti, l = job
        dst = out[name] if l is None else out[name][l]
        a = _normal(tuple(dst.shape), std, seed, 1, ti, 0 if l is None else l + 1)
        dst.copy_(torch.from_numpy(a))

    n = threads or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(n) as ex:
        list(ex.map(run, jobs))
    out["attn_norm"] = torch.ones(nl, d, dtype=tdt)
    out["ffn_norm"] = torch.ones(nl, d, dtype=tdt)
    out["final_norm"] = torch.ones(d, dtype=tdt)
    return out


def rope_table(max_seq, head_dim, base=10000.0):
    """cos, sin float32 [max_seq, head_dim/2]: angle(pos, m) = pos * base^(-2m/head_dim),
    evaluated in float64 and rounded once."""
    m = np.arange(head_dim // 2, dtype=np.float64)
    theta = base ** (-2.0 * m / head_dim)
    ang = np.arange(max_seq, dtype=np.float64)[:, None] * theta[None, :]
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


def uniform_tokens(shape, V, seed, tag=0):
    return _rng(seed, 2, tag).integers(0, V, size=shape, dtype=np.int64).astype(np.int32)


def normal_logits(shape, std, seed, tag=0):
    """float32 N(0, std) draws (draft logits of configs 1-2, noise of the sigma recipe)."""
    return _normal(shape, std, seed, 3, tag)


def sample_categorical(logits, seed, tag=0):
    """One draw per row of softmax(logits) by the Gumbel-max trick (host side:
    this is how the synthetic drafter 'samples' its tokens)."""
    logits = np.asarray(logits, dtype=np.float64)
    g = _rng(seed, 4, tag).gumbel(size=logits.shape)
    return np.argmax(logits + g, axis=-1).astype(np.int32)


def random_kv(shape, seed, tag=0, dtype=torch.bfloat16, std=1.0, threads=None):
    """Direct fill of cache rows with N(0, std) values (timing and full-size
    parity runs where a real prefill of thousands of rows is too slow on the CPU).
    Generated slice by slice along the first axis (one generator per slice)."""
    out = torch.empty(shape, dtype=dtype)

    def run(i):
        out[i].copy_(torch.from_numpy(_normal(tuple(shape[1:]), std, seed, 5, tag, i)))

    with ThreadPoolExecutor(threads or min(16, os.cpu_count() or 1)) as ex:
        list(ex.map(run, range(shape[0])))
    return out


def neighbour_table(V, k, seed, tag=0):
    """Synthetic codebook-neighbour table int32 [V, k]: nbr[x, 0] = x, the rest
    distinct random other entries (stands in for nearest-neighbour sets of a
    trained VQ codebook, which is not available)."""
    g = _rng(seed, 6, tag)
    nbr = np.empty((V, k), dtype=np.int32)
    for x in range(V):
        others = g.choice(V - 1, size=k - 1, replace=False)
        others = others + (others >= x)
        nbr[x, 0] = x
        nbr[x, 1:] = others
    return nbr
