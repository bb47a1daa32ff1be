"""mulo_verify_step under HIP graph capture: the step enqueues kernels only (no allocation, no host
synchronisation, no memset node), so a caller may record it once on the context's stream and replay it.
Every replay, with other inputs in the same buffers and eager library work between the replays, must
reproduce the eager call bit for bit."""
import numpy as np
import pytest
import torch

import paper_2601_05149_amd as mulo
from tests.gpu_util import DEV, decide_buffers, make_ctx, say
from workloads import configs as WC
from workloads import generators as G

pytestmark = pytest.mark.gpu

KEYS = ("tokens_out", "accept", "mask", "t0", "stats", "tokens_hi", "logits")


def test_verify_step_captured_once_replays_bit_for_bit():
    c = WC.get("cfg2")
    m, B, L, Pn, V = c["model"], c["B"], c["L"], c["prefix"], c["model"]["vocab"]
    n_lo, h_blk = (L // c["W"] // c["r"]) * c["w"], L // c["W"] // c["r"]
    w = G.make_weights(m, seed=0)
    side = torch.cuda.Stream()          # default priority; the context launches on it
    with torch.cuda.stream(side):
        ctx, _, _ = make_ctx(m, w, B, c["max_seq"], L)
        kv = mulo.alloc_kv(ctx, DEV)
        prefix = G.uniform_tokens((B, Pn), V, 0, tag=0)
        mulo.mulo_verify_forward(ctx, kv, B, Pn, 0, torch.tensor(prefix, device=DEV), None,
                                 torch.empty(B, Pn, V, device=DEV))
        # the buffers the recorded call reads and writes
        dl = torch.empty(B, n_lo, V, device=DEV)
        dt = torch.empty(B, n_lo, dtype=torch.int32, device=DEV)
        prev = torch.empty(B, dtype=torch.int32, device=DEV)
        out = decide_buffers(B, L)
        out["tokens_hi"] = torch.empty(B, L, dtype=torch.int32, device=DEV)
        out["logits"] = torch.empty(B, L, V, device=DEV)
        params = mulo.make_params(c["H"], c["W"], 0, L, c["radius"], c["expand"], seed=3, rng_counter=11)

        def step():
            mulo.mulo_verify_step(ctx, kv, B, Pn, params, h_blk, c["w"], c["r"], dl, 0, dt, prev, out["tokens_out"],
                                  out["accept"], out["mask"], out["t0"], out["stats"], out["tokens_hi"], out["logits"])

        inputs = []
        for i in range(3):
            dli = G.normal_logits((B, n_lo, V), c["draft_std"], 0, tag=20 + i)
            inputs.append((torch.tensor(dli, device=DEV), torch.tensor(G.sample_categorical(dli, 0, tag=20 + i), device=DEV),
                           torch.tensor(G.uniform_tokens((B,), V, 0, tag=30 + i), device=DEV)))

        def load(i):
            dl.copy_(inputs[i][0]); dt.copy_(inputs[i][1]); prev.copy_(inputs[i][2])
            for k in KEYS:
                out[k].fill_(7)

        eager = []
        for i in range(3):              # eager results (the first call also configures every kernel)
            load(i)
            step()
            side.synchronize()
            eager.append({k: out[k].clone() for k in KEYS})
        assert not torch.equal(eager[0]["tokens_out"], eager[1]["tokens_out"])
        side.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    # other buffers for the eager work between the replays
    other = decide_buffers(B, L)
    o_thi = torch.empty(B, L, dtype=torch.int32, device=DEV)
    with torch.cuda.stream(side):
        for rep, i in enumerate((2, 0, 1, 0)):
            load(i)
            graph.replay()
            side.synchronize()
            for k in KEYS:
                assert torch.equal(out[k], eager[i][k]), "replay %d (inputs %d): %s differs from the eager call" % (rep, i, k)
            # eager work of the same context between the replays: a step on other inputs into other buffers
            j = (i + 1) % 3
            mulo.mulo_verify_step(ctx, kv, B, Pn, params, h_blk, c["w"], c["r"], inputs[j][0], 0, inputs[j][1], inputs[j][2],
                                  other["tokens_out"], other["accept"], other["mask"], other["t0"], other["stats"], o_thi,
                                  None)
            side.synchronize()
            assert torch.equal(other["tokens_out"], eager[j]["tokens_out"])
        say("  4 replays of the recorded step equal the eager calls bit for bit")
    del graph
