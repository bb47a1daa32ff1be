"""GPU test of the entry point that allocates nothing, mulo_accept_local_resample_static: through the C ABI its
outputs must equal, bit for bit, those of mulo_accept_local_resample (whose oracle parity is
tests/test_gpu_decide.py) on the same seeded inputs -- on two calls in a row, the second with a smaller input, so
that nothing of the first call's row statistics in the static scratch can leak into the second."""
import numpy as np
import pytest
import torch

import paper_2601_05149_amd as mulo
from oracle import step as ST
from tests.gpu_util import DEV, compare_decisions, decide_buffers, dev, say, to_np
from tests.test_gpu_decide import clean_inputs, decide_ctx

pytestmark = pytest.mark.gpu


def both(ctx, V, zp, q, toks, **pk):
    B, L, _ = zp.shape
    params = mulo.make_params(**pk)
    z_d, q_d, t_d = dev(zp, torch.float32), dev(q, torch.float32), dev(toks, torch.int32)
    ref, got = decide_buffers(B, L), decide_buffers(B, L)
    p_ref, p_got = torch.empty(B, L, V, device=DEV), torch.full((B, L, V), -1.0, device=DEV)
    mulo.mulo_accept_local_resample(ctx, B, params, z_d, q_d, None, L * V, t_d, ref["tokens_out"], ref["accept"],
                                    ref["mask"], ref["t0"], ref["stats"], p_ref)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    mulo.mulo_accept_local_resample_static(V, B, params, z_d, q_d, None, L * V, t_d, got["tokens_out"], got["accept"],
                                           got["mask"], got["t0"], got["stats"], p_got)
    torch.cuda.synchronize()
    say("  free device memory around the call: %d -> %d bytes" % (free_before, torch.cuda.mem_get_info()[0]))
    ref, got = to_np(ref), to_np(got)
    for k in ref:
        assert np.array_equal(ref[k], got[k]), k
    assert torch.equal(p_ref, p_got)
    return got


def test_static_entry_point_equals_the_context_one_on_two_calls_in_a_row():
    V = 4096
    ctx = decide_ctx(V, 4, 1024)
    # first call: 3 x 1024 rows (fills 3072 slots of the static scratch); second call: 2 x 128 rows
    for B, L, W, n0, H, seed in ((3, 1024, 32, 0, 32, 21), (2, 128, 16, 128, 16, 22)):
        say("static decision stage B=%d L=%d" % (B, L))
        zp, q, toks = clean_inputs(B, L, V, 1.0, seed)
        pk = dict(H=H, W=W, n0=n0, L=L, radius=1, expand=1, seed=seed, rng_counter=5)
        got = both(ctx, V, zp, q, toks, **pk)
        assert 0 < got["stats"][:, 1].min(), "the inputs must produce rejections"
        # and against the oracle directly, to the bar of the decision-stage tests
        ref = ST.decide(zp, q, None, toks, W=W, n0=n0, radius=1, expand=1, seed=seed, rng_counter=5)
        rep = compare_decisions(got, ref, toks, q, None, label="static B=%d L=%d" % (B, L))
        say("  flips %d, near ties %d, boundary draws %d" % (rep["flips"], rep["near_ties"], rep["tok_mismatch"]))


def test_static_entry_point_argument_errors():
    V, B, L = 1024, 1, 64
    z = torch.zeros(B, L, V, device=DEV)
    t = torch.zeros(B, L, dtype=torch.int32, device=DEV)
    o = decide_buffers(B, L)
    args = lambda **kw: (z, z, None, L * V, t, o["tokens_out"], o["accept"], o["mask"], o["t0"], o["stats"])
    ok = dict(H=8, W=8, n0=0, L=64, radius=1)
    with pytest.raises(mulo.MuloError) as e:        # more rows than the static scratch holds
        mulo.mulo_accept_local_resample_static(V, 2048, mulo.make_params(**ok), *args())
    assert e.value.status == 2
    with pytest.raises(mulo.MuloError) as e:
        mulo.mulo_accept_local_resample_static(V + 2, B, mulo.make_params(**ok), *args())
    assert e.value.status == 6
    with pytest.raises(mulo.MuloError) as e:
        mulo.mulo_accept_local_resample_static(V, B, mulo.make_params(**dict(ok, L=60)), *args())
    assert e.value.status == 2
    assert (o["tokens_out"] == -7).all(), "a rejected call must not write"
