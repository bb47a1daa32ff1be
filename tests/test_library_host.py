"""CPU-side checks of the C ABI: the library loads, exports every symbol the
header declares, and its host-only argument checks behave.  No compute."""
import ctypes as C
import os
import re

import pytest

import paper_2601_05149_amd as mulo
from paper_2601_05149_amd import binding as BD
from workloads import configs as WC

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(BD.LIB_PATH):
        from paper_2601_05149_amd import build
        build.build_lib()
    return mulo.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "mulo.h")).read()
    declared = set(re.findall(r"MULO_API\s+[\w\s\*]+?\b(mulo_\w+)\s*\(", header))
    assert declared == set(BD.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    seen = {lib.mulo_status_string(i) for i in range(7)}
    assert len(seen) == 7 and all(seen)
    assert lib.mulo_status_string(99)


def test_model_cfg_checks(lib):
    for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5_L1024"):
        c = WC.get(name)
        cfg = mulo.make_cfg(c["model"], c["B"], c["max_seq"], c["L"])
        assert lib.mulo_check_model_cfg(C.byref(cfg)) == 0
        assert lib.mulo_workspace_bytes(C.byref(cfg)) > 0
    c = WC.get("cfg2")
    bad = mulo.make_cfg(c["model"], 4, c["max_seq"], 256)
    bad.n_heads = 15
    assert lib.mulo_check_model_cfg(C.byref(bad)) == 2          # heads * head_dim != d
    bad = mulo.make_cfg(c["model"], 4, c["max_seq"], 256)
    bad.vocab = 8190
    assert lib.mulo_check_model_cfg(C.byref(bad)) == 6
    bad = mulo.make_cfg(c["model"], 0, c["max_seq"], 256)
    assert lib.mulo_check_model_cfg(C.byref(bad)) == 3
    bad = mulo.make_cfg(c["model"], 4, 100, 256)
    assert lib.mulo_check_model_cfg(C.byref(bad)) == 2          # block longer than the cache
    assert lib.mulo_check_model_cfg(None) == 1
    assert lib.mulo_workspace_bytes(C.byref(bad)) == 0
    # the second copy of the weights for the weight-streaming kernels: bf16 only, 0 or 1, and it is part of the workspace
    plain = mulo.make_cfg(c["model"], 4, c["max_seq"], 256)
    copy = mulo.make_cfg(c["model"], 4, c["max_seq"], 256, stream_copy=True)
    assert lib.mulo_check_model_cfg(C.byref(copy)) == 0
    m = c["model"]
    w_bytes = 2 * (m["n_layers"] * (4 * m["d_model"] ** 2 + 3 * m["d_ffn"] * m["d_model"]) + m["vocab"] * m["d_model"])
    # ... plus the partial sums of the largest projection of a 256-token call: K slices x tokens x columns floats, with
    # as many K slices per 128-column group as keep the launch within 256 workgroups (at most 8, at least 8 k-steps each)
    def ksum(ncols, K, M=256):
        ks = max(1, min(8, 256 // ((ncols + 127) // 128)))
        return min(ks, max(1, K // 32 // 8)) * M * ncols * 4
    d_, f_, V_ = m["d_model"], m["d_ffn"], m["vocab"]
    k_bytes = max(ksum(3 * d_, d_), ksum(d_, d_), ksum(2 * f_, d_), ksum(d_, f_), ksum(V_, d_))
    extra = lib.mulo_workspace_bytes(C.byref(copy)) - lib.mulo_workspace_bytes(C.byref(plain)) - w_bytes - k_bytes
    assert 0 <= extra < 1024          # buffers start on 256-byte boundaries
    copy.stream_copy = 2
    assert lib.mulo_check_model_cfg(C.byref(copy)) == 3
    f32 = mulo.make_cfg(WC.get("cfg1")["model"], 1, 296, 256)
    f32.stream_copy = 1
    assert lib.mulo_check_model_cfg(C.byref(f32)) == 6


def test_step_param_checks(lib):
    c = WC.get("cfg2")
    cfg = mulo.make_cfg(c["model"], 4, c["max_seq"], 256)
    ok = lambda **kw: lib.mulo_check_step_params(C.byref(cfg), kw.pop("B", 4), C.byref(BD.StepParams(**kw)))
    base = dict(H=32, W=32, n0=256, L=256, radius=1, expand=1, pool_k=1, nbr=None, resample_mode=0, seed=0,
                rng_counter=0)
    assert ok(**base) == 0
    assert ok(**{**base, "L": 250}) == 2            # not whole rows
    assert ok(**{**base, "n0": 40}) == 2            # block does not start on a row
    assert ok(**{**base, "n0": 896}) == 2           # runs past the grid
    assert ok(**{**base, "L": 512}) == 2            # longer than max_block
    assert ok(**{**base, "radius": -2}) == 3
    assert ok(**{**base, "radius": -1}) == 0        # raster-scan rule
    assert ok(**{**base, "pool_k": 4}) == 1         # pooling without a table
    assert ok(**{**base, "resample_mode": 2}) == 0  # every marked position re-drawn from p
    assert ok(**{**base, "resample_mode": 3}) == 3
    assert ok(**{**base, "accept_mode": 1, "tau": 1e-4}) == 0   # threshold rule (Eq. 5)
    assert ok(**{**base, "accept_mode": 1, "tau": -1.0}) == 3
    assert ok(**{**base, "accept_mode": 1, "tau": float("nan")}) == 3
    assert ok(**{**base, "accept_mode": 2}) == 3
    assert ok(**{**base, "B": 5}) == 2
    assert lib.mulo_check_step_params(C.byref(cfg), 4, None) == 1
    # a block whose accept flags do not fit the LDS of the per-sequence kernel
    long_cfg = mulo.make_cfg(c["model"], 1, 1 << 19, 1 << 18)
    huge = dict(base, H=512, W=512, n0=0, L=1 << 18)
    assert lib.mulo_check_step_params(C.byref(long_cfg), 1, C.byref(BD.StepParams(**huge))) == 6
    assert lib.mulo_check_step_params(C.byref(long_cfg), 1, C.byref(BD.StepParams(**dict(huge, L=1 << 17)))) == 0


def test_create_rejects_bad_arguments_without_a_gpu_call(lib):
    out = C.c_void_p()
    c = WC.get("cfg1")
    cfg = mulo.make_cfg(c["model"], 1, c["max_seq"], 256)
    assert lib.mulo_create(None, None, None, C.byref(out)) == 1
    w = BD.Weights()                                 # all NULL
    assert lib.mulo_create(C.byref(cfg), C.byref(w), None, C.byref(out)) == 1
    assert not out.value
    lib.mulo_destroy(None)                           # allowed


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: the benchmark says so and exits before it touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300, cwd=root)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr + r.stdout and '"metric"' not in r.stdout


def test_static_entry_point_rejects_bad_arguments_before_any_gpu_call(lib):
    """mulo_accept_local_resample_static checks its arguments on the host first (no device is touched)."""
    V, B, L = 1024, 1, 64
    ok = BD.StepParams(H=8, W=8, n0=0, L=L, radius=1, expand=1, pool_k=1, nbr=None, resample_mode=0, seed=0, rng_counter=0)
    one = C.c_void_p(256)       # never dereferenced: every call below fails its checks
    call = lambda vocab, b, p, logits=one: lib.mulo_accept_local_resample_static(
        None, vocab, b, p, logits, one, None, L * V, one, one, one, one, one, one, None)
    assert call(V, B, C.byref(ok), logits=None) == 1
    assert call(V, B, None) == 1
    assert call(2, B, C.byref(ok)) == 3
    assert call(V + 2, B, C.byref(ok)) == 6
    assert call(V, BD.MULO_STATIC_MAX_ROWS // L + 1, C.byref(ok)) == 2         # more rows than the static scratch
    bad = BD.StepParams(H=8, W=8, n0=0, L=60, radius=1, expand=1, pool_k=1, nbr=None, resample_mode=0, seed=0, rng_counter=0)
    assert call(V, B, C.byref(bad)) == 2
    header = open(os.path.join(ROOT, "include", "mulo.h")).read()
    assert "#define MULO_STATIC_MAX_ROWS %d" % BD.MULO_STATIC_MAX_ROWS in header
