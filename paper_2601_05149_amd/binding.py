"""ctypes binding of libmulo: the same entry points as include/mulo.h, taking
torch tensors (device memory) and marshalling them to plain pointers.  No
computation happens here, and there is no fallback: if the library is missing
or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmulo.so")

MULO_OK = 0
MULO_F32, MULO_BF16 = 0, 1
STATUS_NAMES = {0: "MULO_OK", 1: "MULO_ERR_NULL", 2: "MULO_ERR_SHAPE", 3: "MULO_ERR_RANGE",
                4: "MULO_ERR_ALLOC", 5: "MULO_ERR_HIP", 6: "MULO_ERR_UNSUPPORTED"}
EXPORTS = ["mulo_status_string", "mulo_check_model_cfg", "mulo_check_step_params", "mulo_workspace_bytes",
           "mulo_create", "mulo_destroy", "mulo_upsample_draft", "mulo_verify_forward",
           "mulo_accept_local_resample", "mulo_accept_local_resample_static", "mulo_verify_step", "mulo_resample_sequential", "mulo_rejection_islands", "mulo_resample_islands", "mulo_workspace_read", "mulo_profile",
           "mulo_profile_read"]


class MuloError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (%s)" % (where, STATUS_NAMES.get(status, status), status_string(status)))


class ModelCfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "head_dim", "d_ffn", "vocab",
                                         "max_batch", "max_seq", "max_block", "dtype")] + [("rms_eps", C.c_float),
                                                                                             ("stream_copy", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("embed", "attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate",
                                          "w_up", "w_down", "final_norm", "lm_head", "rope_cos", "rope_sin")]


class KV(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p)]


class StepParams(C.Structure):
    _fields_ = [("H", C.c_int32), ("W", C.c_int32), ("n0", C.c_int32), ("L", C.c_int32),
                ("radius", C.c_int32), ("expand", C.c_int32), ("pool_k", C.c_int32),
                ("nbr", C.c_void_p), ("resample_mode", C.c_int32),
                ("seed", C.c_uint64), ("rng_counter", C.c_uint64),
                ("accept_mode", C.c_int32), ("tau", C.c_float), ("cfg_scale", C.c_float)]


_lib = None


def load_library():
    """dlopen libmulo.so (built in-tree by paper_2601_05149_amd/build.py); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libmulo.so is not built: run `python -m paper_2601_05149_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    P, I32, I64 = C.c_void_p, C.c_int32, C.c_int64
    lib.mulo_status_string.restype = C.c_char_p
    lib.mulo_status_string.argtypes = [C.c_int]
    lib.mulo_check_model_cfg.argtypes = [C.POINTER(ModelCfg)]
    lib.mulo_check_step_params.argtypes = [C.POINTER(ModelCfg), I32, C.POINTER(StepParams)]
    lib.mulo_workspace_bytes.restype = C.c_uint64
    lib.mulo_workspace_bytes.argtypes = [C.POINTER(ModelCfg)]
    lib.mulo_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(Weights), P, C.POINTER(P)]
    lib.mulo_destroy.restype = None
    lib.mulo_destroy.argtypes = [P]
    lib.mulo_upsample_draft.argtypes = [P, I32, I32, I32, I32, P, I32, P, P, P, P, P]
    lib.mulo_verify_forward.argtypes = [P, C.POINTER(KV), I32, I32, I32, P, P, P]
    lib.mulo_accept_local_resample.argtypes = [P, I32, C.POINTER(StepParams), P, P, P, I64, P, P, P, P, P, P, P]
    lib.mulo_accept_local_resample_static.argtypes = [P, I32, I32, C.POINTER(StepParams), P, P, P, I64, P, P, P, P, P, P, P]
    lib.mulo_verify_step.argtypes = [P, C.POINTER(KV), I32, I32, C.POINTER(StepParams), I32, I32, I32, P, I32,
                                     P, P, P, P, P, P, P, P, P]
    lib.mulo_resample_sequential.argtypes = [P, C.POINTER(KV), I32, I32, I32, I32, C.c_uint64, C.c_uint64, P, P, P, P]
    lib.mulo_rejection_islands.argtypes = [P, I32, I32, I32, I32, P, P, P, P]
    lib.mulo_resample_islands.argtypes = [P, C.POINTER(KV), I32, I32, I32, I32, I32, C.c_uint64, C.c_uint64, P, P, P, P, P, P]
    lib.mulo_workspace_read.argtypes = [P, I32, P, C.c_uint64]
    lib.mulo_profile.argtypes = [P, I32]
    lib.mulo_profile_read.argtypes = [P, C.POINTER(C.c_float), C.POINTER(I32)]
    for n in EXPORTS:
        if n not in ("mulo_status_string", "mulo_workspace_bytes", "mulo_destroy"):
            getattr(lib, n).restype = C.c_int
    _lib = lib
    return lib


def status_string(status):
    return load_library().mulo_status_string(int(status)).decode()


def _ptr(t, dtype=None, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise ValueError("required tensor is None")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libmulo takes contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected %s, got %s" % (dtype, t.dtype))
    return t.data_ptr()


def _check(status, where):
    if status != MULO_OK:
        raise MuloError(status, where)


def make_cfg(model, max_batch, max_seq, max_block, stream_copy=False):
    bf16 = model["dtype"] == "bf16"
    return ModelCfg(model["n_layers"], model["d_model"], model["n_heads"], model["head_dim"], model["d_ffn"],
                    model["vocab"], max_batch, max_seq, max_block,
                    MULO_BF16 if bf16 else MULO_F32, model.get("rms_eps", 1e-5), 1 if (stream_copy and bf16) else 0)


MULO_ACCEPT_RATIO, MULO_ACCEPT_TAU = 0, 1


def make_params(H, W, n0, L, radius, expand=1, pool_k=1, nbr=None, resample_mode=0, seed=0, rng_counter=0,
                accept_mode=MULO_ACCEPT_RATIO, tau=0.0, cfg_scale=0.0):
    return StepParams(H, W, n0, L, radius, expand, pool_k, _ptr(nbr, torch.int32, True), resample_mode,
                      seed, rng_counter, accept_mode, tau, cfg_scale)


class Ctx:
    """Owns a mulo_ctx* and keeps the weight tensors alive (the library borrows them)."""

    def __init__(self, handle, cfg, keep):
        self.handle, self.cfg, self._keep = handle, cfg, keep
        self.tdtype = torch.bfloat16 if cfg.dtype == MULO_BF16 else torch.float32

    def __del__(self):
        try:
            mulo_destroy(self)
        except Exception:
            pass


def mulo_create(cfg, weights, rope_cos, rope_sin, stream=None):
    """weights: dict of device tensors (see mulo_weights); returns Ctx."""
    lib = load_library()
    tdt = torch.bfloat16 if cfg.dtype == MULO_BF16 else torch.float32
    names = ["embed", "attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down",
             "final_norm", "lm_head"]
    w = Weights(*[_ptr(weights[n], tdt) for n in names], _ptr(rope_cos, torch.float32), _ptr(rope_sin, torch.float32))
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    out = C.c_void_p()
    _check(lib.mulo_create(C.byref(cfg), C.byref(w), C.c_void_p(st), C.byref(out)), "mulo_create")
    return Ctx(out, cfg, [weights, rope_cos, rope_sin])


def mulo_destroy(ctx):
    if ctx is not None and ctx.handle:
        load_library().mulo_destroy(ctx.handle)
        ctx.handle = None


def alloc_kv(ctx, device="cuda", zero=True):
    """Allocate the KV cache in the layout mulo_kv documents; returns (k, v) tensors."""
    c = ctx.cfg
    mk = torch.zeros if zero else torch.empty
    k = mk(c.n_layers, c.max_batch, c.n_heads, c.max_seq, c.head_dim, dtype=ctx.tdtype, device=device)
    v = mk(c.n_layers, c.max_batch, c.n_heads, c.head_dim, c.max_seq, dtype=ctx.tdtype, device=device)
    return k, v


def mulo_upsample_draft(ctx, B, h, w, r, draft, input_is_probs, draft_tokens, tokens_hi, q_lo, q_row, q_hi=None):
    f32, i32 = torch.float32, torch.int32
    _check(load_library().mulo_upsample_draft(
        ctx.handle, B, h, w, r, _ptr(draft, f32), int(input_is_probs), _ptr(draft_tokens, i32),
        _ptr(tokens_hi, i32), _ptr(q_lo, f32), _ptr(q_row, i32), _ptr(q_hi, f32, True)), "mulo_upsample_draft")


def mulo_verify_forward(ctx, kv, B, L, P, in_tokens, in_embeds, logits):
    kvs = KV(_ptr(kv[0], ctx.tdtype), _ptr(kv[1], ctx.tdtype))
    _check(load_library().mulo_verify_forward(
        ctx.handle, C.byref(kvs), B, L, P, _ptr(in_tokens, torch.int32, True), _ptr(in_embeds, ctx.tdtype, True),
        _ptr(logits, torch.float32)), "mulo_verify_forward")


def mulo_accept_local_resample(ctx, B, params, logits, q, q_row, q_batch_stride, draft_tokens, tokens_out,
                               accept, mask, t0, stats, p_probs=None):
    f32, i32, u8 = torch.float32, torch.int32, torch.uint8
    _check(load_library().mulo_accept_local_resample(
        ctx.handle, B, C.byref(params), _ptr(logits, f32), _ptr(q, f32, True), _ptr(q_row, i32, True),
        int(q_batch_stride), _ptr(draft_tokens, i32), _ptr(tokens_out, i32), _ptr(accept, u8), _ptr(mask, u8),
        _ptr(t0, i32), _ptr(stats, i32), _ptr(p_probs, f32, True)), "mulo_accept_local_resample")


MULO_STATIC_MAX_ROWS = 65536


def mulo_accept_local_resample_static(vocab, B, params, logits, q, q_row, q_batch_stride, draft_tokens, tokens_out,
                                      accept, mask, t0, stats, p_probs=None, stream=None):
    """The decision stage without a context (allocates nothing); stream: a raw hipStream_t or None for
    torch's current stream."""
    f32, i32, u8 = torch.float32, torch.int32, torch.uint8
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    _check(load_library().mulo_accept_local_resample_static(
        C.c_void_p(st), vocab, B, C.byref(params), _ptr(logits, f32), _ptr(q, f32, True), _ptr(q_row, i32, True),
        int(q_batch_stride), _ptr(draft_tokens, i32), _ptr(tokens_out, i32), _ptr(accept, u8), _ptr(mask, u8),
        _ptr(t0, i32), _ptr(stats, i32), _ptr(p_probs, f32, True)), "mulo_accept_local_resample_static")


def mulo_verify_step(ctx, kv, B, P, params, h_blk, w, r, draft, input_is_probs, draft_tokens, prev_tokens,
                     tokens_out, accept, mask, t0, stats, tokens_hi=None, logits=None):
    f32, i32, u8 = torch.float32, torch.int32, torch.uint8
    kvs = KV(_ptr(kv[0], ctx.tdtype), _ptr(kv[1], ctx.tdtype))
    _check(load_library().mulo_verify_step(
        ctx.handle, C.byref(kvs), B, P, C.byref(params), h_blk, w, r, _ptr(draft, f32, True), int(input_is_probs),
        _ptr(draft_tokens, i32), _ptr(prev_tokens, i32), _ptr(tokens_out, i32), _ptr(accept, u8),
        _ptr(mask, u8), _ptr(t0, i32), _ptr(stats, i32), _ptr(tokens_hi, i32, True), _ptr(logits, f32, True)),
        "mulo_verify_step")


def mulo_resample_sequential(ctx, kv, B, P, L, u_start, seed, rng_counter, prev_tokens, mask, tokens, logits=None):
    f32, i32, u8 = torch.float32, torch.int32, torch.uint8
    kvs = KV(_ptr(kv[0], ctx.tdtype), _ptr(kv[1], ctx.tdtype))
    _check(load_library().mulo_resample_sequential(
        ctx.handle, C.byref(kvs), B, P, L, u_start, C.c_uint64(seed), C.c_uint64(rng_counter), _ptr(prev_tokens, i32),
        _ptr(mask, u8), _ptr(tokens, i32), _ptr(logits, f32, True)), "mulo_resample_sequential")


def mulo_rejection_islands(ctx, B, W, n0, L, mask, island, rank, counts):
    i32, u8 = torch.int32, torch.uint8
    _check(load_library().mulo_rejection_islands(ctx.handle, B, W, n0, L, _ptr(mask, u8), _ptr(island, i32), _ptr(rank, i32),
                                                 _ptr(counts, i32)), "mulo_rejection_islands")


def mulo_resample_islands(ctx, kv, B, P, L, n_passes, max_islands, seed, rng_counter, prev_tokens, mask, rank, tokens,
                          logits=None, overflow=None):
    f32, i32, u8 = torch.float32, torch.int32, torch.uint8
    kvs = KV(_ptr(kv[0], ctx.tdtype), _ptr(kv[1], ctx.tdtype))
    _check(load_library().mulo_resample_islands(
        ctx.handle, C.byref(kvs), B, P, L, n_passes, max_islands, C.c_uint64(seed), C.c_uint64(rng_counter),
        _ptr(prev_tokens, i32), _ptr(mask, u8), _ptr(rank, i32), _ptr(tokens, i32), _ptr(logits, f32, True),
        _ptr(overflow, i32, True)), "mulo_resample_islands")


MULO_WS_RESIDUAL, MULO_WS_NORMED, MULO_WS_Q, MULO_WS_ATTN, MULO_WS_FFN = range(5)


def mulo_workspace_read(ctx, which, dst):
    """Copy a workspace buffer of the last forward pass into the (contiguous, device) tensor dst."""
    _check(load_library().mulo_workspace_read(ctx.handle, which, _ptr(dst), dst.numel() * dst.element_size()),
           "mulo_workspace_read")


PROF_CLASSES = ["gemm_qkv", "gemm_out", "gemm_gate_up", "gemm_down", "gemm_lm_head", "attention", "norm_embed",
                "upsample", "accept", "mask_sample", "other"]


def mulo_profile(ctx, enable):
    _check(load_library().mulo_profile(ctx.handle, int(enable)), "mulo_profile")


def mulo_profile_read(ctx):
    """Returns {class name: (milliseconds, launches)} accumulated since the last read."""
    n = len(PROF_CLASSES)
    ms, cnt = (C.c_float * n)(), (C.c_int32 * n)()
    _check(load_library().mulo_profile_read(ctx.handle, ms, cnt), "mulo_profile_read")
    return {PROF_CLASSES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}
