#!/usr/bin/env python3
"""Benchmark of the MuLo-SD verification step (libmulo) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4] [--no-cpu-baseline]

One "step" = one mulo_verify_step call (up-sample -> target forward over the
draft block against the KV cache -> accept test -> local expansion -> residual
re-draw) over one batch of synthetic input already resident in HBM.  Prints ONE
JSON line: verified image tokens/s (B*L / step time), a roofline object for the
dominant kernel (the gate|up projection GEMM, bf16 MFMA bound) measured with HIP
events on the library's stream during the timed steps, per-kernel-class figures,
and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def cpu_model_name():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(c, w, cos, sin, seed, sigma):
    """The oracle as it stands on a bounded sample of the workload: batch element 0, two low-resolution rows (2 r grid
    rows) of the last block as the draft block, against the full-length seeded cache, draft made by the workload's
    recipe (target-like logits of an un-timed oracle pass over a provisional draft + sigma noise).  Only the
    verification step is timed."""
    import numpy as np
    import torch

    from oracle import decoder as OD
    from oracle import step as OS
    from oracle import upsample as OU
    from workloads import generators as G
    m = c["model"]
    nl, nh, dh, V = m["n_layers"], m["n_heads"], m["head_dim"], m["vocab"]
    h_blk = min(2, c["L"] // c["W"] // c["r"])   # low-resolution rows behind the sample block
    Ls = h_blk * c["W"] * c["r"]
    P = c["max_seq"] - c["L"]
    dec = OD.DecoderOracle(m, w, cos, sin, 1, P + Ls, round_bf16=(m["dtype"] == "bf16"))
    dec.k[:, 0, :P] = G.random_kv((nl, nh, P, dh), seed, tag=0).permute(0, 2, 1, 3).to(dec.k.dtype)
    dec.v[:, 0, :P] = G.random_kv((nl, nh, P, dh), seed, tag=1).permute(0, 2, 1, 3).to(dec.v.dtype)
    n_lo = h_blk * c["w"]
    prev = np.zeros(1, np.int32)
    y0 = G.uniform_tokens((1, n_lo), V, seed, tag=7)
    x0 = OU.upsample_draft(np.zeros((1, n_lo, 1)), y0, h_blk, c["w"], c["r"], input_is_probs=True)[0]
    z_p = dec.forward(np.concatenate([prev.reshape(1, 1), x0[:, :Ls - 1]], axis=1).astype(np.int32), P).numpy()   # un-timed
    child0 = (np.arange(h_blk)[:, None] * c["r"] * c["W"] + np.arange(c["w"])[None, :] * c["r"]).reshape(-1)
    dl = (z_p[:, child0, :] + sigma * G.normal_logits((1, n_lo, V), 1.0, seed, tag=8)).astype(np.float32)
    dt = G.sample_categorical(dl, seed, tag=8)
    threads = torch.get_num_threads()
    t0 = time.perf_counter()
    ref = OS.verify_step(dec, P, dl, dt, prev, h_blk=h_blk, w=c["w"], r=c["r"], W=c["W"],
                         n0=c["T"] - c["L"], radius=c["radius"], expand=c["expand"], seed=seed, rng_counter=0)
    dt_s = time.perf_counter() - t0
    return {"value": Ls / dt_s, "unit": "verified tokens/s", "cores": threads, "cpu": cpu_model_name(), "kind": "oracle",
            "sample": "batch element 0, one %d-token block (%d grid rows) at P=%d of workload %s, draft by the workload's "
                      "recipe (sigma %.2g, acceptance %.2f), all %d layers, float64; %.1f s including the per-call "
                      "bf16->float64 weight conversion" % (Ls, h_blk * c["r"], P, c["name"], sigma,
                                                            float(ref["accept"].mean()), nl, dt_s)}


def resample_bench(mulo, ctx, kv, c, B, L, P, V, rate, seed, gen):
    """Re-sampling of the marked positions of one block (Alg. 1 Step 6; Sec. 3.4): a synthetic verification rejects
    each position with probability `rate`, R_X is the radius-1 neighbourhood of the rejections from the first one
    on (Eq. 6-7), and both re-samplers run on it.  Prints one JSON line."""
    import numpy as np
    import torch
    dev = "cuda:0"
    W = c["W"]
    rows = L // W
    rng = np.random.default_rng(seed)
    rej = rng.random((B, rows, W)) < rate
    rej[:, rows // 2, W // 2] = True                       # at least one rejection per sequence
    mask = np.zeros_like(rej)
    for b, i, j in zip(*np.nonzero(rej)):
        mask[b, max(i - 1, 0):i + 2, max(j - 1, 0):j + 2] = True
    mask = mask.reshape(B, L)
    t0s = [int(np.flatnonzero(rej[b].reshape(-1))[0]) for b in range(B)]
    for b in range(B):
        mask[b, :t0s[b]] = False
    mask_d = torch.tensor(mask.astype(np.uint8), device=dev)
    island = torch.empty(B, L, dtype=torch.int32, device=dev)
    rank = torch.empty_like(island)
    counts = torch.empty(B, 2, dtype=torch.int32, device=dev)
    mulo.mulo_rejection_islands(ctx, B, W, c["T"] - L, L, mask_d, island, rank, counts)
    cn = counts.cpu().numpy()
    cap, passes = int(cn[:, 0].max()), int(cn[:, 1].max())
    tokens = torch.randint(0, V, (B, L), generator=gen, device=dev, dtype=torch.int32)
    prev = torch.zeros(B, dtype=torch.int32, device=dev)
    u_start = min(t0s)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t)

    ms_isl = timed(lambda: mulo.mulo_resample_islands(ctx, kv, B, P, L, passes, cap, seed, 0, prev, mask_d, rank, tokens))
    ms_seq = timed(lambda: mulo.mulo_resample_sequential(ctx, kv, B, P, L, u_start, seed, 0, prev, mask_d, tokens))
    tok1 = torch.randint(0, V, (B, 1), generator=gen, device=dev, dtype=torch.int32)
    z1 = torch.empty(B, 1, V, device=dev)
    ms_tok = timed(lambda: [mulo.mulo_verify_forward(ctx, kv, B, 1, P + L - 1, tok1, None, z1) for _ in range(20)]) / 20
    print(json.dumps({
        "metric": "re-sampling of one verified block (1 GPU)", "unit": "ms", "higher_is_better": False, "data": "synthetic",
        "config": {"workload": "%s: last block, B=%d L=%d P=%d, rejection rate %g, radius 1" % (c["name"], B, L, P, rate),
                   "stream_copy": int(ctx.cfg.stream_copy)},
        "marked_positions": int(mask.sum()), "islands_per_sequence": cn[:, 0].tolist(), "largest_island": cn[:, 1].tolist(),
        "island_passes": passes, "slots_per_pass": B * cap, "sequential_steps": L - u_start,
        "ms_islands": round(ms_isl, 2), "ms_sequential": round(ms_seq, 2), "ms_single_token_step": round(ms_tok, 3),
        "ms_per_island_pass": round(ms_isl / max(passes, 1), 3)}), flush=True)


def traffic_from_profile(workload):
    """HBM bytes per launch of the roofline kernel (both kernels of the gate|up projection): FETCH_SIZE and WRITE_SIZE
    of two rocprofv3 --pmc runs of this benchmark, scaled by the copy-kernel calibration; read from the line
    `roofline kernel traffic per launch: N bytes` of profiles/verify_step_<workload>_hbm_traffic.md (bench.py
    cannot run the profiler on itself).  None when that summary is absent."""
    import re
    path = os.path.join(ROOT, "profiles", "verify_step_%s_hbm_traffic.md" % workload)
    try:
        m = re.search(r"roofline kernel traffic per launch:\s*([0-9.eE+]+)\s*bytes", open(path).read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def run_workload(mulo, name, wd, rope, steps, warmup, sigma=None, first_block=False, profile="roofline", want_ctx=False,
                 stream_copy=False):
    """Times `steps` mulo_verify_step calls of workload `name` (inputs resident in HBM) and returns its figures."""
    import torch

    from paper_2601_05149_amd.binding import PROF_CLASSES
    from workloads import configs as WC
    dev = "cuda:0"
    c = WC.get(name)
    m = c["model"]
    B, L, V, seed = c["B"], c["L"], m["vocab"], c["seed"]
    sigma = sigma if sigma is not None else (c["sigma"] if c["sigma"] is not None else 1.0)
    P = c["prefix"] if first_block else c["max_seq"] - L     # last block of the image: the largest cache
    n0 = 0 if first_block else c["T"] - L
    h_blk = L // c["W"] // c["r"]
    n_lo = h_blk * c["w"]
    log("workload %s%s: B=%d L=%d P=%d V=%d" % (c["name"], " (first block)" if first_block else "", B, L, P, V))
    # stream_copy: the context keeps the weights once more in the order of the weight-streaming kernels (re-sampling runs)
    cfg = mulo.make_cfg(m, B, c["max_seq"], L, stream_copy=stream_copy)
    ctx = mulo.mulo_create(cfg, wd, rope[0], rope[1])
    kv = mulo.alloc_kv(ctx, dev, zero=False)
    # cache rows [0, P): seeded N(0, 1) values (a stand-in for the prefilled prefix + committed blocks)
    gen = torch.Generator(device=dev).manual_seed(seed)
    kv[0][:, :, :, :P].normal_(generator=gen)
    kv[1][:, :, :, :, :P].normal_(generator=gen)

    # draft recipe ("target-like logits + N(0, sigma)"): provisional uniform draft -> un-timed forward ->
    # draft logits = target logits of the top-left child + sigma * noise -> draft tokens ~ softmax(draft logits)
    prov = torch.randint(0, V, (B, n_lo), generator=gen, device=dev, dtype=torch.int32)
    thi = torch.empty(B, L, dtype=torch.int32, device=dev)
    q_lo = torch.empty(B, n_lo, V, device=dev)
    q_row = torch.empty(L, dtype=torch.int32, device=dev)
    mulo.mulo_upsample_draft(ctx, B, h_blk, c["w"], c["r"], torch.zeros(B, n_lo, V, device=dev), 0, prov, thi, q_lo,
                             q_row, None)
    prev = torch.randint(0, V, (B,), generator=gen, device=dev, dtype=torch.int32)
    inp = torch.cat([prev.reshape(B, 1), thi[:, :L - 1]], dim=1).contiguous()
    zp = torch.empty(B, L, V, device=dev)
    mulo.mulo_verify_forward(ctx, kv, B, L, P, inp, None, zp)
    r = c["r"]
    child0 = (torch.arange(h_blk, device=dev)[:, None] * r * c["W"] + torch.arange(c["w"], device=dev)[None, :] * r).reshape(-1)
    draft_logits = zp[:, child0, :].contiguous()
    del zp, q_lo
    draft_logits.add_(torch.randn(B, n_lo, V, generator=gen, device=dev), alpha=sigma)
    gumbel = torch.rand(B, n_lo, V, generator=gen, device=dev).clamp_min_(1e-20).log_().neg_().log_().neg_()
    draft_tokens = gumbel.add_(draft_logits).argmax(-1).to(torch.int32).contiguous()
    del gumbel

    out = dict(tokens_out=torch.empty(B, L, dtype=torch.int32, device=dev),
               accept=torch.empty(B, L, dtype=torch.uint8, device=dev),
               mask=torch.empty(B, L, dtype=torch.uint8, device=dev),
               t0=torch.empty(B, dtype=torch.int32, device=dev),
               stats=torch.empty(B, 4, dtype=torch.int32, device=dev))

    def step(i):
        params = mulo.make_params(c["H"], c["W"], n0, L, c["radius"], c["expand"], seed=seed, rng_counter=i)
        mulo.mulo_verify_step(ctx, kv, B, P, params, h_blk, c["w"], r, draft_logits, 0, draft_tokens, prev,
                              out["tokens_out"], out["accept"], out["mask"], out["t0"], out["stats"])

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # inside the timed region only the roofline kernel's class is bracketed by events (a pair costs a few microseconds
    # of stream time; bracketing all ~520 launches of a step costs about 2.5 %)
    if profile == "all":
        mulo.mulo_profile(ctx, 1)
    elif profile == "roofline":
        mulo.mulo_profile(ctx, 0x100 | PROF_CLASSES.index("gemm_gate_up"))
    # per-step marks on the library's stream (torch's current one): recorded, not waited for, inside the timed region
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t_start = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step(warmup + i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt_s = time.perf_counter() - t_start
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    prof_timed = mulo.mulo_profile_read(ctx) if profile != "none" else {}
    prof_steps = steps
    prof = prof_timed
    if profile == "roofline":
        # every other class from two extra, un-timed steps with all launches bracketed
        mulo.mulo_profile(ctx, 1)
        for i in range(2):
            step(warmup + steps + i)
        prof = mulo.mulo_profile_read(ctx)
        prof["gemm_gate_up"] = tuple(x * 2.0 / steps for x in prof_timed["gemm_gate_up"])   # the timed region's, per 2 steps
        prof_steps = 2
    mulo.mulo_profile(ctx, 0)
    ms_per_step = 1e3 * dt_s / steps
    stats = out["stats"].cpu().numpy()
    acc_rate = float(stats[:, 0].sum()) / (B * L)
    marked = float(stats[:, 2].sum()) / (B * L)

    # algorithmic work per launch
    d, f, nl = m["d_model"], m["d_ffn"], m["n_layers"]
    M = B * L
    flops = {"gemm_qkv": 2.0 * M * 3 * d * d, "gemm_out": 2.0 * M * d * d, "gemm_gate_up": 2.0 * M * 2 * f * d,
             "gemm_down": 2.0 * M * d * f, "gemm_lm_head": 2.0 * M * V * d,
             # causal attention: query j sees P + j + 1 keys; 4 * d flops per (query, key)
             "attention": 4.0 * d * B * sum(P + j + 1 for j in range(L))}
    byts = {"upsample": 2.0 * 4 * V * B * n_lo,            # read draft logits, write q_lo
            # every marked position reads its logit row; its draft row is shared with the r*r - 1 siblings
            "mask_sample": 4.0 * V * M * marked * (1.0 + 1.0 / (r * r))}
    kernels = {}
    for name_, (ms, n) in prof.items():
        if n == 0:
            continue
        avg = ms / n
        e = {"avg_ms": round(avg, 4), "launches_per_step": n / prof_steps}
        if name_ in flops and m["dtype"] == "bf16":
            e.update(bound="mfma", achieved=round(flops[name_] / (avg * 1e-3) / 1e12, 1), unit="TFLOP/s")
            e["frac"] = round(e["achieved"] / PEAK_BF16_TFLOPS, 4)
            if name_ == "attention":   # K and V rows of every (sequence, head) read once per launch
                kv_bytes = 2.0 * 2 * d * B * (P + L)
                e["kv_gbs"] = round(kv_bytes / (avg * 1e-3) / 1e9, 1)
        elif name_ in byts:
            per_step_ms = ms / prof_steps      # the class's launches of a step together (they differ in size)
            e["ms_per_step"] = round(per_step_ms, 4)
            e.update(bound="hbm", achieved=round(byts[name_] / (per_step_ms * 1e-3) / 1e9, 1), unit="GB/s")
            e["frac"] = round(e["achieved"] / PEAK_HBM_GBS, 4)
        elif name_ == "accept":
            e["note"] = ("row statistics come from the lm-head epilogue; this kernel merges them and gathers one logit "
                         "per position (no pass over the logits)")
        kernels[name_] = e
    roof = None
    if "gemm_gate_up" in kernels and "achieved" in kernels["gemm_gate_up"]:
        k = kernels["gemm_gate_up"]
        roof = {"bound": "mfma", "kernel": "k_gemm_bf16<EPI_SWIGLU> (gate|up projection + SwiGLU)",
                "achieved": k["achieved"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": k["frac"],
                "traffic": None if first_block else traffic_from_profile(c["name"]), "avg_ms": k["avg_ms"],
                "flops_per_launch": flops["gemm_gate_up"], "measured": "HIP events around every launch of the timed steps"}
    fwd_flops = nl * (flops["gemm_qkv"] + flops["gemm_out"] + flops["gemm_gate_up"] + flops["gemm_down"]
                      + flops["attention"]) + flops["gemm_lm_head"]
    res = {"value": round(M / (ms_per_step * 1e-3), 1), "ms_per_step": round(ms_per_step, 3),
           "config": {"workload": "%s: %s decoder, B=%d, draft block L=%d of a %dx%d grid (%s block, P=%d cache rows), "
                                  "V=%d, radius %d, sigma %.2g" % (c["name"], c["model_name"], B, L, c["H"], c["W"],
                                                                    "first" if first_block else "last", P, V, c["radius"], sigma),
                      "acceptance_rate": round(acc_rate, 4), "marked_fraction": round(marked, 4)},
           "accepted_tokens_per_s": round(M * (1.0 - marked) / (ms_per_step * 1e-3), 1),
           "ms_per_step_median": round(per_step[len(per_step) // 2], 3), "ms_per_step_min": round(per_step[0], 3),
           "step_tflops": round(fwd_flops / (ms_per_step * 1e-3) / 1e12, 1),
           "step_frac_of_bf16_peak": round(fwd_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
           "roofline": roof, "kernels": kernels}
    if want_ctx:
        return res, c, ctx, kv, gen
    del ctx, kv
    torch.cuda.empty_cache()
    return res, c, sigma


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg5_L1024",
                    help="default: the largest single-GPU workload (batch 16, 1024-token blocks); cfg1..cfg4, cfg5_L256, ...")
    ap.add_argument("--sigma", type=float, default=None, help="draft-logit noise std (default: the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--profile-all", action="store_true",
                    help="bracket every kernel class inside the timed region (adds ~3 %% to the step); default: only the "
                         "roofline kernel there, every class in two extra un-timed steps")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the secondary points (cfg4 last and first block) that the default run adds")
    ap.add_argument("--constant-weights", type=float, default=None, metavar="C",
                    help="diagnostic, never the reported workload: every weight matrix is filled with C, so the operands "
                         "of the matrix instructions stop changing from one to the next; the same kernels then show what "
                         "they sustain when the chip does not lower its clock with the switching activity of the data")
    ap.add_argument("--resample", type=float, default=None, metavar="RATE",
                    help="instead of the verify step: time the re-sampling of the workload's last block after a "
                         "synthetic verification with this fraction of rejected positions (radius 1) - "
                         "mulo_resample_islands against mulo_resample_sequential, and one single-token target step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB read + 1 GiB write element-wise kernel (scale for HBM byte counters)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2601_05149_amd as mulo
    from workloads import configs as WC
    from workloads import generators as G

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if a.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"read_bytes": src.numel() * 4, "write_bytes": dst.numel() * 4,
                                             "launches": 3}}), flush=True)
        return
    mulo.load_library()                   # fails loudly if the HIP library is not built
    dev = "cuda:0"
    c = WC.get(a.workload)
    m = c["model"]
    log("generating %s weights ..." % c["model_name"])
    w = G.make_weights(m, seed=c["seed"])
    cos, sin = G.rope_table(WC.get("cfg5_L1024")["max_seq"] if c["model_name"] == "7b" else c["max_seq"], m["head_dim"])
    wd = {k: v.to(dev) for k, v in w.items()}
    if a.constant_weights is not None:
        for name, t in wd.items():
            if t.dim() >= 2 and "norm" not in name:
                t.fill_(a.constant_weights)
    rope = (torch.tensor(cos[:c["max_seq"]], device=dev), torch.tensor(sin[:c["max_seq"]], device=dev))

    if a.resample is not None:
        _, c, ctx, kv, gen = run_workload(mulo, a.workload, wd, rope, 1, 1, a.sigma, profile="none", want_ctx=True,
                                          stream_copy=m["dtype"] == "bf16")
        resample_bench(mulo, ctx, kv, c, c["B"], c["L"], c["max_seq"] - c["L"], m["vocab"], a.resample, c["seed"], gen)
        return

    profile = "none" if a.no_profile else ("all" if a.profile_all else "roofline")
    main_res, c, sigma = run_workload(mulo, a.workload, wd, rope, a.steps, a.warmup, a.sigma, profile=profile)
    res = {"metric": "verified image tokens/sec (1 GPU) per verify step", "value": main_res.pop("value"),
           "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
           "ms_per_step": main_res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": m["dtype"],
           "data": "synthetic" if a.constant_weights is None else "synthetic, CONSTANT weights (clock diagnostic, not the workload)"}
    res.update(main_res)
    # secondary points, outside the timed region of the headline: the batch-4 1024-token workload at its last block
    # (the largest cache) and at its first block (P = the prefix only) for contrast
    if a.workload == "cfg5_L1024" and not a.no_extra:
        extra = {}
        for key, fb in (("cfg4", False), ("cfg4_first_block", True)):
            cc = WC.get("cfg4")
            r4, _, _ = run_workload(mulo, "cfg4", wd, (rope[0][:cc["max_seq"]].contiguous(), rope[1][:cc["max_seq"]].contiguous()),
                                    5, 2, a.sigma, first_block=fb, profile=profile)
            extra[key] = {k: r4[k] for k in ("value", "ms_per_step", "config", "step_tflops", "step_frac_of_bf16_peak",
                                             "roofline", "kernels")}
        res["other_workloads"] = extra
    if a.no_cpu_baseline:
        res["cpu_baseline"] = None
    else:
        log("timing the CPU oracle on a bounded sample ...")
        del wd
        torch.cuda.empty_cache()
        res["cpu_baseline"] = cpu_baseline(c, w, cos, sin, c["seed"], sigma)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
