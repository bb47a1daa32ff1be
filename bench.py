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


def cpu_baseline(c, w, cos, sin, seed):
    """The oracle as it stands on a bounded sample: batch element 0, two low-resolution rows (2 r grid rows)
    as the draft block, against the full-length seeded cache."""
    import numpy as np
    import torch

    from oracle import decoder as OD
    from oracle import step as OS
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
    dl = G.normal_logits((1, n_lo, V), 2.0, seed, tag=7)
    dt = G.sample_categorical(dl, seed, tag=7)
    threads = torch.get_num_threads()
    t0 = time.perf_counter()
    OS.verify_step(dec, P, dl, dt, np.zeros(1, np.int32), h_blk=h_blk, w=c["w"], r=c["r"], W=c["W"],
                   n0=c["T"] - c["L"], radius=c["radius"], expand=c["expand"], seed=seed, rng_counter=0)
    dt_s = time.perf_counter() - t0
    return {"value": Ls / dt_s, "unit": "verified tokens/s", "cores": threads, "kind": "oracle",
            "sample": "batch element 0, one %d-token block (%d grid rows) at P=%d of workload %s, all %d layers, "
                      "float64; %.1f s including the per-call bf16->float64 weight conversion" % (
                          Ls, h_blk * c["r"], P, c["name"], nl, dt_s)}


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
        "config": {"workload": "%s: last block, B=%d L=%d P=%d, rejection rate %g, radius 1" % (c["name"], B, L, P, rate)},
        "marked_positions": int(mask.sum()), "islands_per_sequence": cn[:, 0].tolist(), "largest_island": cn[:, 1].tolist(),
        "island_passes": passes, "slots_per_pass": B * cap, "sequential_steps": L - u_start,
        "ms_islands": round(ms_isl, 2), "ms_sequential": round(ms_seq, 2), "ms_single_token_step": round(ms_tok, 3),
        "ms_per_island_pass": round(ms_isl / max(passes, 1), 3)}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--sigma", type=float, default=None, help="draft-logit noise std (default: the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events")
    ap.add_argument("--profile-all", action="store_true",
                    help="bracket every kernel class (adds ~3 %% to the step); default: only the roofline kernel")
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

    import numpy as np
    import torch

    import paper_2601_05149_amd as mulo
    from paper_2601_05149_amd.binding import PROF_CLASSES
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
    B, L, V, seed = c["B"], c["L"], m["vocab"], c["seed"]
    sigma = a.sigma if a.sigma is not None else (c["sigma"] if c["sigma"] is not None else 1.0)
    P = c["max_seq"] - L                  # last block of the image: the largest cache
    n0 = c["T"] - L
    h_blk = L // c["W"] // c["r"]
    n_lo = h_blk * c["w"]

    log("workload %s: B=%d L=%d P=%d V=%d; generating weights ..." % (c["name"], B, L, P, V))
    w = G.make_weights(m, seed=seed)
    cos, sin = G.rope_table(c["max_seq"], m["head_dim"])
    wd = {k: v.to(dev) for k, v in w.items()}
    cfg = mulo.make_cfg(m, B, c["max_seq"], L)
    ctx = mulo.mulo_create(cfg, wd, torch.tensor(cos, device=dev), torch.tensor(sin, device=dev))
    kv = mulo.alloc_kv(ctx, dev)
    # cache rows [0, P): seeded N(0, 1) values (a stand-in for the prefilled prefix + committed blocks)
    gen = torch.Generator(device=dev).manual_seed(seed)
    kv[0][:, :, :, :P].normal_(generator=gen)
    kv[1][:, :, :, :, :P].normal_(generator=gen)

    if a.resample is not None:
        resample_bench(mulo, ctx, kv, c, B, L, P, V, a.resample, seed, gen)
        return

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
    draft_logits = (zp[:, child0, :] + sigma * torch.randn(B, n_lo, V, generator=gen, device=dev)).contiguous()
    gumbel = -torch.log(-torch.log(torch.rand(B, n_lo, V, generator=gen, device=dev).clamp_min(1e-20)))
    draft_tokens = (draft_logits + gumbel).argmax(-1).to(torch.int32).contiguous()
    del zp, gumbel, q_lo

    out = dict(tokens_out=torch.empty(B, L, dtype=torch.int32, device=dev),
               accept=torch.empty(B, L, dtype=torch.uint8, device=dev),
               mask=torch.empty(B, L, dtype=torch.uint8, device=dev),
               t0=torch.empty(B, dtype=torch.int32, device=dev),
               stats=torch.empty(B, 4, dtype=torch.int32, device=dev))

    def step(i):
        params = mulo.make_params(c["H"], c["W"], n0, L, c["radius"], c["expand"], seed=seed, rng_counter=i)
        mulo.mulo_verify_step(ctx, kv, B, P, params, h_blk, c["w"], r, draft_logits, 0, draft_tokens, prev,
                              out["tokens_out"], out["accept"], out["mask"], out["t0"], out["stats"])

    log("warm-up ...")
    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    if not a.no_profile:
        mulo.mulo_profile(ctx, 1 if a.profile_all else 0x100 | PROF_CLASSES.index("gemm_gate_up"))
    # per-step marks on the library's stream (torch's current one): recorded, not waited for, inside the timed region
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(a.steps + 1)]
    t_start = time.perf_counter()
    marks[0].record()
    for i in range(a.steps):
        step(a.warmup + i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt_s = time.perf_counter() - t_start
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(a.steps))
    prof = mulo.mulo_profile_read(ctx) if not a.no_profile else {}
    mulo.mulo_profile(ctx, 0)
    ms_per_step = 1e3 * dt_s / a.steps
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
            "accept": 4.0 * V * M,                        # logits once
            "mask_sample": 8.0 * V * M * marked}          # logits + draft row of every marked position
    kernels = {}
    for name, (ms, n) in prof.items():
        if n == 0:
            continue
        avg = ms / n
        e = {"avg_ms": round(avg, 4), "launches_per_step": n / a.steps}
        if name in flops:
            e.update(bound="mfma", achieved=round(flops[name] / (avg * 1e-3) / 1e12, 1), unit="TFLOP/s")
            e["frac"] = round(e["achieved"] / PEAK_BF16_TFLOPS, 4)
            if name == "attention":   # K and V rows of every (sequence, head) read once per launch
                kv_bytes = 2.0 * 2 * d * B * (P + L)
                e["kv_gbs"] = round(kv_bytes / (avg * 1e-3) / 1e9, 1)
        elif name in byts:
            e.update(bound="hbm", achieved=round(byts[name] / (avg * 1e-3) / 1e9, 1), unit="GB/s")
            e["frac"] = round(e["achieved"] / PEAK_HBM_GBS, 4)
        kernels[name] = e
    # HBM bytes per launch of the roofline kernel: FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 (KiB per dispatch, scale
    # factors from the --calibrate-copy runs) of two rocprofv3 --pmc runs of this benchmark; a stored measurement,
    # summarised in profiles/verify_step_cfg4_hbm_traffic.md (both kernels of the projection, the 256x256-tile one and the
    # 128x256-tile one for the sparse last round: 1007.9 + 134.3 MB fetched, 87.0 + 6.3 MB written)
    measured_traffic = {"cfg4": 1.2355e9}
    roof = None
    if "gemm_gate_up" in kernels:
        k = kernels["gemm_gate_up"]
        roof = {"bound": "mfma", "kernel": "k_gemm_bf16<EPI_SWIGLU> (gate|up projection + SwiGLU)",
                "achieved": k["achieved"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": k["frac"],
                "traffic": measured_traffic.get(c["name"]), "avg_ms": k["avg_ms"], "flops_per_launch": flops["gemm_gate_up"]}
    fwd_flops = nl * (flops["gemm_qkv"] + flops["gemm_out"] + flops["gemm_gate_up"] + flops["gemm_down"]
                      + flops["attention"]) + flops["gemm_lm_head"]

    res = {"metric": "verified image tokens/sec (1 GPU) per verify step", "value": round(M / (ms_per_step * 1e-3), 1),
           "unit": "tokens/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(ms_per_step, 3),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": m["dtype"], "data": "synthetic",
           "config": {"workload": "%s: %s decoder, B=%d, draft block L=%d of a %dx%d grid (last block, P=%d cache rows), "
                                  "V=%d, radius %d, sigma %.2g" % (c["name"], c["model_name"], B, L, c["H"], c["W"], P, V,
                                                                    c["radius"], sigma),
                      "acceptance_rate": round(acc_rate, 4), "marked_fraction": round(marked, 4)},
           "accepted_tokens_per_s": round(M * (1.0 - marked) / (ms_per_step * 1e-3), 1),
           "ms_per_step_median": round(per_step[len(per_step) // 2], 3), "ms_per_step_min": round(per_step[0], 3),
           "step_tflops": round(fwd_flops / (ms_per_step * 1e-3) / 1e12, 1),
           "step_frac_of_bf16_peak": round(fwd_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
           "roofline": roof, "kernels": kernels}
    if a.no_cpu_baseline:
        res["cpu_baseline"] = None
    else:
        log("timing the CPU oracle on a bounded sample ...")
        del ctx
        res["cpu_baseline"] = cpu_baseline(c, w, cos, sin, seed)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
