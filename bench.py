#!/usr/bin/env python3
"""Benchmark of the SJD++ decoding path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--config cfg4]

A "step" is one sjd_step: one causal forward over the Jacobi window (conditional + unconditional branch) plus
verification, residual resampling and reuse.  W untimed steps, then exactly K timed steps (a finished image is
re-prefilled outside the timed region); one JSON line on stdout.  Inputs are synthetic: random-init weights of the
named shape and random prompts, resident in HBM before the timed region starts.

The headline workload is the largest configuration that one GPU holds (cfg4: the 7B shape, 8 prompts decoded
together, 512 GEMM rows).  Without --config the line also carries, under "all_configs", one whole image of every
smaller configuration (cfg0 .. cfg3), timed from its first to its last step.
"""
import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VECTOR_PEAK_TFLOPS = 157.3
HEADLINE = "cfg4"
SECONDARY = ("cfg0", "cfg1", "cfg2", "cfg3")


def gemm_shapes(arch, M):
    d, H, Hkv, F = arch["d_model"], arch["n_heads"], arch["n_kv_heads"], arch["d_ff"]
    hd = d // H
    Vs = arch["sample_hi"] - arch["sample_lo"]
    return {"gemm_qkv": (M, (H + 2 * Hkv) * hd, d), "gemm_out": (M, d, H * hd), "gemm_gate_up": (M, 2 * F, d),
            "gemm_down": (M, d, F), "gemm_head": (M, Vs, d)}


def library_gemm_us(cfg, M, repeats=30):
    """The vendor library's bf16 GEMM (torch.matmul) at the configuration's five projection shapes: normal random
    operands, six weight matrices in rotation so that none is served from a cache, HIP-event time per call.  Context for
    the MFMA-bound kernels' numbers: the plain product only, none of what the path's kernels fold into theirs (RMSNorm
    scaling, rotary embedding and KV page writes, SwiGLU, guidance), under the same power limit."""
    import torch
    out = {}
    for name, (m, n, k) in gemm_shapes(cfg["arch"], M).items():
        a = torch.randn(m, k, device="cuda", dtype=torch.bfloat16)
        ws = [torch.randn(n, k, device="cuda", dtype=torch.bfloat16) for _ in range(6)]
        for w in ws:
            a @ w.t()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(repeats):
            a @ ws[i % 6].t()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / repeats
        out[name] = {"shape_mnk": [m, n, k], "avg_us": round(us, 2), "tflops": round(2.0 * m * n * k / us / 1e6, 1)}
        del a, ws
    return out


def head_is_fused(cfg, M):
    """The vocabulary head combines the two guidance branches itself (one fp32 row per position instead of two) on the
    bf16 fused path for windows of 32 and for one sequence with a window of 16."""
    arch = cfg["arch"]
    return cfg["dtype"] == "bf16" and (arch["d_model"] // arch["n_heads"]) % 64 == 0 and (cfg["window"] == 32 or (cfg["window"] == 16 and M == 32))


def algorithmic_bytes(name, cfg, M, mean_ctx, sparse_rows):
    """Bytes one launch of a kernel class must move at least once (weights / KV / logits once, operands once)."""
    arch = cfg["arch"]
    esz = 4 if cfg["dtype"] == "f32" else 2
    shapes = gemm_shapes(arch, M)
    fused = sparse_rows and head_is_fused(cfg, M)
    if name in shapes:
        m, n, k = shapes[name]
        out_rows = m // 2 if (name == "gemm_head" and fused) else m
        return n * k * esz + m * k * esz + out_rows * n * 4
    hd = arch["d_model"] // arch["n_heads"]
    if name == "window_attention":
        segs = M // cfg["window"]
        return 2 * mean_ctx * arch["n_kv_heads"] * hd * esz * segs
    if name == "sample_rows":
        Vs = arch["sample_hi"] - arch["sample_lo"]
        # in: two logit rows per position, or the one row of guided logits the fused head wrote; out: the dense weight
        # row, or the kept (id, weight) pairs (8 bytes each)
        out = min(cfg["top_k"], Vs) * 8 if sparse_rows else Vs * 4
        return (M // 2) * (Vs * 4 * (1 if fused else 2) + out)
    return None


def kernel_rooflines(kernels, cfg, M, mean_ctx, sparse_rows):
    """Per kernel class: which roofline bounds it (the larger of bytes / HBM peak and flops / matrix-core peak), the
    algorithmic bytes or flops of one launch, what the launch achieved and the fraction of that peak."""
    arch = cfg["arch"]
    out = {}
    for name, k in kernels.items():
        t = k["avg_us"] * 1e-6
        ab = algorithmic_bytes(name, cfg, M, mean_ctx, sparse_rows)
        if not ab or t <= 0:
            out[name] = {"bound": "latency", "avg_us": k["avg_us"]}
            continue
        r = {"bound": "hbm", "algorithmic_bytes": int(ab), "achieved": round(ab / t / 1e9, 1), "peak": HBM_PEAK_GBS,
             "unit": "GB/s", "avg_us": k["avg_us"]}
        if name.startswith("gemm"):
            m, n, kk = gemm_shapes(arch, M)[name]
            flops = 2.0 * m * n * kk
            peak = MFMA_BF16_PEAK_TFLOPS if cfg["dtype"] == "bf16" else FP32_VECTOR_PEAK_TFLOPS
            r["flops"] = flops
            r["TFLOPs"] = round(flops / t / 1e12, 2)
            r["mfma_frac" if cfg["dtype"] == "bf16" else "alu_frac"] = round(flops / t / 1e12 / peak, 4)
            r["hbm_frac"] = round(ab / t / 1e9 / HBM_PEAK_GBS, 4)
            if flops / (peak * 1e12) > ab / (HBM_PEAK_GBS * 1e9):    # above the ridge the contraction bounds the launch
                r.update({"bound": "mfma" if cfg["dtype"] == "bf16" else "alu", "achieved": r["TFLOPs"], "peak": peak,
                          "unit": "TFLOP/s"})
        r["frac"] = round(r["achieved"] / r["peak"], 4)
        out[name] = r
    return out


def run_config(name, args, steps, warmup, trace_steps, whole_image, overrides=True, keep_host_weights=False):
    """Builds the synthetic model of configuration `name`, decodes, and returns (result dict, host weights or None).
    whole_image: time every step of one image (steps is ignored); else exactly `steps` steps after `warmup`."""
    import numpy as np
    import torch
    import workload
    from workload.generate import make_weights_torch
    import paper_2512_07503_amd as sjd
    from paper_2512_07503_amd.binding import StepResult

    cfg = workload.get_config(name)
    if overrides:
        if args.window: cfg["window"] = args.window
        if args.n_seqs: cfg["n_seqs"] = args.n_seqs
        if args.tau is not None: cfg["tau"] = args.tau
        if args.top_k: cfg["top_k"] = args.top_k
    arch, L, S, N, P = cfg["arch"], cfg["window"], cfg["n_seqs"], cfg["n_image"], cfg["prompt_len"]
    M = S * 2 * L
    tdtype = torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16
    t0 = time.time()
    weights = make_weights_torch(arch, cfg["seed"], cfg["head_alpha"], "cuda", tdtype)
    cond, uncond = workload.make_prompts(arch, cfg["seed"], S, P)
    dec = sjd.Decoder(arch, weights, cfg["dtype"], L, P + N, max_seqs=S, cfg_scale=cfg["cfg_scale"],
                      temperature=cfg["temperature"], top_k=cfg["top_k"], reuse_tau=cfg["tau"], seed=cfg["seed"],
                      kernel_flags=args.kernel_flags if overrides else 0, init_mode=args.init_mode if overrides else 0,
                      row_width=(args.row_width if overrides else 0) or int(round(N ** 0.5)))
    host_weights = None
    if keep_host_weights:
        host_weights = {k: ([t.float().cpu().numpy() for t in v] if isinstance(v, list) else v.float().cpu().numpy())
                        for k, v in weights.items()}
    del weights
    torch.cuda.empty_cache()
    setup_s = time.time() - t0
    res = (StepResult * S)()

    def prefill():
        rc = dec.prefill(cond, uncond, [N] * S)
        assert rc == 0, rc

    # ---- W warm-up steps, then exactly K timed steps (or every step of one image)
    prefill()
    images_steps, cur_steps = [], 0
    timed_steps, timed_tokens, timed_s = 0, 0, 0.0
    accepted_hist = []
    done_warm = 0
    if whole_image:
        for _ in range(warmup):
            assert dec.step_raw(res) == 0
        prefill()
        warmup_left, steps = 0, 1 << 30
    else:
        warmup_left = warmup
    while timed_steps < steps:
        warm = done_warm < warmup_left
        budget = (warmup_left - done_warm) if warm else (steps - timed_steps)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        n_here, tok_here, finished = 0, 0, False
        while n_here < budget and not finished:
            rc = dec.step_raw(res)
            assert rc == 0, rc
            n_here += 1
            cur_steps += 1
            finished = True
            for s in range(S):
                tok_here += res[s].n_finalized
                if res[s].n_finalized:
                    accepted_hist.append(res[s].n_accepted)
                finished = finished and bool(res[s].done)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        if warm:
            done_warm += n_here
        else:
            timed_steps += n_here
            timed_tokens += tok_here
            timed_s += dt
        if finished:
            images_steps.append(cur_steps)
            cur_steps = 0
            prefill()
            if whole_image:
                break
    ms_per_step = 1e3 * timed_s / timed_steps
    tokens_per_s = timed_tokens / timed_s
    if not images_steps and not args.no_finish_image:   # finish the image (untimed) to know the forwards per image
        while True:
            dec.step_raw(res)
            cur_steps += 1
            if all(res[s].done for s in range(S)):
                break
        images_steps.append(cur_steps)
        prefill()
    forwards_per_image = float(np.mean(images_steps)) if images_steps else None

    # ---- per-kernel durations with HIP events on the library's stream, right after the timed region
    tokens_done = [0] * S
    for _ in range(args.trace_skip if overrides else 0):
        dec.step_raw(res)
        for s in range(S):
            tokens_done[s] += res[s].n_finalized
        if all(res[s].done for s in range(S)):
            break
    kernels, mean_ctx, traced = {}, P - 1, 0
    if trace_steps > 0:
        dec.trace(True)
        dec.trace_reset()
        mean_ctx_sum = 0
        for _ in range(trace_steps):
            mean_ctx_sum += P - 1 + tokens_done[0]
            dec.step_raw(res)
            traced += 1
            for s in range(S):
                tokens_done[s] += res[s].n_finalized
            if all(res[s].done for s in range(S)):
                break
        dec.trace(False)
        tr = dec.trace_read()
        mean_ctx = mean_ctx_sum / max(traced, 1)
        for kname, (launches, total_ms) in tr.items():
            if launches == 0 or traced == 0:
                continue
            kernels[kname] = {"launches_per_step": launches / traced, "avg_us": round(1e3 * total_ms / launches, 2),
                              "ms_per_step": round(total_ms / traced, 4)}
    sparse_rows = bool(getattr(dec, "sparse_rows", False))
    rooflines = kernel_rooflines(kernels, cfg, M, mean_ctx, sparse_rows)
    esz = 4 if cfg["dtype"] == "f32" else 2
    shp = gemm_shapes(arch, M)
    step_weight_bytes = esz * (arch["n_layers"] * sum(shp[g][1] * shp[g][2] for g in ("gemm_qkv", "gemm_out", "gemm_gate_up", "gemm_down"))
                               + shp["gemm_head"][1] * shp["gemm_head"][2])
    step_flops = 2.0 * M * step_weight_bytes / esz
    out = {
        "name": name, "cfg": cfg, "M": M, "dtype": cfg["dtype"],
        "workload": f"{name}: {arch['n_layers']} layers, d_model {arch['d_model']}, {arch['n_heads']} heads "
                    f"({arch['n_kv_heads']} kv), d_ff {arch['d_ff']}, sampled vocab {arch['sample_hi'] - arch['sample_lo']}, "
                    f"prompt {P}, {N} image tokens x {S} seq, window {L}, top-k {cfg['top_k']}, CFG {cfg['cfg_scale']}, "
                    f"tau {cfg['tau']}, random-init weights",
        "tokens_per_s": tokens_per_s, "ms_per_step": ms_per_step, "timed_steps": timed_steps,
        "forwards_per_image": forwards_per_image,
        "tokens_per_step": float(np.mean(accepted_hist)) + 1.0 if accepted_hist else None,
        "step_floor_ms_weights_at_hbm_peak": 1e3 * step_weight_bytes / (HBM_PEAK_GBS * 1e9),
        "step_floor_ms_gemm_flops_at_mfma_peak": 1e3 * step_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12) if cfg["dtype"] == "bf16" else None,
        "kernels": kernels, "rooflines": rooflines, "mean_ctx": mean_ctx, "setup_s": setup_s,
        "cond": cond, "uncond": uncond,
    }
    dec.close()
    del dec
    torch.cuda.empty_cache()
    return out, host_weights


def cpu_baseline_of(r, host_weights, args):
    """The oracle as it stands, on this machine's host cores, on a bounded sample of the same workload."""
    from oracle import oracle
    cfg = r["cfg"]
    arch, L, N = cfg["arch"], cfg["window"], cfg["n_image"]
    cores = oracle.set_num_threads(0)
    sample_prompt = min(cfg["prompt_len"], 8)
    big = arch["n_layers"] * arch["d_model"] >= 100000          # the 7B shapes: one sequence, one or two steps
    S = 1 if big else cfg["n_seqs"]
    o = oracle.Oracle(arch, host_weights, L, sample_prompt + N, cfg_scale=cfg["cfg_scale"], top_k=cfg["top_k"],
                      reuse_tau=cfg["tau"], seed=cfg["seed"], max_seqs=S)
    c2 = [c[-sample_prompt:] for c in r["cond"][:S]]
    u2 = [u[-sample_prompt:] for u in r["uncond"][:S]]
    print(f"cpu baseline: oracle prefill + steps on {cores} threads ...", file=sys.stderr, flush=True)
    tc = time.perf_counter()
    o.prefill(c2, u2, [N] * S)
    print(f"cpu baseline: prefill done after {time.perf_counter() - tc:.0f} s", file=sys.stderr, flush=True)
    n_cpu, tok_cpu = 0, 0
    t_steps = time.perf_counter()
    while True:
        res = o.step()
        n_cpu += 1
        print(f"cpu baseline: step {n_cpu} done after {time.perf_counter() - tc:.0f} s", file=sys.stderr, flush=True)
        tok_cpu += sum(x["n_finalized"] for x in res)
        el = time.perf_counter() - tc
        if (args.cpu_steps and n_cpu >= args.cpu_steps) or (not args.cpu_steps and el > 15.0) or all(x["done"] for x in res):
            break
    t_cpu = time.perf_counter() - t_steps
    o.close()
    return {"value": round(tok_cpu / t_cpu, 3), "unit": "image tokens/s", "cores": cores, "kind": "oracle",
            "ms_per_step": round(1e3 * t_cpu / n_cpu, 1),
            "sample": f"{n_cpu} oracle step(s) of {S} of the workload's {cfg['n_seqs']} sequence(s) after a "
                      f"{sample_prompt}-token prompt (context {sample_prompt - 1}..), double precision"}


def stored_traffic(config, kernel):
    """HBM bytes per launch measured with rocprofv3 --pmc (profiles/pmc_traffic.json) and the commit they were taken on."""
    try:
        table = json.load(open(os.path.join(ROOT, "profiles", "pmc_traffic.json"))).get(config, {})
        k = table.get("kernels", {}).get(kernel)
        if k:
            return k["fetch_bytes"] + k["write_bytes"], table.get("commit")
    except (OSError, ValueError, KeyError):
        pass
    return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default=None, help="one configuration only (default: cfg4 as the headline plus one image of each smaller one)")
    ap.add_argument("--trace-steps", type=int, default=20)
    ap.add_argument("--trace-skip", type=int, default=0,
                    help="untimed steps between the prefill and the traced steps: per-kernel durations deep in the image "
                         "(long cache) instead of at its start")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true")
    ap.add_argument("--cpu-steps", type=int, default=0, help="oracle steps in the CPU baseline (0 = sized to ~20 s)")
    ap.add_argument("--kernel-flags", type=int, default=0)
    ap.add_argument("--n-seqs", type=int, default=0, help="override the configuration's number of prompts decoded together")
    ap.add_argument("--window", type=int, default=0, help="override the configuration's Jacobi window L (1 = plain autoregressive decoding)")
    ap.add_argument("--tau", type=float, default=None, help="override the reuse threshold (inf = SJD without token reuse, Eq. 6)")
    ap.add_argument("--top-k", type=int, default=0, help="override top-K (1 = greedy Jacobi decoding)")
    ap.add_argument("--init-mode", type=int, default=0,
                    help="initialisation of new window slots: 0 uniform, 1 repeat left, 2 repeat above, 3 / 4 resample from the distribution of the left / upper neighbour")
    ap.add_argument("--row-width", type=int, default=0, help="tokens per image row for --init-mode 2 and 4 (default: sqrt of the image tokens)")
    ap.add_argument("--no-finish-image", action="store_true", help="do not run the image to its end for forwards/image")
    ap.add_argument("--whole-image", action="store_true", help="time every step of one image instead of --steps steps")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the vendor library's bf16 GEMM at the headline configuration's projection shapes (key library_gemm)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference dispatch for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; sequences are independent and would shard by prompt with no "
              "communication, but no multi-GPU path exists here. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calib_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")   # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    headline = args.config or HEADLINE
    all_configs = None
    if args.config is None and not args.no_all_configs:
        all_configs = {}
        for name in SECONDARY:
            print(f"bench: one image of {name} ...", file=sys.stderr, flush=True)
            r, _ = run_config(name, args, steps=0, warmup=3, trace_steps=min(args.trace_steps, 10), whole_image=True, overrides=False)
            all_configs[name] = {
                "workload": r["workload"], "value": round(r["tokens_per_s"], 2), "unit": "image tokens/s",
                "ms_per_step": round(r["ms_per_step"], 4), "steps": r["timed_steps"], "timed": "every step of one image",
                "forwards_per_image": r["forwards_per_image"], "tokens_per_step": round(r["tokens_per_step"], 4),
                "gemm_rows": r["M"], "dtype": r["dtype"],
                "step_floor_ms_weights_at_hbm_peak": round(r["step_floor_ms_weights_at_hbm_peak"], 4),
                "rooflines": {k: v for k, v in r["rooflines"].items() if v["bound"] != "latency"},
            }
    print(f"bench: {headline}, {args.warmup} + {args.steps} steps ...", file=sys.stderr, flush=True)
    r, host_weights = run_config(headline, args, steps=args.steps, warmup=args.warmup, trace_steps=args.trace_steps,
                                 whole_image=args.whole_image, keep_host_weights=not args.no_cpu_baseline)
    cfg, kernels, rooflines = r["cfg"], r["kernels"], r["rooflines"]
    roofline = None
    dominant = max(kernels, key=lambda n: kernels[n]["ms_per_step"]) if kernels else None
    if dominant:
        roofline = dict(rooflines[dominant])
        roofline["kernel"] = dominant
        roofline["launches_per_step"] = kernels[dominant]["launches_per_step"]
        roofline["traffic"], commit = stored_traffic(headline, dominant)
        if roofline["traffic"] is not None:
            roofline["traffic_source"] = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this kernel and workload, scaled by the same "
                                          f"counter's reading of a 256 MiB copy; bytes per launch, measured at commit {commit}")
    for kname, k in kernels.items():
        k.update({x: y for x, y in rooflines.get(kname, {}).items() if x not in ("avg_us",)})
    cpu_baseline = cpu_baseline_of(r, host_weights, args) if host_weights is not None else None
    try:
        head_commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip() or None
    except OSError:
        head_commit = None

    out = {
        "metric": "image tokens/sec/GPU", "value": round(r["tokens_per_s"], 2), "unit": "image tokens/s", "n_gpus": 1,
        "steps": r["timed_steps"], "warmup": args.warmup, "ms_per_step": round(r["ms_per_step"], 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": r["workload"], "window": cfg["window"], "n_seqs": cfg["n_seqs"], "gemm_rows": r["M"],
                   "head_alpha": round(cfg["head_alpha"], 4), "head_alpha_calibrated": cfg["head_alpha_calibrated"]},
        "forwards_per_image": round(r["forwards_per_image"], 2) if r["forwards_per_image"] else None,
        "tokens_per_step": round(r["tokens_per_step"], 4) if r["tokens_per_step"] else None,
        "step_floor_ms_weights_at_hbm_peak": round(r["step_floor_ms_weights_at_hbm_peak"], 4),
        "step_floor_ms_gemm_flops_at_mfma_peak": round(r["step_floor_ms_gemm_flops_at_mfma_peak"], 4) if r["step_floor_ms_gemm_flops_at_mfma_peak"] else None,
        "roofline": roofline, "cpu_baseline": cpu_baseline, "kernels": kernels, "all_configs": all_configs,
        "setup_s": round(r["setup_s"], 1), "commit": head_commit,
    }
    if args.library_gemm and cfg["dtype"] == "bf16":
        out["library_gemm"] = library_gemm_us(cfg, r["M"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
