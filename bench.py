#!/usr/bin/env python3
"""Benchmark of the SJD++ decoding path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--config cfg1]

A "step" is one sjd_step: one causal forward over the Jacobi window (conditional + unconditional branch) plus
verification, residual resampling and reuse.  W untimed steps, then exactly K timed steps (a finished image is
re-prefilled outside the timed region); one JSON line on stdout.  Inputs are synthetic: random-init weights of the
named shape and random prompts, resident in HBM before the timed region starts.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0


def gemm_shapes(arch, M):
    d, H, Hkv, F = arch["d_model"], arch["n_heads"], arch["n_kv_heads"], arch["d_ff"]
    hd = d // H
    Vs = arch["sample_hi"] - arch["sample_lo"]
    return {"gemm_qkv": (M, (H + 2 * Hkv) * hd, d), "gemm_out": (M, d, H * hd), "gemm_gate_up": (M, 2 * F, d),
            "gemm_down": (M, d, F), "gemm_head": (M, Vs, d)}


def algorithmic_bytes(name, cfg, M, mean_ctx):
    """Bytes one launch of a kernel class must move at least once (weights / KV / logits once, operands once)."""
    arch = cfg["arch"]
    esz = 4 if cfg["dtype"] == "f32" else 2
    shapes = gemm_shapes(arch, M)
    if name in shapes:
        m, n, k = shapes[name]
        return n * k * esz + m * k * esz + m * n * 4
    hd = arch["d_model"] // arch["n_heads"]
    if name == "window_attention":
        segs = M // cfg["window"]
        return 2 * mean_ctx * arch["n_kv_heads"] * hd * esz * segs
    if name == "sample_rows":
        Vs = arch["sample_hi"] - arch["sample_lo"]
        return (M // 2) * Vs * 4 * 3          # two logit rows in, one weight row out, per position
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="cfg1")
    ap.add_argument("--trace-steps", type=int, default=20)
    ap.add_argument("--trace-skip", type=int, default=0,
                    help="untimed steps between the prefill and the traced steps: per-kernel durations deep in the image "
                         "(long cache) instead of at its start")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference dispatch for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; sequences are independent and would shard by prompt with no "
              "communication, but no multi-GPU path exists here. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workload
    from workload.generate import make_weights_torch
    import paper_2512_07503_amd as sjd

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calib_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")   # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    cfg = workload.get_config(args.config)
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
                      kernel_flags=args.kernel_flags, init_mode=args.init_mode,
                      row_width=args.row_width or int(round(N ** 0.5)))
    host_weights = None
    if not args.no_cpu_baseline:
        host_weights = {k: ([t.float().cpu().numpy() for t in v] if isinstance(v, list) else v.float().cpu().numpy())
                        for k, v in weights.items()}
    del weights
    torch.cuda.empty_cache()
    setup_s = time.time() - t0

    from paper_2512_07503_amd.binding import StepResult
    res = (StepResult * S)()

    def prefill():
        rc = dec.prefill(cond, uncond, [N] * S)
        assert rc == 0, rc

    # ---- W warm-up steps, then exactly K timed steps
    prefill()
    images_steps, cur_steps = [], 0
    timed_steps, timed_tokens, timed_s = 0, 0, 0.0
    accepted_hist = []
    kv_sum = 0
    done_warm = 0
    tokens_done = [0] * S
    while timed_steps < args.steps:
        warm = done_warm < args.warmup
        budget = (args.warmup - done_warm) if warm else (args.steps - timed_steps)
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
                    kv_sum += P - 1 + tokens_done[s]
                    tokens_done[s] += res[s].n_finalized
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
            tokens_done = [0] * S
            prefill()
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
    for _ in range(args.trace_skip):
        dec.step_raw(res)
        for s in range(S):
            tokens_done[s] += res[s].n_finalized
        if all(res[s].done for s in range(S)):
            break
    dec.trace(True)
    dec.trace_reset()
    traced, mean_ctx_sum = 0, 0
    for _ in range(args.trace_steps):
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
    kernels = {}
    for name, (launches, total_ms) in tr.items():
        if launches == 0 or traced == 0:
            continue
        avg_ms = total_ms / launches
        entry = {"launches_per_step": launches / traced, "avg_us": round(1e3 * avg_ms, 2),
                 "ms_per_step": round(total_ms / traced, 4)}
        ab = algorithmic_bytes(name, cfg, M, mean_ctx)
        if ab:
            entry["GBps"] = round(ab / (avg_ms * 1e-3) / 1e9, 1)
        if name.startswith("gemm"):
            m, n, k = gemm_shapes(arch, M)[name]
            entry["TFLOPs"] = round(2.0 * m * n * k / (avg_ms * 1e-3) / 1e12, 2)
        kernels[name] = entry
    roofline = None
    dominant = max(kernels, key=lambda n: kernels[n]["ms_per_step"]) if kernels else None
    dom = kernels.get(dominant)
    if dom: roofline = {"kernel": dominant, "bound": "hbm", "achieved": dom.get("GBps"), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(dom["GBps"] / HBM_PEAK_GBS, 4) if dom.get("GBps") else None, "traffic": None,
                "avg_us": dom["avg_us"], "launches_per_step": dom["launches_per_step"]}
    if dom:
        try:   # HBM bytes per launch measured with rocprofv3 --pmc (profiles/pmc_traffic.json), if this config has them
            pmc = json.load(open(os.path.join(ROOT, "profiles", "pmc_traffic.json"))).get(args.config, {}).get("kernels", {})
            key = dominant if dominant in pmc else None
            if key:
                roofline["traffic"] = pmc[key]["fetch_bytes"] + pmc[key]["write_bytes"]
                roofline["traffic_source"] = "rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE scaled by a 256 MiB copy; bytes per launch"
        except (OSError, ValueError, KeyError):
            pass
        roofline["algorithmic_bytes"] = algorithmic_bytes(dominant, cfg, M, mean_ctx)
    if dom and dominant.startswith("gemm") and M >= 320:      # above the ridge (~312 flop/B) the contraction is MFMA-bound
        roofline.update({"bound": "mfma", "achieved": dom["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(dom["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4)})
    esz = 4 if cfg["dtype"] == "f32" else 2
    shp = gemm_shapes(arch, M)
    step_weight_bytes = esz * (arch["n_layers"] * sum(shp[g][1] * shp[g][2] for g in ("gemm_qkv", "gemm_out", "gemm_gate_up", "gemm_down"))
                               + shp["gemm_head"][1] * shp["gemm_head"][2])
    step_floor_ms = 1e3 * step_weight_bytes / (HBM_PEAK_GBS * 1e9)

    # ---- CPU baseline: the oracle as it stands, on this machine's host cores, bounded sample
    cpu_baseline = None
    if host_weights is not None:
        from oracle import oracle
        cores = oracle.set_num_threads(0)
        sample_prompt = min(P, 8)
        o = oracle.Oracle(arch, host_weights, L, sample_prompt + N, cfg_scale=cfg["cfg_scale"], top_k=cfg["top_k"],
                          reuse_tau=cfg["tau"], seed=cfg["seed"], max_seqs=S)
        c2 = [c[-sample_prompt:] for c in cond]
        u2 = [u[-sample_prompt:] for u in uncond]
        print(f"cpu baseline: oracle prefill + steps on {cores} threads ...", file=sys.stderr, flush=True)
        tc = time.perf_counter()
        o.prefill(c2, u2, [N] * S)
        n_cpu, tok_cpu = 0, 0
        t_steps = time.perf_counter()
        while True:
            r = o.step()
            n_cpu += 1
            print(f"cpu baseline: step {n_cpu} done after {time.perf_counter() - tc:.0f} s", file=sys.stderr, flush=True)
            tok_cpu += sum(x["n_finalized"] for x in r)
            el = time.perf_counter() - tc
            if (args.cpu_steps and n_cpu >= args.cpu_steps) or (not args.cpu_steps and el > 15.0) or all(x["done"] for x in r):
                break
        t_cpu = time.perf_counter() - t_steps
        cpu_baseline = {"value": round(tok_cpu / t_cpu, 3), "unit": "image tokens/s", "cores": cores, "kind": "oracle",
                        "ms_per_step": round(1e3 * t_cpu / n_cpu, 1),
                        "sample": f"{n_cpu} oracle steps of the same workload after a {sample_prompt}-token prompt "
                                  f"(context {sample_prompt - 1}..), double precision"}
        o.close()

    out = {
        "metric": "image tokens/sec/GPU", "value": round(tokens_per_s, 2), "unit": "image tokens/s", "n_gpus": 1,
        "steps": timed_steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": f"{args.config}: {arch['n_layers']} layers, d_model {arch['d_model']}, {arch['n_heads']} heads "
                               f"({arch['n_kv_heads']} kv), d_ff {arch['d_ff']}, sampled vocab {arch['sample_hi'] - arch['sample_lo']}, "
                               f"prompt {P}, {N} image tokens x {S} seq, window {L}, top-k {cfg['top_k']}, CFG {cfg['cfg_scale']}, "
                               f"tau {cfg['tau']}, random-init weights",
                   "window": L, "n_seqs": S, "gemm_rows": M, "head_alpha": round(cfg["head_alpha"], 4),
                   "head_alpha_calibrated": cfg["head_alpha_calibrated"]},
        "forwards_per_image": round(forwards_per_image, 2) if forwards_per_image else None,
        "tokens_per_step": round(float(np.mean(accepted_hist)) + 1.0, 4) if accepted_hist else None,
        "step_floor_ms_weights_at_hbm_peak": round(step_floor_ms, 4),
        "roofline": roofline, "cpu_baseline": cpu_baseline, "kernels": kernels, "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
