"""Calibrates the output-head multiplier of every workload so that the sampling distribution (after guidance,
temperature and top-K) has a mean entropy of 4 nats, and writes workload/head_alpha.json.

Uses only the CPU oracle: one forward of the conditional and the unconditional sequence (prompt + T uniformly random
image tokens) with an unscaled head; the head is linear, so scaling it by alpha scales the logits by alpha, and alpha
is found by bisection on the entropy of the oracle's own sampling rows.

    python -m oracle.calibrate_alpha cfg0 cfg1 [cfg2 cfg3]     (cfg4 shares cfg2's model)
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import workload  # noqa: E402
from oracle import oracle  # noqa: E402

OUT = os.path.join(ROOT, "workload", "head_alpha.json")
T = 12  # image positions whose distributions are averaged


def entropy_at(alpha, lc, lu, cfg):
    hs = []
    for k in range(lc.shape[0]):
        e, Z = oracle.sampling_row(lc[k] * np.float32(alpha), lu[k] * np.float32(alpha), cfg["cfg_scale"],
                                   cfg["temperature"], cfg["top_k"])
        p = e[e > 0].astype(np.float64)
        p /= p.sum()
        hs.append(float(-(p * np.log(p)).sum()))
    return float(np.mean(hs))


def calibrate(name, target=4.0):
    cfg = workload.get_config(name)
    arch = cfg["arch"]
    t0 = time.time()
    w = workload.make_weights(arch, cfg["seed"], 1.0, cfg["dtype"])
    cond, uncond = workload.make_prompts(arch, cfg["seed"], 1, cfg["prompt_len"])
    rng = np.random.Generator(np.random.Philox(key=cfg["seed"] + 3000))
    img = rng.integers(arch["sample_lo"], arch["sample_hi"], T, dtype=np.int32)
    print(f"{name}: weights ready after {time.time() - t0:.0f} s", flush=True)
    lc = oracle.forward_logits(arch, w, np.concatenate([cond[0], img]))[-T:]
    print(f"{name}: conditional forward done after {time.time() - t0:.0f} s", flush=True)
    lu = oracle.forward_logits(arch, w, np.concatenate([uncond[0], img]))[-T:]
    lo, hi = 1e-3, 1e3
    for _ in range(40):
        mid = (lo * hi) ** 0.5
        if entropy_at(mid, lc, lu, cfg) > target:
            lo = mid
        else:
            hi = mid
    alpha = (lo * hi) ** 0.5
    h = entropy_at(alpha, lc, lu, cfg)
    print(f"{name}: alpha {alpha:.4f} entropy {h:.3f} nats ({time.time() - t0:.0f} s)", flush=True)
    return alpha


def main():
    names = sys.argv[1:] or ["cfg0", "cfg1"]
    table = {}
    if os.path.exists(OUT):
        table = json.load(open(OUT))
    for n in names:
        table[n] = round(calibrate(n), 4)
        if n == "cfg2":
            table["cfg4"] = table[n]
        with open(OUT, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
            f.write("\n")


if __name__ == "__main__":
    main()
