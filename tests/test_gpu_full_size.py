"""The 7B-class benchmark shapes at full depth, width, vocabulary and batch, in the launch configuration bench.py
times (fused / tile kernels, replayed graph): properties that hold at any size.  (The comparison of these shapes
with the oracle at full depth, and the stated tolerance, are in test_gpu_full_depth_oracle.py.)
  * a step is reproducible bit for bit (restore the state saved before it and run it again), verdicts included;
  * the fused path is no further from the library's fp32 mode (plain fp32 kernels on the same bf16-valued weights) than
    an independent bf16 implementation of the same forward, the plain reference kernels (`KERNELS_REFERENCE`: no
    MFMA, separate normalisation / rotary / SwiGLU kernels): its distance is the storage format's, not the kernels'.
Decisions at these vocabulary sizes are compared with the oracle in test_gpu_decide.py.
"""
import numpy as np
import pytest

import workload
from helpers import logits_error

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,S", [("cfg2", 1), ("cfg3", 1), ("cfg4", 8)])
def test_full_size_step_against_the_fp32_path(name, S):
    import torch
    import paper_2512_07503_amd as sjd
    from workload.generate import make_weights_torch
    cfg = workload.get_config(name)
    arch = dict(cfg["arch"])
    L, P, N = cfg["window"], 48, 96
    weights = make_weights_torch(arch, cfg["seed"], cfg["head_alpha"], "cuda", torch.bfloat16)
    cond, uncond = workload.make_prompts(arch, cfg["seed"], S, P)

    def decoder(flags, dtype, w):
        d = sjd.Decoder(arch, w, dtype, L, P + N, max_seqs=S, cfg_scale=cfg["cfg_scale"], temperature=cfg["temperature"],
                        top_k=cfg["top_k"], reuse_tau=cfg["tau"], seed=cfg["seed"], kernel_flags=flags | sjd.KEEP_LOGITS)
        assert d.prefill(cond, uncond, [N] * S) == 0
        return d

    g = decoder(0, "bf16", weights)
    les = [g.window(s)[2] for s in range(S)]
    snap = g.snapshot()
    res = g.step()
    got = g.logits()
    assert np.isfinite(got).all()
    # the same step again from the saved state: identical bits
    g.restore(snap)
    assert g.step() == res
    assert np.array_equal(g.logits(), got)
    del g
    r = decoder(sjd.KERNELS_REFERENCE, "bf16", weights)
    r.step()
    plain = r.logits()
    del r
    w32 = {k: ([t.float() for t in v] if isinstance(v, list) else v.float()) for k, v in weights.items()}
    del weights
    f = decoder(0, "f32", w32)
    f.step()
    want = f.logits()
    err_fused, err_plain = logits_error(got, want, les), logits_error(plain, want, les)
    print(name, "worst |d| / max|logit| of a row against fp32: fused", err_fused[1], "plain bf16 kernels", err_plain[1])
    assert err_fused[1] <= 1.1 * err_plain[1], (err_fused, err_plain)
