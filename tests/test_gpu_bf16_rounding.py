"""bf16 mode against a CPU emulation of its own rounding points.

The oracle computes in double precision from the bf16 weight values, so in bf16 mode the GPU may differ from it by
what storing activations in bf16 costs (held to 3e-2 of a logits row's maximum in test_gpu_e2e.py).  This file
separates that format error from kernel error: a second, independent CPU forward (torch, double precision, written
here, not part of the oracle and not of the product) rounds to bf16 exactly where the fused GPU path stores bf16 --
the stream copy that feeds each projection, norm gains folded into the weights, the row scale taken from the rounded
stream, rotated queries / keys, values, attention probabilities and their sum, the attention output, the MLP hidden
activations and, in the attention, probabilities rounded relative to the running maximum of the 32-token blocks a
wavefront has walked -- and accumulates everything else in double.

What remains between it and the GPU is fp32 accumulation.  A projection output is a sum of some hundred products of
random sign, which fp32 gets right to about 1.6e-5 relative; a value that close to a bf16 rounding boundary (spacing
2^-8 relative) rounds the other way on the GPU than in double, which happens to roughly 0.8 % of all rounded values
and costs a whole ulp each time.  Against the +-half-ulp error that every rounded value carries anyway (the format
error, i.e. the distance to the double-precision oracle) these flips have sqrt(0.008 / 0.083) = 0.3 of the RMS.
That 0.3 is the first-order figure for one rounding point in isolation.  Through the layers it compounds: a stream in
which 0.8 % of the values sit one ulp off moves every projection output by sqrt(0.008) = 0.09 of the bf16 spacing of
its inputs, and an output that lands within that distance of a rounding boundary (twice 0.09 / 2 of all of them, i.e.
9 %, not 0.8 %) now also rounds the other way.  With 9 % flips of a whole ulp the same RMS ratio is
sqrt(0.09 / 0.083) = 1.04 per rounding point, diluted again by the sqrt(n) averaging of the next projection; the two
effects settle between the 0.3 of the first point and about half the format error, which is the 0.3-0.5 measured
(4e-3 to 8e-3 of a logits row's maximum).  The test compares maxima over the same logits, which for two near-Gaussian
fields scale by the same sqrt(2 ln N) and so keep the ratio.  The bound is 0.6: twice the isolated-point estimate, a
fifth above the largest ratio seen, and well below the 1.0 and more that an error outside the rounding model gives
(dropping any single rounding point from the emulation moves its logits by 2e-3 to 2e-2, i.e. by as much as the
whole distance to the oracle) -- together with the absolute bound of 1e-2 on the distance to the emulation.
"""
import numpy as np
import pytest

import workload
from helpers import make_pair

pytestmark = pytest.mark.gpu


def _emulated_logits(arch, w, tokens, running_max):
    """Causal forward over `tokens` with the GPU path's rounding points; returns [T][V_s] float64 logits.
    running_max: attention probabilities of a 32-token block are rounded relative to the largest score of the blocks
    up to it (one wavefront walks the context: the chunk + merge kernels) or of that block alone (one block per
    wavefront: the one-pass kernel at these context lengths)."""
    import torch
    f64 = torch.float64

    def t(a):
        return torch.from_numpy(np.asarray(a)).to(f64)

    def rb(x):  # round to nearest-even bf16, back to double
        return x.to(torch.float32).to(torch.bfloat16).to(f64)

    d, H, Hkv, F = arch["d_model"], arch["n_heads"], arch["n_kv_heads"], arch["d_ff"]
    hd, T, eps = d // H, len(tokens), arch["rms_eps"]
    x = t(w["tok_emb"])[torch.as_tensor(np.asarray(tokens), dtype=torch.long)]   # bf16 values already
    pos = torch.arange(T, dtype=f64)
    freq = torch.tensor(arch["rope_theta"], dtype=f64) ** (-2.0 * torch.arange(hd // 2, dtype=f64) / hd)
    ang = pos[:, None] * freq[None, :]
    cos, sin = torch.cos(ang).to(torch.float32).to(f64), torch.sin(ang).to(torch.float32).to(f64)   # fp32 tables

    def rope(v):  # [T][heads][hd], pairs (j, j + hd/2)
        a, b = v[..., : hd // 2], v[..., hd // 2:]
        c, s = cos[:, None, :], sin[:, None, :]
        return torch.cat([a * c - b * s, b * c + a * s], -1)

    def normed_linear(xb, W, gain):
        """(xb W'^T) * inv_rms with W' = bf16(W * gain) and inv_rms from the rounded stream, as the kernels do."""
        inv = 1.0 / torch.sqrt((xb * xb).mean(-1, keepdim=True) + eps)
        return (xb @ rb(t(W) * t(gain)[None, :]).T) * inv

    causal = torch.tril(torch.ones(T, T, dtype=torch.bool))
    for l in range(arch["n_layers"]):
        xb = rb(x)
        q = rb(rope(normed_linear(xb, w["wq"][l], w["attn_norm"][l]).view(T, H, hd)))
        k = rb(rope(normed_linear(xb, w["wk"][l], w["attn_norm"][l]).view(T, Hkv, hd)))
        v = rb(normed_linear(xb, w["wv"][l], w["attn_norm"][l]).view(T, Hkv, hd))
        k, v = k.repeat_interleave(H // Hkv, 1), v.repeat_interleave(H // Hkv, 1)
        s = torch.einsum("ihd,jhd->hij", q, k) / np.sqrt(hd)
        s = s.masked_fill(~causal[None], float("-inf"))
        m_all = s.amax(-1, keepdim=True)
        num, den, m_run = torch.zeros(H, T, hd, dtype=f64), torch.zeros(H, T, 1, dtype=f64), None
        for j0 in range(0, T, 32):
            sb = s[:, :, j0:j0 + 32]
            m_blk = sb.amax(-1, keepdim=True)
            m_run = m_blk if (m_run is None or not running_max) else torch.maximum(m_run, m_blk)
            m_use = torch.where(torch.isinf(m_run), torch.zeros_like(m_run), m_run)
            p = rb(torch.exp(sb - m_use))                           # probabilities as multiplied: bf16
            scale = torch.exp(m_use - m_all)                        # fp32 on the GPU, not rounded again
            num += torch.einsum("hij,jhd->hid", p, v[j0:j0 + 32]) * scale
            den += p.sum(-1, keepdim=True) * scale
        o = (num / den).transpose(0, 1)
        x = x + rb(o.reshape(T, H * hd)) @ t(w["wo"][l]).T
        xb = rb(x)
        g = normed_linear(xb, w["w_gate"][l], w["mlp_norm"][l])
        u = normed_linear(xb, w["w_up"][l], w["mlp_norm"][l])
        x = x + rb(g / (1.0 + torch.exp(-g)) * u) @ t(w["w_down"][l]).T
    head = np.asarray(w["lm_head"])[arch["sample_lo"]: arch["sample_hi"]]
    return normed_linear(rb(x), head, w["final_norm"]).numpy()


@pytest.mark.parametrize("name,layers,flags", [("small_fused64", None, 0), ("small_fused128", None, 0), ("small_fused64", None, 8),
                                               ("cfg1", 2, 0), ("cfg3", 1, 0)])
def test_bf16_logits_match_the_emulated_rounding_points(oracle, name, layers, flags):
    cfg = workload.get_config(name)
    arch = dict(cfg["arch"], n_layers=layers or cfg["arch"]["n_layers"])
    stress = name.startswith("small")
    w = workload.make_weights(arch, cfg["seed"], 6.0 if stress else cfg["head_alpha"], "bf16", std=0.08 if stress else 0.02,
                              random_gains=True)
    o, g, cond, uncond, n_img = make_pair(oracle, cfg, weights=w, n_layers=arch["n_layers"], n_seqs=1, kernel_flags=flags,
                                          prompt_len=min(cfg["prompt_len"], 40), n_image=min(cfg["n_image"], 64))
    worst_emul, worst_oracle = 0.0, 0.0
    for step in range(3):
        toks, _, Le = g.window(0)
        final = g.tokens(0)
        want_oracle = o.peek_logits()
        g.step()
        got = g.logits()
        o.step_from_logits(got)
        for b, prompt in enumerate((cond[0], uncond[0])):
            # the branch's whole sequence: prompt, image tokens final so far (the last one is the anchor), drafts
            seq = list(prompt) + list(final) + [int(x) for x in toks[1:Le]]
            ref = _emulated_logits(arch, w, seq, running_max=bool(flags & 8))[len(seq) - Le:]
            for k in range(Le):
                scale = np.abs(ref[k]).max()
                worst_emul = max(worst_emul, float(np.abs(got[0, b, k] - ref[k]).max() / scale))
                worst_oracle = max(worst_oracle, float(np.abs(got[0, b, k] - want_oracle[0, b, k]).max() / scale))
    print(name, "GPU vs emulated rounding points:", worst_emul, " GPU vs double-precision oracle:", worst_oracle)
    assert worst_emul <= 1e-2, (worst_emul, worst_oracle)
    assert worst_emul <= 0.6 * worst_oracle   # the rounding points explain the distance to the oracle, up to flips
