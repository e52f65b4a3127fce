"""Shared helpers of the GPU parity tests: build the oracle and the GPU decoder from the same seeded inputs."""
import numpy as np

import workload


def gpu_weights(w, dtype):
    import torch
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    out = {}
    for k, v in w.items():
        if isinstance(v, list):
            out[k] = [torch.from_numpy(a).to("cuda").to(td).contiguous() for a in v]
        else:
            out[k] = torch.from_numpy(v).to("cuda").to(td).contiguous()
    return out


def make_pair(oracle, cfg, weights=None, window=None, n_image=None, prompt_len=None, n_seqs=None, top_k=None, tau=None,
              seed=None, kernel_flags=0, kv_page_tokens=0, head_alpha=None, std=0.02, random_gains=False, n_layers=None,
              init_mode=0, row_width=0, drop_logits=False):
    """Returns (oracle decoder, gpu decoder, cond, uncond, n_image list) on identical inputs.  The GPU decoder keeps its
    logits (the comparison protocol downloads them every step) unless drop_logits."""
    import paper_2512_07503_amd as sjd
    arch = dict(cfg["arch"])
    if n_layers is not None:
        arch["n_layers"] = n_layers
    L = window or cfg["window"]
    N = n_image or cfg["n_image"]
    P = prompt_len or cfg["prompt_len"]
    S = n_seqs or cfg["n_seqs"]
    K = top_k or cfg["top_k"]
    tau = cfg["tau"] if tau is None else tau
    seed = cfg["seed"] if seed is None else seed
    alpha = cfg["head_alpha"] if head_alpha is None else head_alpha
    if weights is None:
        weights = workload.make_weights(arch, cfg["seed"], alpha, cfg["dtype"], std=std, random_gains=random_gains)
    cond, uncond = workload.make_prompts(arch, cfg["seed"], S, P)
    n_img = [N] * S if np.isscalar(N) else list(N)
    max_ctx = P + max(n_img)
    o = oracle.Oracle(arch, weights, L, max_ctx, cfg_scale=cfg["cfg_scale"], temperature=cfg["temperature"], top_k=K,
                      reuse_tau=tau, seed=seed, max_seqs=S, init_mode=init_mode, row_width=row_width)
    g = sjd.Decoder(arch, gpu_weights(weights, cfg["dtype"]), cfg["dtype"], L, max_ctx, max_seqs=S,
                    cfg_scale=cfg["cfg_scale"], temperature=cfg["temperature"], top_k=K, reuse_tau=tau, seed=seed,
                    kernel_flags=kernel_flags | (0 if drop_logits else sjd.KEEP_LOGITS), kv_page_tokens=kv_page_tokens,
                    init_mode=init_mode, row_width=row_width)
    assert o.prefill(cond, uncond, n_img) == 0
    assert g.prefill(cond, uncond, n_img) == 0
    return o, g, cond, uncond, n_img


def assert_same_state(o, g, n_seqs, where=""):
    for s in range(n_seqs):
        ot, orf, on = o.window(s)
        gt, grf, gn = g.window(s)
        assert on == gn, (where, s, on, gn)
        assert np.array_equal(ot[:on], gt[:gn]), (where, s, ot, gt)
        assert np.array_equal(orf[1:on], grf[1:gn]), (where, s, orf, grf)
        assert np.array_equal(o.tokens(s), g.tokens(s)), (where, s)


def logits_error(got, want, Le_rows):
    """max abs difference and max over rows of max|d| / max|want| on the active rows."""
    worst_abs, worst_rel = 0.0, 0.0
    for s, le in enumerate(Le_rows):
        for b in range(2):
            for k in range(le):
                d = np.abs(got[s, b, k] - want[s, b, k]).max()
                worst_abs = max(worst_abs, float(d))
                worst_rel = max(worst_rel, float(d / max(np.abs(want[s, b, k]).max(), 1e-30)))
    return worst_abs, worst_rel
