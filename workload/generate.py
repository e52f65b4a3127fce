"""Seeded random weights and prompts (numpy on the host; torch on a device for the large shapes)."""
import numpy as np

_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")


def round_to_bf16(a):
    """float32 array -> the nearest bfloat16 values (ties to even), still stored as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(a.shape)


def _shapes(arch):
    d, H, Hkv, F = arch["d_model"], arch["n_heads"], arch["n_kv_heads"], arch["d_ff"]
    hd = d // H
    return dict(wq=(H * hd, d), wk=(Hkv * hd, d), wv=(Hkv * hd, d), wo=(d, H * hd), w_gate=(F, d), w_up=(F, d),
                w_down=(d, F))


def make_weights(arch, seed, head_alpha=1.0, dtype="f32", std=0.02, random_gains=False):
    """dict of float32 numpy arrays: N(0, std) matrices, unit norm gains, head scaled by head_alpha.

    dtype == "bf16" rounds every array to bfloat16-representable values.
    random_gains draws the norm gains from U(0.5, 1.5) (tests only: unit gains
    would hide a missing gain multiply)."""
    rng = np.random.Generator(np.random.Philox(key=seed + 1000))
    d, V = arch["d_model"], arch["vocab"]
    fix = round_to_bf16 if dtype == "bf16" else (lambda x: x)

    def normal(shape, scale=std):
        return fix((rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)).astype(np.float32))

    def gain():
        if random_gains:
            return fix(rng.uniform(0.5, 1.5, d).astype(np.float32))
        return np.ones(d, dtype=np.float32)

    w = {name: [] for name in _PER_LAYER}
    w["tok_emb"] = normal((V, d))
    shapes = _shapes(arch)
    for _ in range(arch["n_layers"]):
        w["attn_norm"].append(gain())
        for name in ("wq", "wk", "wv", "wo"):
            w[name].append(normal(shapes[name]))
        w["mlp_norm"].append(gain())
        for name in ("w_gate", "w_up", "w_down"):
            w[name].append(normal(shapes[name]))
    w["final_norm"] = gain()
    w["lm_head"] = normal((V, d), std * head_alpha)
    return w


def make_weights_torch(arch, seed, head_alpha, device, dtype, std=0.02):
    """Same distributions generated directly on a torch device (for shapes too big to draw on the host)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed + 1000)
    d, V = arch["d_model"], arch["vocab"]

    def normal(shape, scale=std):
        return (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * scale).to(dtype)

    w = {name: [] for name in _PER_LAYER}
    w["tok_emb"] = normal((V, d))
    shapes = _shapes(arch)
    for _ in range(arch["n_layers"]):
        w["attn_norm"].append(torch.ones(d, device=device, dtype=dtype))
        for name in ("wq", "wk", "wv", "wo"):
            w[name].append(normal(shapes[name]))
        w["mlp_norm"].append(torch.ones(d, device=device, dtype=dtype))
        for name in ("w_gate", "w_up", "w_down"):
            w[name].append(normal(shapes[name]))
    w["final_norm"] = torch.ones(d, device=device, dtype=dtype)
    w["lm_head"] = normal((V, d), std * head_alpha)
    return w


def make_prompts(arch, seed, n_seqs, prompt_len):
    """(cond, uncond): lists of int32 arrays, ids uniform over the vocabulary.  The two prompts of a
    sequence are independent except for their last id, which plays the start-of-image marker (Sec. 3.1)."""
    rng = np.random.Generator(np.random.Philox(key=seed + 2000))
    cond, uncond = [], []
    for _ in range(n_seqs):
        c = rng.integers(0, arch["vocab"], prompt_len, dtype=np.int32)
        u = rng.integers(0, arch["vocab"], prompt_len, dtype=np.int32)
        u[-1] = c[-1]
        cond.append(c)
        uncond.append(u)
    return cond, uncond
