"""Pins of the oracle's transformer forward (CPU only): a reference built from torch library routines
in double precision, and the structural properties a causal cached forward must have."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workload


def _torch_reference(arch, w, tokens):
    """Pre-norm decoder forward over a whole sequence with torch CPU library ops in float64.
    RoPE is written as a complex multiplication (x_i + j x_{i+hd/2}) * exp(j pos theta^(-2i/hd))."""
    d, H, Hkv = arch["d_model"], arch["n_heads"], arch["n_kv_heads"]
    hd = d // H
    T = len(tokens)
    t = lambda a: torch.from_numpy(np.asarray(a)).double()
    x = t(w["tok_emb"])[torch.as_tensor(tokens, dtype=torch.long)]
    pos = torch.arange(T, dtype=torch.float64)
    freq = arch["rope_theta"] ** (-torch.arange(0, hd // 2, dtype=torch.float64) * 2 / hd)
    rot = torch.polar(torch.ones(T, hd // 2, dtype=torch.float64), pos[:, None] * freq[None, :])  # [T, hd/2]

    def rope(v):  # v [T, heads, hd]
        c = torch.complex(v[..., : hd // 2], v[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([c.real, c.imag], dim=-1)

    for l in range(arch["n_layers"]):
        xn = F.rms_norm(x, (d,), t(w["attn_norm"][l]), arch["rms_eps"])
        q = rope(F.linear(xn, t(w["wq"][l])).view(T, H, hd))
        k = rope(F.linear(xn, t(w["wk"][l])).view(T, Hkv, hd))
        v = F.linear(xn, t(w["wv"][l])).view(T, Hkv, hd)
        k = k.repeat_interleave(H // Hkv, dim=1)
        v = v.repeat_interleave(H // Hkv, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           is_causal=True)[0]
        x = x + F.linear(o.transpose(0, 1).reshape(T, H * hd), t(w["wo"][l]))
        xn = F.rms_norm(x, (d,), t(w["mlp_norm"][l]), arch["rms_eps"])
        x = x + F.linear(F.silu(F.linear(xn, t(w["w_gate"][l]))) * F.linear(xn, t(w["w_up"][l])), t(w["w_down"][l]))
    xn = F.rms_norm(x, (d,), t(w["final_norm"]), arch["rms_eps"])
    head = t(w["lm_head"])[arch["sample_lo"]:arch["sample_hi"]]
    return F.linear(xn, head).numpy()


@pytest.mark.parametrize("name", ["toy", "small_f32", "small_sub", "small_bf16"])
def test_forward_matches_torch_library_reference(oracle, name):
    cfg = workload.get_config(name)
    arch = cfg["arch"]
    w = workload.make_weights(arch, cfg["seed"], 8.0, cfg["dtype"], std=0.08, random_gains=True)
    tokens = np.random.default_rng(1).integers(0, arch["vocab"], 23).astype(np.int32)
    got = oracle.forward_logits(arch, w, tokens)
    want = _torch_reference(arch, w, tokens)
    assert got.shape == want.shape
    assert np.abs(want).max() > 0.5
    assert np.abs(got - want).max() < 1e-5 * max(1.0, np.abs(want).max())


def test_single_layer_single_head_special_case(oracle):
    arch = dict(n_layers=1, d_model=8, n_heads=1, n_kv_heads=1, d_ff=12, vocab=10, sample_lo=0, sample_hi=10,
                rms_eps=1e-5, rope_theta=10000.0)
    w = workload.make_weights(arch, 3, 5.0, "f32", std=0.3, random_gains=True)
    tokens = np.array([1, 7, 7, 2, 9], dtype=np.int32)
    assert np.abs(oracle.forward_logits(arch, w, tokens) - _torch_reference(arch, w, tokens)).max() < 1e-6


def test_causality(oracle):
    cfg = workload.get_config("small_f32")
    arch = cfg["arch"]
    w = workload.make_weights(arch, 5, 8.0, std=0.08)
    rng = np.random.default_rng(2)
    a = rng.integers(0, arch["vocab"], 12).astype(np.int32)
    b = a.copy()
    b[7:] = rng.integers(0, arch["vocab"], 5)
    la, lb = oracle.forward_logits(arch, w, a), oracle.forward_logits(arch, w, b)
    assert np.array_equal(la[:7], lb[:7])          # rows before the change are untouched
    assert np.abs(la[7:] - lb[7:]).max() > 1e-3    # rows from the change on do depend on it


def test_cache_consistency(oracle):
    """A window forward on top of c cached tokens equals the last rows of one full forward over c + n tokens."""
    cfg = workload.get_config("small_sub")
    arch = cfg["arch"]
    w = workload.make_weights(arch, 6, 8.0, std=0.08, random_gains=True)
    toks = np.random.default_rng(3).integers(0, arch["vocab"], 17).astype(np.int32)
    full = oracle.forward_logits(arch, w, toks)
    for c in (0, 1, 9, 16):
        win = oracle.forward_window_logits(arch, w, toks[:c], toks[c:])
        assert np.abs(win - full[c:]).max() < 1e-6


def test_positions_after_a_cached_prefix(oracle):
    """Rotary positions of a window that starts at cache offset c: equal to rows c.. of the torch reference, whose
    rotation is a complex multiplication by exp(j pos theta^(-2i/hd)), at two different offsets and a small theta
    (so that the rotation angles are large)."""
    arch = dict(n_layers=1, d_model=16, n_heads=2, n_kv_heads=2, d_ff=24, vocab=12, sample_lo=0, sample_hi=12,
                rms_eps=1e-5, rope_theta=100.0)
    w = workload.make_weights(arch, 8, 6.0, std=0.3)
    win = np.array([3, 5, 1, 9], dtype=np.int32)
    outs = {}
    for c in (2, 5):
        prefix = np.arange(c, dtype=np.int32)
        got = oracle.forward_window_logits(arch, w, prefix, win)
        want = _torch_reference(arch, w, np.concatenate([prefix, win]))[c:]
        assert np.abs(got - want).max() < 1e-6
        outs[c] = got
    assert np.abs(outs[2] - outs[5]).max() > 1e-3
