"""Workload table: the five benchmark configurations plus small test shapes.

Every entry is a plain dict:
  arch        transformer shape (sample_lo/sample_hi = id range that is sampled)
  dtype       "f32" or "bf16" (storage of weights / KV cache on the GPU)
  prompt_len  conditioning tokens (the unconditional prompt has the same length)
  n_image     image tokens to generate per sequence
  window      Jacobi window L (anchor + L-1 drafts)
  top_k, cfg_scale, temperature, tau, seed, n_seqs
  head_alpha  multiplier on the N(0, 0.02) output head so that the sampling
              distribution has an entropy near 4 nats (written by
              oracle/calibrate_alpha.py; None = closed-form first guess)
"""
import copy
import json
import math
import os


def _arch(n_layers, d_model, n_heads, n_kv_heads, d_ff, vocab, sample_lo=0, sample_hi=None):
    return dict(n_layers=n_layers, d_model=d_model, n_heads=n_heads, n_kv_heads=n_kv_heads, d_ff=d_ff,
                vocab=vocab, sample_lo=sample_lo, sample_hi=vocab if sample_hi is None else sample_hi,
                rms_eps=1e-5, rope_theta=10000.0)


def _cfg(arch, dtype, prompt_len, n_image, window, top_k, seed, n_seqs=1):
    return dict(arch=arch, dtype=dtype, prompt_len=prompt_len, n_image=n_image, window=window, top_k=top_k,
                cfg_scale=3.0, temperature=1.0, tau=0.5, seed=seed, n_seqs=n_seqs, head_alpha=None)


CONFIGS = {
    # tiny fp32 model, 16x16 image tokens
    "cfg0": _cfg(_arch(2, 256, 4, 4, 1024, 4096), "f32", 32, 256, 16, 256, 0),
    # LlamaGen-XL-shaped, 24x24 image tokens
    "cfg1": _cfg(_arch(36, 1280, 20, 20, 3456, 16384), "bf16", 120, 576, 16, 1000, 1),
    # Chameleon / Lumina-mGPT-7B-shaped, 48 rows of 48 tokens + a row-end token each
    "cfg2": _cfg(_arch(32, 4096, 32, 32, 11008, 65536), "bf16", 64, 48 * 49, 32, 2000, 2),
    # Emu3-8B-shaped (GQA), visual sub-range of the vocabulary sampled
    "cfg3": _cfg(_arch(32, 4096, 32, 8, 14336, 184622, 151854, 151854 + 32768), "bf16", 64, 4096, 32, 2048, 3),
    # throughput batch: 8 prompts on the cfg2 shape
    "cfg4": _cfg(_arch(32, 4096, 32, 32, 11008, 65536), "bf16", 64, 48 * 49, 32, 2000, 4, n_seqs=8),
}

# small shapes for unit tests (oracle runs them in milliseconds)
TINY = {
    "toy": _cfg(_arch(1, 16, 2, 2, 32, 8), "f32", 3, 3, 3, 8, 11),
    "small_f32": _cfg(_arch(2, 64, 4, 2, 128, 512), "f32", 9, 40, 8, 50, 12),
    "small_bf16": _cfg(_arch(2, 128, 4, 2, 256, 1024), "bf16", 11, 48, 16, 100, 13),
    # shapes that take the fused small-M bf16 path (head_dim 64 / 128, M = 32 / 64)
    "small_fused64": _cfg(_arch(2, 256, 4, 2, 512, 2048), "bf16", 13, 60, 16, 100, 15),
    "small_fused128": _cfg(_arch(3, 256, 2, 1, 352, 1500, 20, 1460), "bf16", 70, 90, 32, 200, 16),
    # 5 sequences x 2 x window 32 = 320 rows: the many-row projection kernels (tile kernels when forced by flag, else
    # row groups), with a ragged last row tile and ragged last column tiles (d = 192, F = 352, 1440 sampled ids)
    "small_tile": _cfg(_arch(2, 192, 3, 1, 352, 1500, 20, 1460), "bf16", 20, 70, 32, 150, 17, n_seqs=5),
    # a sampled range wide enough (256 column groups) that the vocabulary head runs 64-row groups: window 32, both
    # guidance branches of a position in one workgroup
    "small_wide_vocab": _cfg(_arch(2, 256, 4, 2, 512, 17000, 300, 300 + 16384), "bf16", 9, 70, 32, 500, 18),
    "small_sub": _cfg(_arch(2, 64, 2, 1, 96, 700, 100, 612), "f32", 7, 30, 5, 40, 14, n_seqs=3),
}

_ALPHA_FILE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "head_alpha.json")


def first_guess_alpha(arch):
    """alpha such that i.i.d. Gaussian logits alpha*0.02*sqrt(d)*N(0,1) have entropy ~ ln V - sigma^2/2 = 4."""
    vs = arch["sample_hi"] - arch["sample_lo"]
    gap = max(math.log(vs) - 4.0, 0.05)
    return math.sqrt(2.0 * gap) / (0.02 * math.sqrt(arch["d_model"]))


def get_config(name):
    table = CONFIGS if name in CONFIGS else TINY
    cfg = copy.deepcopy(table[name])
    cfg["name"] = name
    alpha = None
    if os.path.exists(_ALPHA_FILE):
        with open(_ALPHA_FILE) as f:
            alpha = json.load(f).get(name)
    cfg["head_alpha"] = float(alpha) if alpha is not None else first_guess_alpha(cfg["arch"])
    cfg["head_alpha_calibrated"] = alpha is not None
    return cfg
