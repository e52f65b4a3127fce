"""Decision stage on the GPU (sampling distribution, verification, residual / refresh draws, window update) against
the oracle on identical fp32 logits and identical Philox counters: token ids, accept counts, rejection index and the
whole next window must be bit-exact at every step."""
import numpy as np
import pytest

import workload
from helpers import make_pair, assert_same_state

pytestmark = pytest.mark.gpu


def _drive(oracle, cfg_name, n_steps, window, n_image, n_seqs, top_k, tau, seed, scale, drift, prompt_len=4, ranges=None):
    cfg = workload.get_config(cfg_name)
    o, g, cond, uncond, n_img = make_pair(oracle, cfg, window=window, n_image=n_image, prompt_len=prompt_len, n_seqs=n_seqs,
                                          top_k=top_k, tau=tau, seed=seed, n_layers=1)
    S, L, Vs = n_seqs, window, o.Vs
    if ranges is not None:
        for s in range(S):
            first, end = ranges(s, n_img[s], cfg["arch"])
            assert o.set_token_ranges(s, first, end) == 0 and g.set_token_ranges(s, first, end) == 0
    rng = np.random.default_rng(seed + 99)
    Nmax = max(n_img)
    base = (rng.standard_normal((S, 2, Nmax + L, Vs)) * scale).astype(np.float32)   # a row per absolute image position
    done_img = [0] * S
    stats = dict(acc=0, steps=0, rej=0)
    for step in range(n_steps):
        lg = np.zeros((S, 2, L, Vs), dtype=np.float32)
        for s in range(S):
            lg[s] = base[s, :, done_img[s]: done_img[s] + L] + (rng.standard_normal((2, L, Vs)) * drift).astype(np.float32)
        ro = o.step_from_logits(lg)
        rg = g.step_from_logits(lg)
        assert ro == rg, (step, ro, rg)
        assert_same_state(o, g, S, where=f"step {step}")
        for s in range(S):
            done_img[s] += ro[s]["n_finalized"]
            stats["acc"] += ro[s]["n_accepted"]
            stats["rej"] += ro[s]["reject_index"] >= 0
        stats["steps"] += 1
        if all(r["done"] for r in ro):
            break
    return stats


@pytest.mark.parametrize("name,L,N,S,K,tau,seed,scale,drift", [
    ("small_f32", 8, 60, 1, 50, 0.5, 1, 2.0, 0.3),
    ("small_f32", 8, 60, 2, 50, float("inf"), 2, 2.0, 0.3),
    ("small_f32", 16, 33, 3, 512, 0.0, 3, 1.0, 0.1),
    ("small_sub", 5, 30, 3, 40, 0.5, 4, 2.0, 0.5),
    ("small_f32", 1, 12, 1, 50, 0.5, 5, 2.0, 0.3),
    ("small_f32", 2, 9, 2, 1, 0.5, 6, 2.0, 0.0),
    ("small_f32", 70, 200, 1, 50, 0.5, 7, 1.5, 0.05),
])
def test_decisions_bit_exact_small(oracle, name, L, N, S, K, tau, seed, scale, drift):
    st = _drive(oracle, name, 400, L, N, S, K, tau, seed, scale, drift)
    assert st["steps"] > 0


@pytest.mark.parametrize("name,L,N,S,K,tau,seed", [("small_f32", 8, 60, 2, 50, 0.5, 11), ("small_sub", 5, 30, 3, 40, 0.5, 12),
                                                    ("small_f32", 1, 20, 1, 50, 0.5, 13), ("small_f32", 16, 45, 1, 600, float("inf"), 14)])
def test_forced_token_ranges_bit_exact(oracle, name, L, N, S, K, tau, seed):
    """Token ranges per image position (a forced end-of-row token every 7 positions, a sub-range elsewhere, the
    tail of the image unrestricted; different ranges per sequence): decisions and windows identical to the
    oracle's, and the forced tokens come out where they were forced."""
    def ranges(s, n, arch):
        lo0, hi0 = arch["sample_lo"], arch["sample_hi"]
        m = n - 3                                              # the last three positions keep the whole range
        eol = lo0 + 3 + s
        first = np.array([eol if (i + 1) % 7 == 0 else lo0 + 10 * (s + 1) for i in range(m)], dtype=np.int32)
        end = np.array([eol + 1 if (i + 1) % 7 == 0 else hi0 - 5 * s for i in range(m)], dtype=np.int32)
        return first, end
    st = _drive(oracle, name, 400, L, N, S, K, tau, seed, 2.0, 0.3, ranges=ranges)
    assert st["steps"] > 0


def test_token_range_errors(oracle):
    cfg = workload.get_config("small_f32")
    o, g, cond, uncond, n_img = make_pair(oracle, cfg, window=4, n_image=10, prompt_len=4, n_layers=1)
    lo0, hi0 = cfg["arch"]["sample_lo"], cfg["arch"]["sample_hi"]
    ok_lo, ok_hi = np.full(10, lo0, np.int32), np.full(10, hi0, np.int32)
    assert g.set_token_ranges(0, ok_lo, ok_hi) == 0
    assert g.set_token_ranges(1, ok_lo, ok_hi) == -1                                  # no such sequence
    assert g.set_token_ranges(0, ok_hi, ok_hi) == -1                                  # empty range
    assert g.set_token_ranges(0, ok_lo, ok_hi + 1) == -1                              # beyond the sampled ids
    assert g.set_token_ranges(0, np.full(11, lo0, np.int32), np.full(11, hi0, np.int32)) == -1   # more positions than image tokens
    g.decode(100)
    assert len(g.tokens(0)) == 10


def test_decisions_bit_exact_cfg0_shape(oracle):
    """V_s = 4096, K = 256, L = 16 as in the first benchmark configuration, 256 image tokens, to completion."""
    st = _drive(oracle, "cfg0", 400, 16, 256, 1, 256, 0.5, 0, 3.0, 0.15)
    assert st["acc"] > 0 and st["rej"] > 0


@pytest.mark.parametrize("name,top_k,flat", [("cfg2", None, False),
                                             # V_s = 16384: K = 1000 (the kept entries fit the kernel's list), K = 6000
                                             # (they do not: plain pass over the row), K = V_s (no top-K at all)
                                             ("cfg1", None, False), ("cfg1", 6000, False), ("cfg1", 16384, False),
                                             # a row of few distinct values: thousands of ties with the K-th largest
                                             ("cfg1", None, True)])
def test_decisions_bit_exact_large_vocab(oracle, name, top_k, flat):
    """V_s = 65536, K = 2000, L = 32 (the 7B-shaped configurations) and V_s = 16384, two sequences, a few steps."""
    cfg = workload.get_config(name)
    cfg["arch"] = dict(cfg["arch"], d_model=64, n_heads=2, n_kv_heads=2, d_ff=64)   # only V_s matters here
    import helpers
    o, g, *_ = helpers.make_pair(oracle, cfg, window=32, n_image=80, prompt_len=3, n_seqs=2, n_layers=1, top_k=top_k)
    rng = np.random.default_rng(5)
    Vs = o.Vs
    base = (rng.standard_normal((2, 2, 120, Vs)) * 2.5).astype(np.float32)
    if flat:
        base = np.round(base)   # integers -9 .. 9
    pos = [0, 0]
    for step in range(6):
        lg = np.stack([base[s, :, pos[s]: pos[s] + 32] + (rng.standard_normal((2, 32, Vs)) * (0.0 if flat else 0.1)).astype(np.float32)
                       for s in range(2)])
        ro, rg = o.step_from_logits(lg), g.step_from_logits(lg)
        assert ro == rg, (step, ro, rg)
        assert_same_state(o, g, 2, where=f"step {step}")
        for s in range(2):
            pos[s] += ro[s]["n_finalized"]
