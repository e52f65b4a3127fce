"""sjd_snapshot_save / sjd_snapshot_restore: a restored context replays the steps that followed the save.

The oracle has no snapshots (it is a plain program that just keeps running).  The GPU decoder and the oracle decode
in lockstep; at some step the GPU state is saved; both go on (every step still checked against the oracle); then
the GPU context is clobbered (more steps, or another prompt batch), restored, and must produce once more, bit for
bit, the verdicts, windows, tokens and logits it produced after the save - which the oracle had confirmed.
"""
import numpy as np
import pytest

import workload
from helpers import make_pair, assert_same_state, gpu_weights

pytestmark = pytest.mark.gpu


def _run(o, g, S, n_steps, record):
    for _ in range(n_steps):
        rg = g.step()
        glog = g.logits()
        if o is not None:
            assert o.step_from_logits(glog) == rg
            assert_same_state(o, g, S)
        record.append((rg, glog.copy(), [g.window(s) for s in range(S)], [g.tokens(s).copy() for s in range(S)]))
        if all(r["done"] for r in rg):
            break


def _same(a, b):
    assert len(a) == len(b)
    for (ra, la, wa, ta), (rb, lb, wb, tb) in zip(a, b):
        assert ra == rb
        assert np.array_equal(la, lb)   # same kernels on the same state: identical bits
        for (t1, r1, n1), (t2, r2, n2) in zip(wa, wb):
            assert n1 == n2 and np.array_equal(t1[:n1], t2[:n2]) and np.array_equal(r1[1:n1], r2[1:n2])
        for x, y in zip(ta, tb):
            assert np.array_equal(x, y)


@pytest.mark.parametrize("name,init_mode,row_width,clobber,ranges", [
    ("small_f32", 0, 0, "steps", False), ("small_fused64", 0, 0, "steps", False), ("small_fused64", 4, 6, "prefill", False),
    ("small_sub", 3, 0, "prefill", False), ("small_tile", 0, 0, "steps", False),
    # forced-token ranges are part of the state: the batch that takes the context over in between resets them
    ("small_fused64", 0, 0, "prefill", True), ("small_sub", 0, 0, "prefill", True)])
def test_restore_replays_the_steps_after_the_save(oracle, name, init_mode, row_width, clobber, ranges):
    cfg = workload.get_config(name)
    S = cfg["n_seqs"]
    o, g, cond, uncond, n_img = make_pair(oracle, cfg, head_alpha=6.0, std=0.08, random_gains=True, init_mode=init_mode,
                                          row_width=row_width, kernel_flags=16 if name == "small_tile" else 0)
    if ranges:
        lo0, hi0 = cfg["arch"]["sample_lo"], cfg["arch"]["sample_hi"]
        for q in range(S):
            n = n_img[q]
            first = np.array([lo0 + 2 + q if (i + 1) % 5 == 0 else lo0 + 3 * q for i in range(n)], dtype=np.int32)
            end = np.array([lo0 + 3 + q if (i + 1) % 5 == 0 else hi0 - 7 * q for i in range(n)], dtype=np.int32)
            assert o.set_token_ranges(q, first, end) == 0 and g.set_token_ranges(q, first, end) == 0
    before = []
    _run(o, g, S, 4, before)
    snap = g.snapshot()
    after = []
    _run(o, g, S, 6, after)          # confirmed by the oracle step by step
    assert len(after) >= 2
    if clobber == "prefill":         # another batch takes the context over: other prompts, fewer sequences
        c2, u2 = workload.make_prompts(dict(cfg["arch"]), cfg["seed"] + 7, 1, cfg["prompt_len"])
        assert g.prefill(c2, u2, [min(n_img)]) == 0
        _run(None, g, 1, 3, [])
    g.restore(snap)
    assert g.n_seqs == S
    again = []
    _run(None, g, S, len(after), again)
    _same(after, again)
    # a second restore of the same bytes, after the replay moved on
    g.restore(snap)
    again = []
    _run(None, g, S, 2, again)
    _same(after[:2], again)


def make_decoder_only(cfg, kv_page_tokens=0):
    import paper_2512_07503_amd as sjd
    arch = dict(cfg["arch"])
    w = workload.make_weights(arch, cfg["seed"], 6.0, cfg["dtype"], std=0.08, random_gains=True)
    return sjd.Decoder(arch, gpu_weights(w, cfg["dtype"]), cfg["dtype"], cfg["window"], cfg["prompt_len"] + int(np.max(cfg["n_image"])),
                       max_seqs=cfg["n_seqs"], cfg_scale=cfg["cfg_scale"], temperature=cfg["temperature"], top_k=cfg["top_k"],
                       reuse_tau=cfg["tau"], seed=cfg["seed"], kv_page_tokens=kv_page_tokens)


def test_snapshot_size_grows_with_the_accepted_prefix_and_errors_are_reported(oracle):
    import paper_2512_07503_amd as sjd
    cfg = workload.get_config("small_fused64")
    o, g, cond, uncond, n_img = make_pair(oracle, cfg, head_alpha=6.0, std=0.08, random_gains=True, kv_page_tokens=32)
    s0 = g.snapshot()
    for _ in range(30):
        if all(r["done"] for r in g.step()):
            break
    s1 = g.snapshot()
    assert s1.size > s0.size        # more cache pages of accepted positions
    with pytest.raises(sjd.SjdError) as e:
        g.restore(s1[: s1.size - 16])
    assert e.value.code == sjd.EINVAL
    bad = s1.copy()
    bad[0] ^= 0xFF                  # magic
    with pytest.raises(sjd.SjdError) as e:
        g.restore(bad)
    assert e.value.code == sjd.EINVAL
    # a failed restore leaves the context as it was
    ref = g.snapshot()
    assert np.array_equal(ref, s1)
    g.restore(s1)
    g.step()
    # before the first prefill there is nothing to save
    g3 = make_decoder_only(cfg, kv_page_tokens=32)
    with pytest.raises(sjd.SjdError) as e:
        g3.snapshot()
    assert e.value.code == sjd.ESTATE
    g3.restore(s1)                  # ... but a context of the same set-up takes a snapshot without a prefill
    assert g3.step() is not None
    # a context with another sampling set-up does not take it
    o2, g2, *_ = make_pair(oracle, cfg, head_alpha=6.0, std=0.08, random_gains=True, seed=cfg["seed"] + 1, kv_page_tokens=32)
    with pytest.raises(sjd.SjdError) as e:
        g2.restore(s1)
    assert e.value.code == sjd.EINVAL


def test_restore_rejects_state_that_would_index_out_of_bounds(oracle):
    """A buffer of the right size whose decoding state was altered (token counts, cache lengths, window tokens,
    reference rows, page table, stored rows, token ranges) is refused with SJD_EINVAL and leaves the context usable:
    the kernels index memory with these values.  The private layout is retraced here from the context's shape: header,
    page table, step counter, then the per-sequence arrays in their order."""
    import paper_2512_07503_amd as sjd
    cfg = workload.get_config("small_fused64")
    pt = 32
    o, g, cond, uncond, n_img = make_pair(oracle, cfg, head_alpha=6.0, std=0.08, random_gains=True, kv_page_tokens=pt)
    for _ in range(6):
        g.step()
    snap = g.snapshot()
    arch, L, S = cfg["arch"], cfg["window"], 1
    V = arch["sample_hi"] - arch["sample_lo"]
    max_ctx = cfg["prompt_len"] + n_img[0]
    pps = -(-max_ctx // pt)
    sizes = [L * 4, 8, L * 4, 4, 4, 8, 4, max_ctx * 4, 4, L * 4, L * 4] + [L * V * 4] * 4 + [L * 4] * 2 + [L * 8] * 2 + [max_ctx * 4] * 2 + [16]
    names = ["win", "anchor", "ref", "n_img", "n_image", "kv", "Le", "out", "acc", "cand", "cand_new", "ids0", "ids1", "e0", "e1",
             "cnt0", "cnt1", "Z0", "Z1", "alo", "ahi", "res"]
    kv = cfg["prompt_len"] - 1 + len(g.tokens(0))
    hd = arch["d_model"] // arch["n_heads"]
    page_bytes = arch["n_kv_heads"] * pt * hd * 2
    pages = 2 * -(-kv // pt) * page_bytes * 2 * arch["n_layers"]
    header = snap.size - (S * 2 * pps * 4 + 16 + sum(sizes) * S + pages)
    assert 64 <= header <= 256 and header % 16 == 0, header
    off = {"table": header}
    at = header + S * 2 * pps * 4 + 16
    for n, sz in zip(names, sizes):
        off[n] = at
        at += sz * S
    view = snap.view(np.int32) if snap.size % 4 == 0 else None
    assert view is not None
    # what the retraced offsets point at must be what the context reports (else the rest of this test proves nothing)
    toks, refs, Le = g.window(0)
    assert view[off["n_image"] // 4] == n_img[0] and view[off["n_img"] // 4] == len(g.tokens(0)) and view[off["Le"] // 4] == Le
    assert np.array_equal(view[off["win"] // 4 + 1: off["win"] // 4 + Le], toks[1:Le])
    assert view[off["kv"] // 4] == kv

    def refused(word, value):
        bad = snap.copy()
        bad.view(np.int32)[word] = value
        with pytest.raises(sjd.SjdError) as e:
            g.restore(bad)
        assert e.value.code == sjd.EINVAL, (word, value)

    refused(off["n_image"] // 4, 10 ** 6)
    refused(off["n_img"] // 4, -1)
    refused(off["n_img"] // 4, n_img[0] + 1)
    refused(off["Le"] // 4, L + 1)
    refused(off["kv"] // 4, 10 ** 6)
    refused(off["kv"] // 4 + 1, -5)
    refused(off["win"] // 4 + 1, arch["vocab"] + 7)
    refused(off["win"] // 4 + 2, -1)
    refused(off["ref"] // 4 + 1, L)
    refused(off["ref"] // 4 + 1, -3)                       # a kept row, which this set-up (init_mode 0) does not have
    refused(off["anchor"] // 4, arch["vocab"])
    refused(off["table"] // 4 + pps - 1, 10 ** 6)         # a page the decode has not reached yet
    refused(off["table"] // 4 + pps, -1)
    refused(off["cnt0"] // 4, V + 1)
    refused(off["cnt1"] // 4 + 3, -2)
    row_with_ids = next(k for k in range(L) if view[off["cnt0"] // 4 + k] >= 2)
    refused(off["ids0"] // 4 + row_with_ids * V, V)        # an id outside the row
    refused(off["ids0"] // 4 + row_with_ids * V + 1, 0)    # ids not ascending
    refused(off["alo"] // 4 + 3, V)
    refused(off["ahi"] // 4, V + 1)
    refused(off["acc"] // 4, L)
    # the context is as it was: the untouched snapshot still restores and decodes on
    g.restore(snap)
    assert g.step() is not None
