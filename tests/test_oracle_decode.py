"""Pins of the oracle's decoding loop (CPU only): special cases that reduce to textbook decoders, the end-to-end
form of Theorem 1, and the structural properties of the window."""
import math

import numpy as np
import pytest
from scipy import stats

import workload

M0, M1, W0, W1 = 0xD2511F53, 0xCD9E8D57, 0x9E3779B9, 0xBB67AE85


def py_philox(ctr, key):
    """Independent pure-Python Philox4x32-10 (used only by the textbook samplers below)."""
    c, k = list(ctr), list(key)
    for _ in range(10):
        p0, p1 = M0 * c[0], M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
        k = [(k[0] + W0) & 0xFFFFFFFF, (k[1] + W1) & 0xFFFFFFFF]
    return c


def _model(name, alpha=None, std=0.08, seed=None):
    cfg = workload.get_config(name)
    arch = cfg["arch"]
    w = workload.make_weights(arch, cfg["seed"] if seed is None else seed, alpha or 12.0, cfg["dtype"], std=std)
    cond, uncond = workload.make_prompts(arch, cfg["seed"], cfg["n_seqs"], cfg["prompt_len"])
    return cfg, arch, w, cond, uncond


def _guided_double(oracle, arch, w, cond_seq, uncond_seq, s):
    lc = oracle.forward_logits(arch, w, cond_seq)[-1].astype(np.float64)
    lu = oracle.forward_logits(arch, w, uncond_seq)[-1].astype(np.float64)
    return lu + s * (lc - lu)


def test_window_of_one_is_ancestral_sampling(oracle):
    """L = 1: every step draws one token from p(. | prefix) -- ordinary top-K ancestral sampling (Sec. 3.1).
    The textbook sampler here: double-precision softmax of the guided logits over the top-K set, inverse CDF at
    u = U64 / 2^64 with the same Philox words."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    N, K, s, seed = 24, 50, 3.0, 5
    dec = oracle.Oracle(arch, w, 1, cfg["prompt_len"] + N, cfg_scale=s, top_k=K, seed=seed)
    assert dec.prefill(cond, uncond, [N]) == 0
    hist = dec.decode()
    assert len(hist) == N and all(h[0]["n_finalized"] == 1 and h[0]["n_accepted"] == 0 for h in hist)
    got = dec.tokens()
    c, u = list(cond[0]), list(uncond[0])
    for i in range(N):
        z = _guided_double(oracle, arch, w, c, u, s)
        t = np.sort(z)[::-1][K - 1]
        p = np.where(z >= t, np.exp(z - z.max()), 0.0)
        cdf = np.cumsum(p / p.sum())
        words = py_philox([i + 1, 0, 0, 0], [seed, 0])
        uni = ((words[1] << 32) | words[2]) / 2.0 ** 64
        tok = int(np.searchsorted(cdf, uni, side="right"))
        margin = np.abs(cdf - uni).min()
        assert tok == got[i] or margin < 1e-5, (i, tok, got[i], margin)
        c.append(int(got[i]))
        u.append(int(got[i]))


@pytest.mark.parametrize("L,tau,seed", [(1, 0.5, 0), (2, 0.5, 1), (5, 0.5, 2), (8, float("inf"), 3), (8, 0.0, 4),
                                         (7, 0.5, 5)])
def test_top_1_is_greedy_decoding(oracle, L, tau, seed):
    """K = 1 makes every distribution one-hot: acceptance, residual and reuse all degenerate to the deterministic
    Jacobi iteration (Eq. 1), whose fixed point is the greedy AR sequence, reached in at most N forwards (Sec. 3.2)."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    N, s = 20, 3.0
    dec = oracle.Oracle(arch, w, L, cfg["prompt_len"] + N, cfg_scale=s, top_k=1, reuse_tau=tau, seed=seed)
    assert dec.prefill(cond, uncond, [N]) == 0
    hist = dec.decode()
    assert len(hist) <= N
    got = dec.tokens()
    c, u = list(cond[0]), list(uncond[0])
    for i in range(N):
        z = _guided_double(oracle, arch, w, c, u, s)
        top2 = np.sort(z)[-2:]
        tok = int(np.argmax(z))
        assert tok == got[i] or top2[1] - top2[0] < 1e-5
        c.append(int(got[i]))
        u.append(int(got[i]))


def _ar_joint(oracle, arch, w, cond, uncond, V, N, s, K):
    joint = np.zeros(V ** N)
    memo = {}
    for idx in range(V ** N):
        seq = [(idx // V ** i) % V for i in range(N)]
        pr = 1.0
        for i, tok in enumerate(seq):
            key = tuple(seq[:i])
            if key not in memo:
                lc = oracle.forward_logits(arch, w, list(cond) + list(key))[-1]
                lu = oracle.forward_logits(arch, w, list(uncond) + list(key))[-1]
                memo[key] = oracle.sampling_row(lc, lu, s, 1.0, K)
            e, Z = memo[key]
            pr *= oracle.weight_of(float(e[tok])) / Z
        joint[idx] = pr
    assert abs(joint.sum() - 1.0) < 1e-9
    return joint


def _chi_square_against(joint, counts, n, min_cells):
    assert counts.sum() == n
    assert counts[joint == 0].sum() == 0
    # pool cells with small expectation so that the chi-square approximation holds
    order = np.argsort(joint)
    exp, obs, acc_e, acc_o = [], [], 0.0, 0
    for i in order:
        if joint[i] == 0:
            continue
        acc_e += joint[i] * n
        acc_o += counts[i]
        if acc_e >= 20:
            exp.append(acc_e); obs.append(acc_o); acc_e, acc_o = 0.0, 0
    if acc_e > 0:
        exp[-1] += acc_e; obs[-1] += acc_o
    assert len(exp) > min_cells
    assert stats.chisquare(obs, exp).pvalue > 0.01


def test_no_reuse_decoding_has_the_autoregressive_joint_law(oracle):
    """Theorem 1 end to end: with tau = +inf (Eq. 6) the decoded sequence is distributed exactly as ancestral
    sampling.  Toy model, V = 8, N = 3, window 3: the AR joint is enumerated over all 512 sequences."""
    cfg, arch, w, cond, uncond = _model("toy", alpha=0.6, std=0.3)
    V, N, s, K = 8, 3, 3.0, 6
    joint = _ar_joint(oracle, arch, w, cond[0], uncond[0], V, N, s, K)
    n = 400_000
    counts, steps = oracle.decode_trials(arch, w, 3, cond[0], uncond[0], N, n, seed0=1000, cfg_scale=s, top_k=K,
                                         reuse_tau=float("inf"))
    assert 1.0 <= N / (steps / n) <= 3.0
    _chi_square_against(joint, counts, n, 30)


@pytest.mark.parametrize("mode,row_width", [(1, 0), (2, 2), (3, 0), (4, 2)])
def test_spatial_initialisation_keeps_the_autoregressive_joint_law(oracle, mode, row_width):
    """Sec. 4.2: however a new slot is initialised (copy of the left or upper neighbour with a one-hot reference, a
    draw from the neighbour's row with that row as reference), verification against the true proposal keeps the
    output law exact (Theorem 1 holds for any q).  Window 2 on 4 tokens, so new slots do get initialised (after
    every fully accepted window); a wrong reference for them would bend the joint."""
    cfg, arch, w, cond, uncond = _model("toy", alpha=0.6, std=0.3)
    V, N, s, K = 8, 4, 3.0, 6
    joint = _ar_joint(oracle, arch, w, cond[0], uncond[0], V, N, s, K)
    n = 150_000
    counts, steps = oracle.decode_trials(arch, w, 2, cond[0], uncond[0], N, n, seed0=5000 + mode, cfg_scale=s, top_k=K,
                                         reuse_tau=float("inf"), init_mode=mode, row_width=row_width)
    assert 1.0 <= N / (steps / n) <= 2.0
    _chi_square_against(joint, counts, n, 40)


@pytest.mark.parametrize("mode,row_width", [(1, 0), (2, 3), (3, 0), (4, 3), (4, 9)])
def test_spatial_initialisation_fills_new_slots_as_stated(oracle, mode, row_width):
    """New slots of the window after a step: (a) equal the token to their left, (b) equal the token row_width places
    back in the image (uniform in the first image row), both with the one-hot reference; (c) are the inverse-CDF
    draws from the last row of the step with that row as reference; (d) are draws from the row under which the token
    row_width places back became final (recomputed here from the logits of the step that finalised it), or from the
    reference of the draft at that place.  Slots of the first window are uniform."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    L, Vs, lo, N, K = 6, arch["sample_hi"] - arch["sample_lo"], arch["sample_lo"], 40, 60
    P = cfg["prompt_len"]
    seen = 0
    for seed in range(6):
        dec = oracle.Oracle(arch, w, L, P + N, top_k=K, reuse_tau=0.5, seed=seed, init_mode=mode, row_width=row_width)
        assert dec.prefill(cond[:1], uncond[:1], [N]) == 0
        toks, refs, n_slots = dec.window()
        for k in range(1, n_slots):   # first window: uniform whatever the mode
            words = oracle.philox([0, k, 0, 0], [seed, 0])
            assert toks[k] == lo + ((words[3] * Vs) >> 32) and refs[k] == -1
        step = 0
        final_row = {}                             # image index -> (e, Z) of the row under which it became final
        while True:
            step += 1
            Le = dec.window()[2]
            logits = dec.peek_logits()
            n_before = len(dec.tokens())
            res = dec.step()[0]
            for i in range(res["n_finalized"]):
                final_row[n_before + i] = oracle.sampling_row(logits[0, 0, i], logits[0, 1, i], 3.0, 1.0, K)
            if res["done"]:
                break
            a = res["n_accepted"]
            after, refs, Le2 = dec.window()
            final = dec.tokens()
            n_img = len(final)
            for k2 in range(1, Le2):
                k = k2 + a + 1
                if k <= Le:
                    continue                      # carried, refreshed or drawn from the last row: other tests
                seen += 1
                idx = n_img + k2 - 1              # image index of this slot's token
                if mode == 1:
                    assert after[k2] == (final[-1] if k2 == 1 else after[k2 - 1]) and refs[k2] == -2
                elif mode == 2:
                    up = idx - row_width
                    if up >= 0:
                        assert after[k2] == (final[up] if up < n_img else after[up - n_img + 1]) and refs[k2] == -2
                    else:
                        words = oracle.philox([step, k, 0, 0], [seed, 0])
                        assert after[k2] == lo + ((words[3] * Vs) >> 32) and refs[k2] == -1
                elif mode == 3:
                    e, Z = oracle.sampling_row(logits[0, 0, Le - 1], logits[0, 1, Le - 1], 3.0, 1.0, K)
                    words = oracle.philox([step, k, 0, 0], [seed, 0])
                    assert after[k2] == lo + oracle.draw(e, Z, (words[1] << 32) | words[2]) and refs[k2] == Le - 1
                else:
                    up = idx - row_width
                    words = oracle.philox([step, k, 0, 0], [seed, 0])
                    if up < 0:
                        assert after[k2] == lo + ((words[3] * Vs) >> 32) and refs[k2] == -1
                    elif up < n_img:
                        e, Z = final_row[up]
                        assert refs[k2] == -3 - up % row_width
                        assert after[k2] == lo + oracle.draw(e, Z, (words[1] << 32) | words[2])
                    else:
                        j = up - n_img + 1            # the place above is slot j of this window: same distribution
                        assert refs[k2] == refs[j]
                        if refs[j] >= 0:
                            e, Z = oracle.sampling_row(logits[0, 0, refs[j]], logits[0, 1, refs[j]], 3.0, 1.0, K)
                            assert after[k2] == lo + oracle.draw(e, Z, (words[1] << 32) | words[2])
    assert seen > 20


def test_equal_distributions_accept_the_whole_window(oracle):
    """p = q: feeding a second step the rows the drafts were drawn from makes every such draft's ratio 1, so all of
    them are accepted whatever the uniforms are."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    L, Vs, N = 8, arch["sample_hi"] - arch["sample_lo"], 40
    rng = np.random.default_rng(0)
    for seed in range(12):
        dec = oracle.Oracle(arch, w, L, cfg["prompt_len"] + N, top_k=50, seed=seed)
        dec.prefill(cond, uncond, [N])
        lg1 = (rng.standard_normal((1, 2, L, Vs)) * 2).astype(np.float32)
        a = dec.step_from_logits(lg1)[0]["n_accepted"]
        lg2 = (rng.standard_normal((1, 2, L, Vs)) * 2).astype(np.float32)
        lg2[0, :, : L - a - 1] = lg1[0, :, a + 1:]
        r2 = dec.step_from_logits(lg2)[0]
        assert r2["n_accepted"] >= L - a - 1


def test_acceptance_is_monotone_in_the_ratio(oracle):
    rng = np.random.default_rng(1)
    for _ in range(3000):
        wp, wq = int(rng.integers(1, 1 << 40)), int(rng.integers(1, 1 << 40))
        Zp, Zq = int(rng.integers(1 << 40, 1 << 50)), int(rng.integers(1 << 40, 1 << 50))
        u = int(rng.integers(0, 1 << 32))
        if oracle.accept(u, wp, Zp, wq, Zq):
            assert oracle.accept(u, wp + int(rng.integers(0, 1 << 30)), Zp, wq, Zq)   # larger p
            assert oracle.accept(u, wp, Zp, max(wq - int(rng.integers(0, 1 << 30)), 0), Zq)  # smaller q
            assert oracle.accept(u // 2, wp, Zp, wq, Zq)                                # smaller uniform


def test_accepted_length_is_monotone_in_the_window(oracle):
    """Nested windows with shared counters: the first step of a window of L + 1 accepts at least as many drafts as
    the window of L fed the same rows."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    Vs, N = arch["sample_hi"] - arch["sample_lo"], 40
    rng = np.random.default_rng(3)
    for seed in range(10):
        lg = (rng.standard_normal((1, 2, 9, Vs)) * 0.3).astype(np.float32)  # flat rows: frequent acceptance
        prev = -1
        for L in range(2, 10):
            dec = oracle.Oracle(arch, w, L, cfg["prompt_len"] + N, top_k=Vs, seed=seed)
            dec.prefill(cond, uncond, [N])
            a = dec.step_from_logits(np.ascontiguousarray(lg[:, :, :L]))[0]["n_accepted"]
            assert a >= prev
            if 0 <= prev < L - 2:      # the shorter window already rejected a draft: same rejection point
                assert a == prev
            prev = a


def _replay_refresh(oracle, dec_args, lg, tau, seed):
    arch, w, cond, uncond, L, N, K, plen = dec_args
    dec = oracle.Oracle(arch, w, L, plen + N, top_k=K, reuse_tau=tau, seed=seed)
    dec.prefill(cond, uncond, [N])
    before, _, _ = dec.window()
    res = dec.step_from_logits(lg)[0]
    after, refs, n_slots = dec.window()
    return before, res, after, refs, n_slots


@pytest.mark.parametrize("tau", [float("inf"), 0.0, 0.5])
def test_reuse_threshold_semantics(oracle, tau):
    """tau = +inf redraws every slot after the rejection (Eq. 6); tau = 0 keeps every draft with p(x) > 0;
    tau = 0.5 keeps exactly the drafts with p(x) > tau q(x) (Eq. 4-5).  The redrawn tokens are recomputed here
    from the rows with the inverse-CDF primitive and the counters (step, row, seq)."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    L, Vs, N, K = 8, arch["sample_hi"] - arch["sample_lo"], 40, 60
    rng = np.random.default_rng(7)
    seen_keep = seen_redraw = 0
    for seed in range(10):
        lg = (rng.standard_normal((1, 2, L, Vs)) * 1.0).astype(np.float32)
        before, res, after, refs, n_slots = _replay_refresh(oracle, (arch, w, cond, uncond, L, N, K, cfg["prompt_len"]),
                                                            lg, tau, seed)
        a = res["n_accepted"]
        if a >= L - 1:
            continue
        rows = [oracle.sampling_row(lg[0, 0, k], lg[0, 1, k], 3.0, 1.0, K) for k in range(L)]
        for k2 in range(1, L):
            k = k2 + a + 1
            if k <= L - 1:
                e, Z = rows[k - 1]
                x = int(before[k])
                wp = oracle.weight_of(float(e[x]))
                kept = oracle.keep(tau, wp, Z, 1, Vs)   # drafts of the first step have the uniform reference
                if tau == float("inf"):
                    assert not kept
                if tau == 0.0:
                    assert kept == (wp > 0)
                if tau == 0.5:
                    assert kept == (wp / Z > 0.5 / Vs)
                words = oracle.philox([1, k - 1, 0, 0], [seed, 0])
                want = x if kept else oracle.draw(e, Z, (words[1] << 32) | words[2])
                seen_keep += kept
                seen_redraw += not kept
                assert after[k2] == want and refs[k2] == k - 1
            elif k == L:
                e, Z = rows[L - 1]
                words = oracle.philox([1, L - 1, 0, 0], [seed, 0])
                assert after[k2] == oracle.draw(e, Z, (words[1] << 32) | words[2]) and refs[k2] == L - 1
            else:
                words = oracle.philox([1, k, 0, 0], [seed, 0])
                assert after[k2] == (words[3] * Vs) >> 32 and refs[k2] == -1
    assert seen_redraw > 0 if tau != 0.0 else seen_keep > 0


def test_forced_tokens_appear_where_they_are_forced(oracle):
    """Token ranges (sjd.h: forced tokens): a range of one id forces that token at its position for every seed and
    window, the other positions stay inside their ranges, and with L = 1 the decode is ancestral sampling from the
    masked distributions (recomputed with the masked row primitive and the same counters)."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    lo0, hi0, N, K = arch["sample_lo"], arch["sample_hi"], 20, 50
    eol = lo0 + 7
    first = np.array([eol if (i + 1) % 5 == 0 else lo0 + 8 for i in range(N)], dtype=np.int32)
    end = np.array([eol + 1 if (i + 1) % 5 == 0 else hi0 for i in range(N)], dtype=np.int32)
    for L, seed in [(1, 3), (4, 4), (6, 5), (6, 6)]:
        dec = oracle.Oracle(arch, w, L, cfg["prompt_len"] + N, top_k=K, seed=seed)
        assert dec.prefill(cond, uncond, [N]) == 0
        assert dec.set_token_ranges(0, first, end) == 0
        hist = dec.decode()
        toks = dec.tokens()
        assert len(toks) == N and sum(h[0]["n_finalized"] for h in hist) == N
        for i in range(N):
            assert first[i] <= toks[i] < end[i], (L, i, toks[i])
        if L == 1:
            c, u = list(cond[0]), list(uncond[0])
            for i in range(N):
                lc, lu = oracle.forward_logits(arch, w, c)[-1], oracle.forward_logits(arch, w, u)[-1]
                e, Z = oracle.sampling_row(lc, lu, 3.0, 1.0, K, allow=(int(first[i]) - lo0, int(end[i]) - lo0))
                words = oracle.philox([i + 1, 0, 0, 0], [seed, 0])
                assert toks[i] == lo0 + oracle.draw(e, Z, (words[1] << 32) | words[2]), i
                c.append(int(toks[i]))
                u.append(int(toks[i]))
    dec = oracle.Oracle(arch, w, 4, cfg["prompt_len"] + N, top_k=K)
    assert dec.set_token_ranges(0, first, end) == -3                     # before prefill
    dec.prefill(cond, uncond, [N])
    assert dec.set_token_ranges(0, first, first) == -1                   # empty ranges
    assert dec.set_token_ranges(1, first, end) == -1                     # no such sequence
    assert dec.set_token_ranges(0, np.zeros(N + 1, np.int32), np.ones(N + 1, np.int32)) == -1


def test_each_branch_starts_from_its_own_last_prompt_token(oracle):
    """First step with prompts that END differently: row k of each branch must be the model's prediction after that
    branch's own prompt followed by the drafts (recomputed with the plain full-sequence forward)."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    c, u = np.array(cond[0]), np.array(uncond[0][:-3])
    u[-1] = (c[-1] + 5) % arch["vocab"]
    assert c[-1] != u[-1] and len(c) != len(u)
    L, N = 4, 10
    dec = oracle.Oracle(arch, w, L, len(c) + N, top_k=30, seed=9)
    assert dec.prefill([c], [u], [N]) == 0
    win, _, n = dec.window()
    got = dec.peek_logits()
    drafts = [int(t) for t in win[1:n]]
    want_c = oracle.forward_logits(arch, w, list(c) + drafts)[-L:]
    want_u = oracle.forward_logits(arch, w, list(u) + drafts)[-L:]
    assert np.abs(got[0, 0] - want_c).max() < 1e-5 and np.abs(got[0, 1] - want_u).max() < 1e-5
    assert np.abs(got[0, 0, 0] - got[0, 1, 0]).max() > 1e-3     # the two anchors really differ


def test_random_stream_of_a_later_sequence(oracle):
    """The counter is (step, row, SEQUENCE, 0): sequence 2 of a batch fed the same logits as sequence 0 must make
    different draws, and its refresh draws are recomputed here with sequence index 2."""
    cfg, arch, w, cond, uncond = _model("small_f32")
    L, Vs, N, K, seed = 8, arch["sample_hi"] - arch["sample_lo"], 40, 60, 21
    rng = np.random.default_rng(5)
    one = (rng.standard_normal((1, 2, L, Vs)) * 1.0).astype(np.float32)
    lg = np.concatenate([one, one, one], axis=0)
    dec = oracle.Oracle(arch, w, L, cfg["prompt_len"] + N, top_k=K, reuse_tau=float("inf"), seed=seed, max_seqs=3)
    assert dec.prefill(cond * 3, uncond * 3, [N] * 3) == 0
    before = [dec.window(s)[0].copy() for s in range(3)]
    res = dec.step_from_logits(lg)
    rows = [oracle.sampling_row(one[0, 0, k], one[0, 1, k], 3.0, 1.0, K) for k in range(L)]
    s = 2
    for k in range(1, L):     # the initial drafts: counter (0, k, 2, 0), word 3
        assert before[s][k] == arch["sample_lo"] + ((oracle.philox([0, k, s, 0], [seed, 0])[3] * Vs) >> 32)
    a = 0                     # verification with word 0 of (1, k - 1, 2, 0) against the uniform reference
    for k in range(1, L):
        e, Z = rows[k - 1]
        x = int(before[s][k]) - arch["sample_lo"]
        if not oracle.accept(oracle.philox([1, k - 1, s, 0], [seed, 0])[0], oracle.weight_of(float(e[x])), Z, 1, Vs):
            break
        a += 1
    assert res[s]["n_accepted"] == a
    after, refs, n_slots = dec.window(s)
    checked = 0
    for k2 in range(1, n_slots):
        k = k2 + a + 1
        if k <= L:            # tau = inf: every later slot is redrawn from its row with words 1-2 of (1, k - 1, 2, 0)
            e, Z = rows[k - 1]
            words = oracle.philox([1, k - 1, s, 0], [seed, 0])
            assert after[k2] == arch["sample_lo"] + oracle.draw(e, Z, (words[1] << 32) | words[2]) and refs[k2] == k - 1
            checked += 1
    assert checked > 0
    assert not np.array_equal(before[0], before[2])


def test_window_bookkeeping_to_the_end_of_the_image(oracle):
    """Every image token is produced exactly once, the window shrinks at the end, and the step compression
    S = tokens / steps lies in [1, L] (Sec. 5, metrics)."""
    cfg, arch, w, cond, uncond = _model("small_sub")
    for N, L in [(1, 5), (3, 5), (5, 5), (6, 5), (30, 5), (17, 1)]:
        dec = oracle.Oracle(arch, w, L, cfg["prompt_len"] + N, top_k=40, seed=N, max_seqs=3)
        assert dec.prefill(cond, uncond, [N, max(1, N - 1), N]) == 0
        hist = dec.decode(10 * N)
        for s, n in enumerate([N, max(1, N - 1), N]):
            toks = dec.tokens(s)
            assert len(toks) == n
            assert ((toks >= arch["sample_lo"]) & (toks < arch["sample_hi"])).all()
            fin = [h[s]["n_finalized"] for h in hist]
            assert sum(fin) == n
            steps = sum(1 for f in fin if f > 0)
            assert 1.0 <= n / steps <= L
            assert all(0 <= h[s]["n_accepted"] <= L - 1 for h in hist)
            assert all(h[s]["reject_index"] in (-1, h[s]["n_accepted"] + 1) for h in hist)
        assert all(x["done"] for x in hist[-1])


def test_decoding_is_a_function_of_the_seed(oracle):
    cfg, arch, w, cond, uncond = _model("small_f32")
    outs = []
    for seed in (1, 1, 2):
        dec = oracle.Oracle(arch, w, 6, cfg["prompt_len"] + 30, top_k=50, seed=seed)
        dec.prefill(cond, uncond, [30])
        dec.decode()
        outs.append(dec.tokens().copy())
    assert np.array_equal(outs[0], outs[1]) and not np.array_equal(outs[0], outs[2])


def test_error_paths(oracle):
    cfg, arch, w, cond, uncond = _model("small_f32")
    with pytest.raises(ValueError):
        oracle.Oracle(arch, w, 4, 64, top_k=0)
    dec = oracle.Oracle(arch, w, 4, 20, top_k=10)
    assert dec.prefill(cond, uncond, [30]) == -5          # capacity
    assert dec.prefill(cond + cond, uncond + uncond, [5, 5]) == -5   # more sequences than max_seqs
    with pytest.raises(RuntimeError):
        dec.n_seqs = 1
        dec.step()                                         # step before a successful prefill
