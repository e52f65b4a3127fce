"""ctypes binding of the CPU oracle (test infrastructure; never imported by the product path).

Mirrors `sjd_oracle.h`.  Weights are numpy float32 arrays kept alive by the
`Oracle` object; every pointer handed to C is a host pointer.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("d_ff", C.c_int32), ("vocab", C.c_int32),
                ("sample_lo", C.c_int32), ("sample_hi", C.c_int32), ("rms_eps", C.c_double),
                ("rope_theta", C.c_double), ("window", C.c_int32), ("max_ctx", C.c_int32)]


_FP = C.POINTER(C.c_float)
_FPP = C.POINTER(_FP)


class Weights(C.Structure):
    _fields_ = [("tok_emb", _FP), ("final_norm", _FP), ("lm_head", _FP),
                ("attn_norm", _FPP), ("wq", _FPP), ("wk", _FPP), ("wv", _FPP), ("wo", _FPP),
                ("mlp_norm", _FPP), ("w_gate", _FPP), ("w_up", _FPP), ("w_down", _FPP)]


class Sampling(C.Structure):
    _fields_ = [("cfg_scale", C.c_float), ("temperature", C.c_float), ("top_k", C.c_int32),
                ("reuse_tau", C.c_float), ("seed", C.c_uint64), ("init_mode", C.c_int32), ("row_width", C.c_int32)]


class StepResult(C.Structure):
    _fields_ = [("n_accepted", C.c_int32), ("n_finalized", C.c_int32), ("reject_index", C.c_int32),
                ("done", C.c_int32)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b  # noqa: build on demand for CPU tests
            _b.build()
        L = C.CDLL(_LIB_PATH)
        L.oracle_exp_neg.restype = C.c_float
        L.oracle_exp_neg.argtypes = [C.c_float]
        L.oracle_weight_of.restype = C.c_uint64
        L.oracle_weight_of.argtypes = [C.c_float]
        L.oracle_accept.argtypes = [C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64]
        L.oracle_keep.argtypes = [C.c_float, C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint64]
        L.oracle_draw.argtypes = [_FP, C.c_uint64, C.c_int32, C.c_uint64]
        L.oracle_draw_residual.argtypes = [_FP, C.c_uint64, _FP, C.c_uint64, C.c_int32, C.c_uint64]
        L.oracle_draw_residual_onehot.argtypes = [_FP, C.c_uint64, C.c_int32, C.c_int32, C.c_uint64]
        L.oracle_sampling_row.argtypes = [_FP, _FP, C.c_int32, C.c_float, C.c_float, C.c_int32, _FP,
                                          C.POINTER(C.c_uint64)]
        L.oracle_sampling_row.restype = None
        L.oracle_sampling_row_range.argtypes = [_FP, _FP, C.c_int32, C.c_float, C.c_float, C.c_int32, C.c_int32, C.c_int32, _FP,
                                                C.POINTER(C.c_uint64)]
        L.oracle_sampling_row_range.restype = None
        L.oracle_set_token_ranges.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32]
        L.oracle_law_trials.argtypes = [_FP, C.c_uint64, _FP, C.c_uint64, C.c_int32, C.c_uint64, C.c_int64,
                                        C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.oracle_law_trials.restype = None
        L.oracle_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
        L.oracle_philox4x32_10.restype = None
        L.oracle_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(Sampling), C.c_int32,
                                    C.POINTER(C.c_void_p)]
        L.oracle_destroy.argtypes = [C.c_void_p]
        L.oracle_destroy.restype = None
        L.oracle_prefill.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.POINTER(C.c_int32)),
                                     C.POINTER(C.c_int32), C.POINTER(C.POINTER(C.c_int32)),
                                     C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.oracle_step.argtypes = [C.c_void_p, C.POINTER(StepResult)]
        L.oracle_step_from_logits.argtypes = [C.c_void_p, _FP, C.POINTER(StepResult)]
        L.oracle_copy_logits.argtypes = [C.c_void_p, _FP]
        L.oracle_peek_logits.argtypes = [C.c_void_p, _FP]
        L.oracle_get_tokens.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                                        C.POINTER(C.c_int32)]
        L.oracle_get_window.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                        C.POINTER(C.c_int32)]
        L.oracle_set_num_threads.argtypes = [C.c_int32]
        L.oracle_forward_logits.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(C.c_int32),
                                            C.c_int32, _FP]
        L.oracle_forward_window_logits.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights),
                                                   C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32),
                                                   C.c_int32, _FP]
        L.oracle_decode_trials.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(Sampling),
                                           C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                                           C.c_int32, C.c_uint64, C.c_int64, C.POINTER(C.c_int64),
                                           C.POINTER(C.c_int64)]
        _lib = L
    return _lib


def _fp(a):
    return a.ctypes.data_as(_FP)


def _ip(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def philox(ctr, key):
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    o = (C.c_uint32 * 4)()
    lib().oracle_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def exp_neg(x):
    return float(lib().oracle_exp_neg(C.c_float(x)))


def weight_of(e):
    return int(lib().oracle_weight_of(C.c_float(e)))


def sampling_row(logit_c, logit_u, cfg_scale, temperature, top_k, allow=None):
    """allow = (lo, hi): only ids in [lo, hi) of the row can have weight (forced-token mask)."""
    lc = np.ascontiguousarray(logit_c, dtype=np.float32)
    lu = np.ascontiguousarray(logit_u, dtype=np.float32)
    V = lc.shape[0]
    e = np.zeros(V, dtype=np.float32)
    Z = C.c_uint64(0)
    if allow is None:
        lib().oracle_sampling_row(_fp(lc), _fp(lu), V, cfg_scale, temperature, top_k, _fp(e), C.byref(Z))
    else:
        assert 0 <= allow[0] < allow[1] <= V
        lib().oracle_sampling_row_range(_fp(lc), _fp(lu), V, cfg_scale, temperature, top_k, allow[0], allow[1], _fp(e), C.byref(Z))
    return e, int(Z.value)


def weights_of(e):
    return np.array([weight_of(float(x)) for x in e], dtype=np.uint64)


def accept(u32, w_p, Z_p, w_q, Z_q):
    return bool(lib().oracle_accept(u32, w_p, Z_p, w_q, Z_q))


def keep(tau, w_p, Z_p, w_q, Z_q):
    return bool(lib().oracle_keep(C.c_float(tau), w_p, Z_p, w_q, Z_q))


def draw(e_p, Z_p, u64):
    e = np.ascontiguousarray(e_p, dtype=np.float32)
    return int(lib().oracle_draw(_fp(e), Z_p, e.shape[0], u64))


def draw_residual(e_p, Z_p, e_q, Z_q, u64):
    ep = np.ascontiguousarray(e_p, dtype=np.float32)
    if e_q is None:
        return int(lib().oracle_draw_residual(_fp(ep), Z_p, None, 0, ep.shape[0], u64))
    eq = np.ascontiguousarray(e_q, dtype=np.float32)
    return int(lib().oracle_draw_residual(_fp(ep), Z_p, _fp(eq), Z_q, ep.shape[0], u64))


def draw_residual_onehot(e_p, Z_p, x, u64):
    ep = np.ascontiguousarray(e_p, dtype=np.float32)
    return int(lib().oracle_draw_residual_onehot(_fp(ep), Z_p, x, ep.shape[0], u64))


def law_trials(e_p, Z_p, e_q, Z_q, seed, n_trials):
    ep = np.ascontiguousarray(e_p, dtype=np.float32)
    V = ep.shape[0]
    counts = np.zeros(V, dtype=np.int64)
    rej = C.c_int64(0)
    if e_q is None:
        qp, zq = None, 0
    else:
        eq = np.ascontiguousarray(e_q, dtype=np.float32)
        qp, zq = _fp(eq), Z_q
    lib().oracle_law_trials(_fp(ep), Z_p, qp, zq, V, seed, n_trials,
                            counts.ctypes.data_as(C.POINTER(C.c_int64)), C.byref(rej))
    return counts, int(rej.value)


def set_num_threads(n):
    return int(lib().oracle_set_num_threads(n))


class _Model:
    """Holds the C structs for a model given as a dict of numpy float32 arrays.

    `weights` keys: tok_emb, final_norm, lm_head, and per-layer lists attn_norm,
    wq, wk, wv, wo, mlp_norm, w_gate, w_up, w_down."""

    def __init__(self, arch, weights, window, max_ctx):
        self.arch = dict(arch)
        self.keep = []
        self.md = ModelDesc(arch["n_layers"], arch["d_model"], arch["n_heads"], arch["n_kv_heads"],
                            arch["d_ff"], arch["vocab"], arch["sample_lo"], arch["sample_hi"],
                            float(arch.get("rms_eps", 1e-5)), float(arch.get("rope_theta", 10000.0)),
                            window, max_ctx)
        w = Weights()
        for name in ("tok_emb", "final_norm", "lm_head"):
            a = np.ascontiguousarray(weights[name], dtype=np.float32)
            self.keep.append(a)
            setattr(w, name, _fp(a))
        for name in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down"):
            arrs = [np.ascontiguousarray(a, dtype=np.float32) for a in weights[name]]
            assert len(arrs) == arch["n_layers"], name
            self.keep.extend(arrs)
            ptrs = (_FP * len(arrs))(*[_fp(a) for a in arrs])
            self.keep.append(ptrs)
            setattr(w, name, C.cast(ptrs, _FPP))
        self.w = w
        self.Vs = arch["sample_hi"] - arch["sample_lo"]


def forward_logits(arch, weights, tokens):
    """Full causal forward from an empty cache: float32 [n][V_s]."""
    toks = np.ascontiguousarray(tokens, dtype=np.int32)
    m = _Model(arch, weights, 1, len(toks))
    out = np.zeros((len(toks), m.Vs), dtype=np.float32)
    rc = lib().oracle_forward_logits(C.byref(m.md), C.byref(m.w), _ip(toks), len(toks), _fp(out))
    assert rc == 0, rc
    return out


def forward_window_logits(arch, weights, prefix, window):
    pre = np.ascontiguousarray(prefix, dtype=np.int32)
    win = np.ascontiguousarray(window, dtype=np.int32)
    m = _Model(arch, weights, 1, len(pre) + len(win))
    out = np.zeros((len(win), m.Vs), dtype=np.float32)
    rc = lib().oracle_forward_window_logits(C.byref(m.md), C.byref(m.w), _ip(pre), len(pre), _ip(win), len(win),
                                            _fp(out))
    assert rc == 0, rc
    return out


def decode_trials(arch, weights, window, cond, uncond, n_image, n_trials, seed0=0, cfg_scale=3.0,
                  temperature=1.0, top_k=8, reuse_tau=float("inf"), init_mode=0, row_width=0):
    """Histogram of decoded sequences over n_trials seeds (see oracle_decode_trials)."""
    c = np.ascontiguousarray(cond, dtype=np.int32)
    u = np.ascontiguousarray(uncond, dtype=np.int32)
    m = _Model(arch, weights, window, max(len(c), len(u)) + n_image)
    sp = Sampling(cfg_scale, temperature, top_k, reuse_tau, 0, init_mode, row_width)
    counts = np.zeros(m.Vs ** n_image, dtype=np.int64)
    steps = C.c_int64(0)
    rc = lib().oracle_decode_trials(C.byref(m.md), C.byref(m.w), C.byref(sp), _ip(c), len(c), _ip(u), len(u),
                                    n_image, seed0, n_trials, counts.ctypes.data_as(C.POINTER(C.c_int64)),
                                    C.byref(steps))
    assert rc == 0, rc
    return counts, int(steps.value)


class Oracle:
    """The oracle decoder: create -> prefill -> step* (same call shape as the GPU library)."""

    def __init__(self, arch, weights, window, max_ctx, cfg_scale=3.0, temperature=1.0, top_k=2000,
                 reuse_tau=0.5, seed=0, max_seqs=1, init_mode=0, row_width=0):
        self.model = _Model(arch, weights, window, max_ctx)
        self.L = window
        self.Vs = self.model.Vs
        self.sp = Sampling(cfg_scale, temperature, top_k, reuse_tau, seed, init_mode, row_width)
        self.ctx = C.c_void_p()
        rc = lib().oracle_create(C.byref(self.model.md), C.byref(self.model.w), C.byref(self.sp), max_seqs,
                                 C.byref(self.ctx))
        if rc != 0:
            raise ValueError(f"oracle_create failed: {rc}")
        self.n_seqs = 0

    def close(self):
        if self.ctx:
            lib().oracle_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, cond, uncond, n_image_tokens):
        S = len(cond)
        conds = [np.ascontiguousarray(c, dtype=np.int32) for c in cond]
        unconds = [np.ascontiguousarray(c, dtype=np.int32) for c in uncond]
        IP = C.POINTER(C.c_int32)
        cp = (IP * S)(*[_ip(a) for a in conds])
        up = (IP * S)(*[_ip(a) for a in unconds])
        cl = (C.c_int32 * S)(*[len(a) for a in conds])
        ul = (C.c_int32 * S)(*[len(a) for a in unconds])
        ni = (C.c_int32 * S)(*[int(n) for n in n_image_tokens])
        rc = lib().oracle_prefill(self.ctx, S, cp, cl, up, ul, ni)
        if rc == 0:
            self.n_seqs = S
        return rc

    def set_token_ranges(self, seq, first_id, end_id):
        lo = np.ascontiguousarray(first_id, dtype=np.int32)
        hi = np.ascontiguousarray(end_id, dtype=np.int32)
        assert lo.shape == hi.shape and lo.ndim == 1
        return lib().oracle_set_token_ranges(self.ctx, seq, _ip(lo), _ip(hi), len(lo))

    def _results(self, arr):
        return [dict(n_accepted=r.n_accepted, n_finalized=r.n_finalized, reject_index=r.reject_index,
                     done=r.done) for r in arr]

    def step(self):
        res = (StepResult * max(self.n_seqs, 1))()
        rc = lib().oracle_step(self.ctx, res)
        if rc != 0:
            raise RuntimeError(f"oracle_step failed: {rc}")
        return self._results(res)

    def step_from_logits(self, logits):
        lg = np.ascontiguousarray(logits, dtype=np.float32)
        assert lg.size == self.n_seqs * 2 * self.L * self.Vs
        res = (StepResult * self.n_seqs)()
        rc = lib().oracle_step_from_logits(self.ctx, _fp(lg), res)
        if rc != 0:
            raise RuntimeError(f"oracle_step_from_logits failed: {rc}")
        return self._results(res)

    def logits(self):
        out = np.zeros((self.n_seqs, 2, self.L, self.Vs), dtype=np.float32)
        lib().oracle_copy_logits(self.ctx, _fp(out))
        return out

    def peek_logits(self):
        """The oracle's own forward for the current window, without deciding anything."""
        out = np.zeros((self.n_seqs, 2, self.L, self.Vs), dtype=np.float32)
        rc = lib().oracle_peek_logits(self.ctx, _fp(out))
        if rc != 0:
            raise RuntimeError(f"oracle_peek_logits failed: {rc}")
        return out

    def tokens(self, seq=0):
        n = C.c_int32(0)
        lib().oracle_get_tokens(self.ctx, seq, None, 0, C.byref(n))
        out = np.zeros(max(n.value, 1), dtype=np.int32)
        lib().oracle_get_tokens(self.ctx, seq, _ip(out), n.value, C.byref(n))
        return out[:n.value]

    def window(self, seq=0):
        toks = np.zeros(self.L, dtype=np.int32)
        refs = np.zeros(self.L, dtype=np.int32)
        n = C.c_int32(0)
        lib().oracle_get_window(self.ctx, seq, _ip(toks), _ip(refs), C.byref(n))
        return toks, refs, n.value

    def decode(self, max_steps=1 << 30):
        """Steps until every sequence is done; returns the list of per-step results."""
        hist = []
        for _ in range(max_steps):
            r = self.step()
            hist.append(r)
            if all(x["done"] for x in r):
                break
        return hist
