"""ctypes binding of include/sjd.h.  Same names as the C ABI; torch is used for device memory and streams only."""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsjd.so")
_lib = None

F32, BF16 = 0, 1
KERNELS_REFERENCE, NO_GRAPH, KERNELS_ROWGROUPS, ATTENTION_CHUNKED, KERNELS_TILES, NO_L2_WARM, TILES_256_ROWS, NO_ROW_SPLIT, NO_MIXED_WIDTH, NO_K_ROTATION = 1, 2, 4, 8, 16, 32, 64, 128, 256, 512
KEEP_LOGITS, NO_HEAD_FUSION = 1024, 2048
OK, EINVAL, ENOMEM, ESTATE, EDEVICE, ECAPACITY = 0, -1, -2, -3, -4, -5


class SjdError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"sjd error {code}: {message}")
        self.code = code


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "d_ff", "vocab",
                                         "sample_lo", "sample_hi")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "max_seqs", "max_ctx", "window", "kv_page_tokens", "kernel_flags")]


_VPP = C.POINTER(C.c_void_p)


class Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p)] + \
               [(n, _VPP) for n in ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")]


class Sampling(C.Structure):
    _fields_ = [("cfg_scale", C.c_float), ("temperature", C.c_float), ("top_k", C.c_int32), ("reuse_tau", C.c_float),
                ("seed", C.c_uint64), ("init_mode", C.c_int32), ("row_width", C.c_int32)]


class StepResult(C.Structure):
    _fields_ = [("n_accepted", C.c_int32), ("n_finalized", C.c_int32), ("reject_index", C.c_int32), ("done", C.c_int32)]


class TraceEntry(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int64), ("total_ms", C.c_double)]


def library_path():
    return _LIB_PATH


def lib():
    """Loads libsjd.so (built by paper_2512_07503_amd/build.py).  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise SjdError(EDEVICE, f"{_LIB_PATH} is not built; run `python -m paper_2512_07503_amd.build`")
        L = C.CDLL(_LIB_PATH)
        IP, IPP = C.POINTER(C.c_int32), C.POINTER(C.POINTER(C.c_int32))
        L.sjd_create.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(Sampling), C.c_void_p, _VPP]
        L.sjd_prefill.argtypes = [C.c_void_p, C.c_int32, IPP, IP, IPP, IP, IP]
        L.sjd_step.argtypes = [C.c_void_p, C.POINTER(StepResult)]
        L.sjd_destroy.argtypes = [C.c_void_p]
        L.sjd_destroy.restype = None
        L.sjd_get_tokens.argtypes = [C.c_void_p, C.c_int32, IP, C.c_int32, IP]
        L.sjd_get_window.argtypes = [C.c_void_p, C.c_int32, IP, IP, IP]
        L.sjd_last_error.argtypes = [C.c_void_p]
        L.sjd_last_error.restype = C.c_char_p
        L.sjd_debug_copy_logits.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        L.sjd_debug_step_from_logits.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(StepResult)]
        L.sjd_snapshot_size.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
        L.sjd_snapshot_save.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64)]
        L.sjd_snapshot_restore.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
        L.sjd_trace_enable.argtypes = [C.c_void_p, C.c_int32]
        L.sjd_trace_reset.argtypes = [C.c_void_p]
        L.sjd_trace_read.argtypes = [C.c_void_p, C.POINTER(TraceEntry), C.c_int32, IP]
        L.sjd_op_gemm.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_float)]
        L.sjd_op_gemm_static.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                         C.c_int32, C.c_int32, C.c_int32]
        L.sjd_op_window_attention.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                              C.c_int32, C.c_int32, C.POINTER(C.c_float)]
        L.sjd_op_sampling_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                           C.c_int32, C.c_float, C.c_float, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_int32, C.POINTER(C.c_float)]
        L.sjd_set_token_ranges.argtypes = [C.c_void_p, C.c_int32, IP, IP, C.c_int32]
        L.sjd_op_philox.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_void_p, C.c_int32]
        _lib = L
    return _lib


def _check(rc, ctx=None):
    if rc != OK:
        msg = lib().sjd_last_error(ctx)
        raise SjdError(rc, msg.decode() if msg else "")


def _stream_ptr():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


_PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")


class Decoder:
    """sjd_create / sjd_prefill / sjd_step / sjd_destroy on device tensors.

    weights: dict of torch CUDA tensors (float32 for dtype "f32", bfloat16 for "bf16"): tok_emb, final_norm,
    lm_head and per-layer lists attn_norm, wq, wk, wv, wo, mlp_norm, w_gate, w_up, w_down."""

    def __init__(self, arch, weights, dtype, window, max_ctx, max_seqs=1, cfg_scale=3.0, temperature=1.0, top_k=2000,
                 reuse_tau=0.5, seed=0, kv_page_tokens=0, kernel_flags=0, init_mode=0, row_width=0):
        import torch
        want = torch.float32 if dtype == "f32" else torch.bfloat16
        tensors = [weights[n] for n in ("tok_emb", "final_norm", "lm_head")] + [t for n in _PER_LAYER for t in weights[n]]
        for t in tensors:
            if not (t.is_cuda and t.dtype == want and t.is_contiguous()):
                raise SjdError(EINVAL, "weights must be contiguous CUDA tensors of the model dtype")
        self.md = ModelDesc(arch["n_layers"], arch["d_model"], arch["n_heads"], arch["n_kv_heads"], arch["d_ff"],
                            arch["vocab"], arch["sample_lo"], arch["sample_hi"], arch.get("rms_eps", 1e-5),
                            arch.get("rope_theta", 10000.0), F32 if dtype == "f32" else BF16, max_seqs, max_ctx, window,
                            kv_page_tokens, kernel_flags)
        w = Weights()
        for n in ("tok_emb", "final_norm", "lm_head"):
            setattr(w, n, weights[n].data_ptr())
        keep = []
        for n in _PER_LAYER:
            arr = (C.c_void_p * arch["n_layers"])(*[t.data_ptr() for t in weights[n]])
            keep.append(arr)
            setattr(w, n, C.cast(arr, _VPP))
        sp = Sampling(cfg_scale, temperature, top_k, reuse_tau, seed, init_mode, row_width)
        self.ctx = C.c_void_p()
        self.L, self.Vs, self.n_seqs = window, arch["sample_hi"] - arch["sample_lo"], 0
        self.sparse_rows = True   # rows of the sampling distribution are stored as kept (id, weight) pairs
        # The context runs on the caller's current stream, unless that is the default stream: the library can only
        # capture its step into a HIP graph on an ordinary stream, so it then gets one of its own (default priority).
        # Either way the weights must be complete before sjd_create reads them.
        cur = torch.cuda.current_stream()
        cur.synchronize()
        self._stream = cur if cur.cuda_stream != 0 else torch.cuda.Stream()
        _check(lib().sjd_create(C.byref(self.md), C.byref(w), C.byref(sp), C.c_void_p(self._stream.cuda_stream), C.byref(self.ctx)))

    def close(self):
        if getattr(self, "ctx", None):
            lib().sjd_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def prefill(self, cond, uncond, n_image_tokens):
        S = len(cond)
        IP = C.POINTER(C.c_int32)
        conds = [np.ascontiguousarray(c, dtype=np.int32) for c in cond]
        unconds = [np.ascontiguousarray(c, dtype=np.int32) for c in uncond]
        cp = (IP * S)(*[a.ctypes.data_as(IP) for a in conds])
        up = (IP * S)(*[a.ctypes.data_as(IP) for a in unconds])
        cl = (C.c_int32 * S)(*[len(a) for a in conds])
        ul = (C.c_int32 * S)(*[len(a) for a in unconds])
        ni = (C.c_int32 * S)(*[int(n) for n in n_image_tokens])
        rc = lib().sjd_prefill(self.ctx, S, cp, cl, up, ul, ni)
        if rc == OK:
            self.n_seqs = S
        return rc

    @staticmethod
    def _results(arr):
        return [dict(n_accepted=r.n_accepted, n_finalized=r.n_finalized, reject_index=r.reject_index, done=r.done)
                for r in arr]

    def step(self):
        res = (StepResult * max(self.n_seqs, 1))()
        _check(lib().sjd_step(self.ctx, res), self.ctx)
        return self._results(res)

    def step_raw(self, res):
        """sjd_step into a preallocated (StepResult * n) array; returns the status code."""
        return lib().sjd_step(self.ctx, res)

    def step_from_logits(self, logits):
        lg = np.ascontiguousarray(logits, dtype=np.float32)
        assert lg.size == self.n_seqs * 2 * self.L * self.Vs
        res = (StepResult * self.n_seqs)()
        _check(lib().sjd_debug_step_from_logits(self.ctx, lg.ctypes.data_as(C.POINTER(C.c_float)), res), self.ctx)
        return self._results(res)

    def logits(self):
        out = np.zeros((self.n_seqs, 2, self.L, self.Vs), dtype=np.float32)
        _check(lib().sjd_debug_copy_logits(self.ctx, out.ctypes.data_as(C.POINTER(C.c_float))), self.ctx)
        return out

    def set_token_ranges(self, seq, first_id, end_id):
        """sjd_set_token_ranges: position i of sequence seq may only take ids in [first_id[i], end_id[i])."""
        IP = C.POINTER(C.c_int32)
        lo = np.ascontiguousarray(first_id, dtype=np.int32)
        hi = np.ascontiguousarray(end_id, dtype=np.int32)
        assert lo.shape == hi.shape and lo.ndim == 1
        return lib().sjd_set_token_ranges(self.ctx, seq, lo.ctypes.data_as(IP), hi.ctypes.data_as(IP), len(lo))

    def tokens(self, seq=0):
        n = C.c_int32(0)
        _check(lib().sjd_get_tokens(self.ctx, seq, None, 0, C.byref(n)), self.ctx)
        out = np.zeros(max(n.value, 1), dtype=np.int32)
        _check(lib().sjd_get_tokens(self.ctx, seq, out.ctypes.data_as(C.POINTER(C.c_int32)), n.value, C.byref(n)), self.ctx)
        return out[:n.value]

    def window(self, seq=0):
        IP = C.POINTER(C.c_int32)
        toks, refs, n = np.zeros(self.L, dtype=np.int32), np.zeros(self.L, dtype=np.int32), C.c_int32(0)
        _check(lib().sjd_get_window(self.ctx, seq, toks.ctypes.data_as(IP), refs.ctypes.data_as(IP), C.byref(n)), self.ctx)
        return toks, refs, n.value

    def snapshot(self):
        """The decoding state of the current batch as a uint8 array (sjd_snapshot_size + sjd_snapshot_save)."""
        n = C.c_uint64(0)
        _check(lib().sjd_snapshot_size(self.ctx, C.byref(n)), self.ctx)
        buf = np.zeros(n.value, dtype=np.uint8)
        w = C.c_uint64(0)
        _check(lib().sjd_snapshot_save(self.ctx, buf.ctypes.data_as(C.c_void_p), n.value, C.byref(w)), self.ctx)
        return buf[:w.value]

    def restore(self, buf):
        buf = np.ascontiguousarray(buf, dtype=np.uint8)
        _check(lib().sjd_snapshot_restore(self.ctx, buf.ctypes.data_as(C.c_void_p), buf.size), self.ctx)
        # the batch size travels with the snapshot
        self.n_seqs = int(np.frombuffer(buf[:32].tobytes(), dtype=np.int32)[5])

    def decode(self, max_steps=1 << 30):
        hist = []
        for _ in range(max_steps):
            r = self.step()
            hist.append(r)
            if all(x["done"] for x in r):
                break
        return hist

    def trace(self, on):
        _check(lib().sjd_trace_enable(self.ctx, 1 if on else 0), self.ctx)

    def trace_reset(self):
        _check(lib().sjd_trace_reset(self.ctx), self.ctx)

    def trace_read(self):
        n = C.c_int32(0)
        arr = (TraceEntry * 64)()
        _check(lib().sjd_trace_read(self.ctx, arr, 64, C.byref(n)), self.ctx)
        return {arr[i].name.decode(): (int(arr[i].launches), float(arr[i].total_ms)) for i in range(n.value)}


def _dtype_code(t):
    import torch
    return F32 if t.dtype == torch.float32 else BF16


def op_gemm(A, W, flags=0, splits=0, repeat=1):
    """C = A @ W.T through sjd_op_gemm; A [M,K], W [N,K] CUDA tensors (float32 or bfloat16). Returns (C, avg_ms)."""
    import torch
    M, K = A.shape
    N = W.shape[0]
    Cout = torch.empty((M, N), dtype=torch.float32, device=A.device)
    ms = C.c_float(0)
    _check(lib().sjd_op_gemm(_stream_ptr(), _dtype_code(A), flags, A.data_ptr(), W.data_ptr(), Cout.data_ptr(), M, N, K,
                             splits, repeat, C.byref(ms)))
    return Cout, ms.value


def op_gemm_static(A, W, flags=0, splits=0):
    """C = A @ W.T through sjd_op_gemm_static (no allocation inside the library); returns the status code and C."""
    import torch
    M, K = A.shape
    N = W.shape[0]
    Cout = torch.empty((M, N), dtype=torch.float32, device=A.device)
    rc = lib().sjd_op_gemm_static(_stream_ptr(), _dtype_code(A), flags, A.data_ptr(), W.data_ptr(), Cout.data_ptr(), M, N, K,
                                  splits)
    return rc, Cout


def op_window_attention(q, k, v, ctx, page_tokens=64, flags=0, repeat=1):
    """q [n,H,hd], k/v [ctx+n,Hkv,hd] -> out [n,H,hd] float32 through sjd_op_window_attention."""
    import torch
    n, H, hd = q.shape
    Hkv = k.shape[1]
    out = torch.empty((n, H, hd), dtype=torch.float32, device=q.device)
    ms = C.c_float(0)
    _check(lib().sjd_op_window_attention(_stream_ptr(), _dtype_code(q), flags, q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                         out.data_ptr(), n, ctx, H, Hkv, hd, page_tokens, repeat, C.byref(ms)))
    return out, ms.value


def op_sampling_rows(logits_c, logits_u, cfg_scale, temperature, top_k, repeat=1, allow_lo=None, allow_hi=None, kept=False):
    """float32 CUDA [rows,V] x2 -> (e float32 [rows,V], Z int64-viewed uint64 [rows], avg_ms); with kept=True also the
    stored form of the rows: (kept_ids int32 [rows,V], kept_cnt int32 [rows]).  allow_lo / allow_hi: int32 CUDA [rows]."""
    import torch
    rows, V = logits_c.shape
    e = torch.empty((rows, V), dtype=torch.float32, device=logits_c.device)
    Z = torch.zeros(rows, dtype=torch.int64, device=logits_c.device)
    ids = torch.zeros((rows, V), dtype=torch.int32, device=logits_c.device) if kept else None
    cnt = torch.zeros(rows, dtype=torch.int32, device=logits_c.device) if kept else None
    ms = C.c_float(0)
    _check(lib().sjd_op_sampling_rows(_stream_ptr(), logits_c.data_ptr(), logits_u.data_ptr(), e.data_ptr(), Z.data_ptr(),
                                      rows, V, cfg_scale, temperature, top_k,
                                      allow_lo.data_ptr() if allow_lo is not None else None,
                                      allow_hi.data_ptr() if allow_hi is not None else None,
                                      ids.data_ptr() if kept else None, cnt.data_ptr() if kept else None, repeat, C.byref(ms)))
    if kept:
        return e, Z, ms.value, ids, cnt
    return e, Z, ms.value


def op_philox(seed, row, seq, n):
    import torch
    out = torch.zeros(4 * n, dtype=torch.int32, device="cuda")
    _check(lib().sjd_op_philox(_stream_ptr(), seed, row, seq, out.data_ptr(), n))
    return out.cpu().numpy().view(np.uint32).reshape(n, 4)
