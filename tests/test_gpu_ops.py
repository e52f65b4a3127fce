"""GPU kernel parity, one operation at a time, through the C ABI (sjd_op_*), against the CPU oracle or
double-precision numpy.  Integer and bit-level results must be identical; floating point within a stated bound."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sjd():
    import torch
    assert torch.cuda.is_available()
    import paper_2512_07503_amd as m
    m.lib()
    return m


def test_philox_matches_oracle_on_a_million_counters(sjd, oracle):
    n = 1_000_000
    got = sjd.op_philox(0x1234567890ABCDEF, 5, 2, n)
    key = [0x90ABCDEF, 0x12345678]
    idx = np.concatenate([np.arange(0, 2000), np.random.default_rng(0).integers(0, n, 3000), [n - 1]])
    for i in idx:
        assert list(got[i]) == oracle.philox([int(i), 5, 2, 0], key), i
    # the rest by an independent vectorised implementation of the same published algorithm
    c = [np.arange(n, dtype=np.uint64), np.full(n, 5, np.uint64), np.full(n, 2, np.uint64), np.zeros(n, np.uint64)]
    k = [np.uint64(key[0]), np.uint64(key[1])]
    mask = np.uint64(0xFFFFFFFF)
    for _ in range(10):
        p0, p1 = np.uint64(0xD2511F53) * c[0], np.uint64(0xCD9E8D57) * c[2]
        c = [(p1 >> np.uint64(32)) ^ c[1] ^ k[0], p1 & mask, (p0 >> np.uint64(32)) ^ c[3] ^ k[1], p0 & mask]
        k = [(k[0] + np.uint64(0x9E3779B9)) & mask, (k[1] + np.uint64(0xBB67AE85)) & mask]
    assert np.array_equal(got, np.stack(c, axis=1).astype(np.uint32))


@pytest.mark.parametrize("V,K,s,T,scale", [(8, 6, 3.0, 1.0, 1.0), (100, 7, 3.0, 1.0, 2.0), (1000, 100, 3.0, 1.0, 3.0),
                                            (4096, 256, 3.0, 1.0, 3.0), (4097, 4097, 1.5, 0.7, 1.0), (300, 1000, 0.0, 2.0, 5.0),
                                            (16384, 1000, 3.0, 1.0, 3.0), (65536, 2000, 3.0, 1.0, 2.0), (32768, 1, 3.0, 1.0, 2.0),
                                            # wider than the register-resident kernel takes (64 x 1024 ids): the multi-pass kernel
                                            (70001, 2000, 3.0, 1.0, 2.0), (66000, 70000, 3.0, 1.0, 1.0),
                                            # K just below V, K = 2: thresholds at both ends of the row
                                            (4096, 4095, 3.0, 1.0, 3.0), (16384, 2, 3.0, 1.0, 3.0), (32768, 2048, 3.0, 0.05, 2.0)])
def test_sampling_rows_bit_exact(sjd, oracle, V, K, s, T, scale):
    import torch
    rng = np.random.default_rng(V * 7 + K)
    rows = 5
    lc = (rng.standard_normal((rows, V)) * scale).astype(np.float32)
    lu = (rng.standard_normal((rows, V)) * scale).astype(np.float32)
    lc[1, : V // 2] = np.round(lc[1, : V // 2])    # many exact ties, also at the threshold
    lu[1, : V // 2] = np.round(lu[1, : V // 2])
    lc[2] = lu[2]                                   # guidance is the identity
    lc[3] *= 30.0                                   # exponent underflow region (z - max < -60)
    e, Z, _, ids, cnt = sjd.op_sampling_rows(torch.from_numpy(lc).cuda(), torch.from_numpy(lu).cuda(), s, T, K, kept=True)
    e, Z, ids, cnt = e.cpu().numpy(), Z.cpu().numpy().view(np.uint64), ids.cpu().numpy(), cnt.cpu().numpy()
    for r in range(rows):
        e_ref, Z_ref = oracle.sampling_row(lc[r], lu[r], s, T, K)
        assert np.array_equal(e[r].view(np.uint32), e_ref.view(np.uint32)), (r, np.flatnonzero(e[r] != e_ref)[:5])
        assert int(Z[r]) == Z_ref
        # the stored form of the row: ascending ids, every id with a weight among them, at least min(K, V) of them
        kept = ids[r, : cnt[r]]
        assert min(K, V) <= cnt[r] <= V and (np.diff(kept) > 0).all() and kept[0] >= 0 and kept[-1] < V
        assert np.isin(np.flatnonzero(e_ref), kept).all()


@pytest.mark.parametrize("V,K", [(1000, 100), (16384, 1000), (65536, 2000), (70001, 500)])
def test_sampling_rows_with_token_ranges_bit_exact(sjd, oracle, V, K):
    import torch
    rng = np.random.default_rng(V + K)
    ranges = [(0, V), (0, 1), (V - 1, V), (V // 3, V // 3 + K), (5, V - 7), (V // 2, V // 2 + K // 2), (V // 4 - 1, V // 4 + 1)]
    rows = len(ranges)
    lc = (rng.standard_normal((rows, V)) * 2).astype(np.float32)
    lu = (rng.standard_normal((rows, V)) * 2).astype(np.float32)
    lo = torch.tensor([a for a, _ in ranges], dtype=torch.int32).cuda()
    hi = torch.tensor([b for _, b in ranges], dtype=torch.int32).cuda()
    e, Z, _, ids, cnt = sjd.op_sampling_rows(torch.from_numpy(lc).cuda(), torch.from_numpy(lu).cuda(), 3.0, 1.0, K,
                                             allow_lo=lo, allow_hi=hi, kept=True)
    e, Z, ids, cnt = e.cpu().numpy(), Z.cpu().numpy().view(np.uint64), ids.cpu().numpy(), cnt.cpu().numpy()
    for r, (a, b) in enumerate(ranges):
        e_ref, Z_ref = oracle.sampling_row(lc[r], lu[r], 3.0, 1.0, K, allow=(a, b))
        assert np.array_equal(e[r].view(np.uint32), e_ref.view(np.uint32)), (r, a, b)
        assert int(Z[r]) == Z_ref
        kept = ids[r, : cnt[r]]
        assert cnt[r] == min(K, b - a) and kept.min() >= a and kept.max() < b


def _gemm_case(sjd, M, N, K, dtype, flags, splits=0):
    import torch
    rng = np.random.default_rng(M * 131 + N * 7 + K)
    A = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    At, Wt = torch.from_numpy(A).cuda().to(td), torch.from_numpy(W).cuda().to(td)
    got, _ = sjd.op_gemm(At, Wt, flags=flags, splits=splits)
    want = At.double().cpu().numpy() @ Wt.double().cpu().numpy().T     # the rounded operands, exact products
    scale = np.abs(want).max()
    # fp32 accumulation of K terms: error well below K * 2^-24 * |a||w| summed
    assert np.abs(got.cpu().numpy() - want).max() < 2e-5 * scale * max(1.0, np.sqrt(K / 256)), (M, N, K, dtype, flags)


@pytest.mark.parametrize("M,N,K", [(32, 768, 256), (7, 100, 64), (32, 4096, 256), (33, 130, 1024)])
def test_gemm_fp32(sjd, M, N, K):
    _gemm_case(sjd, M, N, K, "f32", 0)


@pytest.mark.parametrize("M,N,K,splits", [(32, 3840, 1280, 0), (32, 1280, 3456, 0), (64, 4096, 4096, 0), (7, 100, 64, 0),
                                           (33, 130, 1024, 3), (96, 2080, 512, 0), (512, 1024, 1024, 0), (32, 16384, 1280, 1),
                                           (1, 64, 16, 0), (40, 32768, 256, 0)])
def test_gemm_bf16_mfma(sjd, M, N, K, splits):
    _gemm_case(sjd, M, N, K, "bf16", 0, splits)


@pytest.mark.parametrize("M,N,K", [(32, 384, 256), (7, 100, 64)])
def test_gemm_bf16_reference_kernel(sjd, M, N, K):
    _gemm_case(sjd, M, N, K, "bf16", sjd.KERNELS_REFERENCE)


def _attention_case(sjd, n, ctx, H, Hkv, hd, dtype, page=64, flags=0):
    import torch
    rng = np.random.default_rng(n * 17 + ctx * 3 + H)
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    q = torch.from_numpy(rng.standard_normal((n, H, hd)).astype(np.float32)).cuda().to(td)
    k = torch.from_numpy(rng.standard_normal((ctx + n, Hkv, hd)).astype(np.float32)).cuda().to(td)
    v = torch.from_numpy(rng.standard_normal((ctx + n, Hkv, hd)).astype(np.float32)).cuda().to(td)
    got, _ = sjd.op_window_attention(q, k, v, ctx, page_tokens=page, flags=flags)
    qd, kd, vd = q.double().cpu().numpy(), k.double().cpu().numpy(), v.double().cpu().numpy()
    want = np.zeros((n, H, hd))
    for i in range(n):
        for h in range(H):
            kv = h // (H // Hkv)
            sc = kd[: ctx + i + 1, kv] @ qd[i, h] / np.sqrt(hd)
            p = np.exp(sc - sc.max())
            want[i, h] = (p / p.sum()) @ vd[: ctx + i + 1, kv]
    tol = 2e-5 if dtype == "f32" else 2e-2   # bf16: probabilities are rounded to bf16 before the PV product
    assert np.abs(got.cpu().numpy() - want).max() < tol * max(1.0, np.abs(want).max()), (n, ctx, H, Hkv, hd, dtype)


@pytest.mark.parametrize("n,ctx,H,Hkv,hd", [(1, 0, 2, 2, 16), (16, 31, 4, 4, 64), (8, 200, 4, 2, 32), (16, 130, 4, 1, 64),
                                             (3, 64, 2, 2, 8)])
def test_window_attention_fp32(sjd, n, ctx, H, Hkv, hd):
    _attention_case(sjd, n, ctx, H, Hkv, hd, "f32", page=32 if ctx < 100 else 64)


@pytest.mark.parametrize("n,ctx,H,Hkv,hd,flags", [(16, 0, 2, 2, 64, 1), (16, 119, 20, 20, 64, 1), (32, 700, 8, 8, 128, 1),
                                                   (32, 300, 8, 2, 128, 1), (1, 77, 4, 4, 64, 1), (16, 0, 2, 2, 64, 0),
                                                   (16, 119, 20, 20, 64, 0), (32, 700, 8, 8, 128, 0), (32, 300, 8, 2, 128, 0),
                                                   (1, 77, 4, 4, 64, 0), (5, 1000, 2, 1, 32, 0), (32, 64, 4, 4, 128, 0),
                                                   # one workgroup per head at the full LlamaGen-shaped context; the same
                                                   # small cases through the chunk + merge kernels (flag 8)
                                                   (16, 690, 20, 20, 64, 0), (16, 690, 20, 20, 64, 8), (16, 119, 20, 20, 64, 8),
                                                   (32, 300, 8, 2, 128, 8), (1, 77, 4, 4, 64, 8), (16, 0, 2, 2, 64, 8),
                                                   # windows longer than one 32-row query tile (paper-sized windows)
                                                   (96, 200, 4, 4, 64, 0), (96, 200, 4, 4, 64, 8), (250, 300, 4, 2, 128, 0),
                                                   (250, 300, 4, 2, 128, 8), (40, 0, 2, 2, 64, 0), (33, 31, 2, 1, 128, 8)])
def test_window_attention_bf16(sjd, n, ctx, H, Hkv, hd, flags):
    _attention_case(sjd, n, ctx, H, Hkv, hd, "bf16", flags=flags)
