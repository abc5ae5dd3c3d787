"""GPU parity of single operators against plain numpy float64 (C ABI entry point tio_op_gemm)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _dev(a, dtype):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def _host(t):
    return t.float().cpu().numpy().astype(np.float64)


CASES = [  # M, N, K, pad of ld
    (128, 128, 64, 0), (200, 136, 72, 0), (256, 384, 256, 0), (130, 1000, 96, 24), (64, 72, 1000, 8),
    (513, 257, 130, 7), (8, 8, 8, 0), (1024, 768, 768, 0),
    (300, 200, 136, -4),       # output and residual rows start on 8-byte, not 16-byte, boundaries (ldc = 8k + 4)
]


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("a_km,b_km", [(0, 0), (0, 1), (1, 1), (1, 0)])
@pytest.mark.parametrize("M,N,K,pad", CASES)
def test_gemm_all_layouts(dtype, a_km, b_km, M, N, K, pad):
    import torch
    import paper_2506_06472_amd as tio
    print(f"gemm {dtype} a_km={a_km} b_km={b_km} M={M} N={N} K={K} pad={pad}", flush=True)
    rng = np.random.default_rng(M * 7 + N * 3 + K + a_km * 2 + b_km)
    r8 = lambda n: (n + 7) // 8 * 8
    # logical operands A[M,K], B[N,K]; stored [rows, ld] or [K, ld]
    lda = (r8(M) if a_km else r8(K)) + 8 * (pad > 0)
    ldb = (r8(N) if b_km else r8(K)) + 8 * (pad > 0)
    ldc = r8(N) + 8 * (pad > 0) + (4 if pad < 0 else 0)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((N, K)).astype(np.float32)
    bias = rng.standard_normal(r8(N)).astype(np.float32)
    R = rng.standard_normal((M, ldc)).astype(np.float32)
    As = np.full((K, lda) if a_km else (M, lda), np.nan, np.float32)     # NaN padding must never leak
    Bs = np.full((K, ldb) if b_km else (N, ldb), np.nan, np.float32)
    if a_km: As[:, :M] = A.T
    else: As[:, :K] = A
    if b_km: Bs[:, :N] = B.T
    else: Bs[:, :K] = B
    dA, dB, dbias, dR = _dev(As, dtype), _dev(Bs, dtype), _dev(bias, dtype), _dev(R, dtype)
    dC = torch.full((M, ldc), 7.0, device="cuda", dtype=dA.dtype)
    dsum = torch.full((r8(M) + 8,), 7.0, device="cuda", dtype=dA.dtype)
    torch.cuda.synchronize()
    for use_bias, use_res in ((0, 0), (1, 1)):
        tio.tio_op_gemm(0, dtype, a_km, b_km, M, N, K, dA.data_ptr(), lda, dB.data_ptr(), ldb,
                        dbias.data_ptr() if use_bias else 0, dR.data_ptr() if use_res else 0, ldc, dC.data_ptr(), ldc,
                        dsum.data_ptr() if use_res else 0)
        torch.cuda.synchronize()
        An = np.nan_to_num(_host(dA)); Bn = np.nan_to_num(_host(dB))
        A64 = An[:, :M].T if a_km else An[:, :K]
        B64 = Bn[:, :N].T if b_km else Bn[:, :K]
        ref = A64 @ B64.T
        if use_bias: ref = ref + _host(dbias)[:N]
        if use_res: ref = ref + _host(dR)[:, :N]
        got = _host(dC)
        assert np.all(got[:, N:] == 7.0), "wrote outside the N columns"
        err = np.abs(got[:, :N] - ref)
        tol = (2.0 ** -8 * np.abs(ref) + 1e-3 * np.sqrt(K)) if dtype == "bf16" else (1e-5 * np.sqrt(K) * (1 + np.abs(ref)))
        assert np.all(err <= tol), (float(err.max()), np.unravel_index(err.argmax(), err.shape))
        rs = _host(dsum)
        if use_res:      # fused row sums of A (the bias gradient of a weight-gradient GEMM)
            ref_rs = A64.sum(1)
            rtol = (2.0 ** -8 * np.abs(ref_rs) + 1e-3 * np.sqrt(K)) if dtype == "bf16" else 1e-5 * np.sqrt(K) * (1 + np.abs(ref_rs))
            assert np.all(np.abs(rs[:M] - ref_rs) <= rtol) and np.all(rs[M:] == 7.0)
        else:
            assert np.all(rs == 7.0)


@pytest.mark.parametrize("a_km,b_km", [(0, 0), (0, 1), (1, 1), (1, 0)])
def test_gemm_large_tile_configuration(a_km, b_km):
    """Enough 256x256 output tiles for the dispatch to pick the large-tile kernel; ragged in M, N and K."""
    import torch
    import paper_2506_06472_amd as tio
    M, N, K = 5900, 5650, 200
    print(f"large-tile gemm a_km={a_km} b_km={b_km}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(11 + 2 * a_km + b_km)
    r8 = lambda n: (n + 7) // 8 * 8
    lda, ldb, ldc = (r8(M) if a_km else r8(K)), (r8(N) if b_km else r8(K)), r8(N)
    dA = torch.randn((K, lda) if a_km else (M, lda), device="cuda", generator=g).to(torch.bfloat16)
    dB = torch.randn((K, ldb) if b_km else (N, ldb), device="cuda", generator=g).to(torch.bfloat16)
    # padding must never leak into the result
    if a_km: dA[:, M:] = float("nan")
    else: dA[:, K:] = float("nan")
    if b_km: dB[:, N:] = float("nan")
    else: dB[:, K:] = float("nan")
    dC = torch.full((M, ldc), 7.0, device="cuda", dtype=torch.bfloat16)
    dsum = torch.full((r8(M) + 8,), 7.0, device="cuda", dtype=torch.bfloat16)
    torch.cuda.synchronize()
    tio.tio_op_gemm(0, "bf16", a_km, b_km, M, N, K, dA.data_ptr(), lda, dB.data_ptr(), ldb, 0, 0, 0, dC.data_ptr(), ldc,
                    dsum.data_ptr())
    torch.cuda.synchronize()
    A64 = _host(dA)[:, :M].T if a_km else _host(dA)[:, :K]
    B64 = _host(dB)[:, :N].T if b_km else _host(dB)[:, :K]
    ref = A64 @ B64.T
    got = _host(dC)
    assert np.all(got[:, N:] == 7.0)
    err = np.abs(got[:, :N] - ref)
    assert np.all(err <= 2.0 ** -8 * np.abs(ref) + 1e-3 * np.sqrt(K)), float(err.max())
    rs, ref_rs = _host(dsum), A64.sum(1)
    assert np.all(np.abs(rs[:M] - ref_rs) <= 2.0 ** -8 * np.abs(ref_rs) + 1e-3 * np.sqrt(K)) and np.all(rs[M:] == 7.0)


def test_gemm_operand_beyond_32bit_offsets():
    """A k-major operand spanning more than 1 GiB takes the kernel with 64-bit addressing."""
    import torch
    import paper_2506_06472_amd as tio
    M, N, K, lda = 136, 72, 8200, 65544
    g = torch.Generator(device="cuda").manual_seed(5)
    dA = torch.zeros((K, lda), device="cuda", dtype=torch.bfloat16)
    dA[:, :M] = torch.randn((K, M), device="cuda", generator=g).to(torch.bfloat16)
    dB = torch.randn((N, K), device="cuda", generator=g).to(torch.bfloat16)
    dC = torch.full((M, N), 7.0, device="cuda", dtype=torch.bfloat16)
    torch.cuda.synchronize()
    tio.tio_op_gemm(0, "bf16", 1, 0, M, N, K, dA.data_ptr(), lda, dB.data_ptr(), K, 0, 0, 0, dC.data_ptr(), N)
    torch.cuda.synchronize()
    ref = _host(dA[:, :M]).T @ _host(dB).T
    err = np.abs(_host(dC) - ref)
    assert np.all(err <= 2.0 ** -8 * np.abs(ref) + 1e-3 * np.sqrt(K)), float(err.max())


def test_gemm_rejects_bad_arguments():
    import torch
    import paper_2506_06472_amd as tio
    x = torch.zeros(64, 64, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(tio.TioError):
        tio.tio_op_gemm(0, "bf16", 0, 0, 64, 64, 64, x.data_ptr(), 60, x.data_ptr(), 64, 0, 0, 0, x.data_ptr(), 64)
    with pytest.raises(tio.TioError):
        tio.tio_op_gemm(0, "bf16", 0, 0, 64, 64, 64, x.data_ptr() + 2, 64, x.data_ptr(), 64, 0, 0, 0, x.data_ptr(), 64)
    with pytest.raises(tio.TioError):
        tio.tio_op_gemm(0, "bf16", 0, 0, 64, 64, 64, x.data_ptr(), 64, x.data_ptr(), 64, 0, 0, 0, x.data_ptr(), 32)


@pytest.mark.parametrize("M,N,K,splits", [(256, 128, 1024, 4), (200, 136, 1000, 3), (768, 768, 2048, 8), (130, 64, 4096, 2)])
def test_gemm_split_contraction_matches_single_pass(M, N, K, splits):
    """dW-shaped product (both operands k-major) with the contraction cut into ranges: same result as the
    oracle product within bf16 rounding, row sums included, nothing written outside the output."""
    import torch
    import paper_2506_06472_amd as tio
    print(f"split gemm M={M} N={N} K={K} splits={splits}", flush=True)
    rng = np.random.default_rng(M + N + K)
    r8 = lambda n: (n + 7) // 8 * 8
    lda, ldb, ldc = r8(M), r8(N), r8(N)
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((N, K)).astype(np.float32)
    As = np.zeros((K, lda), np.float32); As[:, :M] = A.T
    Bs = np.zeros((K, ldb), np.float32); Bs[:, :N] = B.T
    dA, dB = _dev(As, "bf16"), _dev(Bs, "bf16")
    dC = torch.full((M, ldc), 7.0, device="cuda", dtype=torch.bfloat16)
    dsum = torch.full((r8(M) + 8,), 7.0, device="cuda", dtype=torch.bfloat16)
    ws = torch.full((splits * (M * N + M) + 64,), float("nan"), device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()
    tio.tio_op_gemm(0, "bf16", 1, 1, M, N, K, dA.data_ptr(), lda, dB.data_ptr(), ldb, 0, 0, 0, dC.data_ptr(), ldc,
                    dsum.data_ptr(), ws.data_ptr(), splits)
    torch.cuda.synchronize()
    A64, B64 = _host(dA)[:, :M].T, _host(dB)[:, :N].T
    ref = A64 @ B64.T
    got = _host(dC)
    assert np.all(got[:, N:] == 7.0)
    assert np.all(np.abs(got[:, :N] - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-3 * np.sqrt(K))
    rs = _host(dsum)
    ref_rs = A64.sum(1)
    assert np.all(np.abs(rs[:M] - ref_rs) <= 2.0 ** -8 * np.abs(ref_rs) + 1e-3 * np.sqrt(K)) and np.all(rs[M:] == 7.0)
    assert torch.isnan(ws[splits * (M * N + M):]).all()


@pytest.mark.parametrize("dtype,B,T,H,dh,gain", [
    ("bf16", 2, 256, 3, 64, 1), ("bf16", 1, 200, 2, 64, 1), ("bf16", 2, 128, 2, 128, 1), ("bf16", 1, 330, 1, 128, 1),
    ("bf16", 1, 96, 2, 32, 1), ("fp32", 2, 100, 2, 32, 1), ("fp32", 1, 130, 2, 64, 1), ("bf16", 1, 1024, 2, 64, 1),
    ("bf16", 1, 2048, 1, 128, 1), ("bf16", 1, 4096, 1, 128, 1),
    # queries and keys four times as large: scores of +-50, rows whose maximum keeps rising along the keys, so the softmax's
    # reference exponent is raised many times and by more than the range it tolerates
    ("bf16", 1, 700, 2, 128, 4), ("bf16", 2, 300, 2, 64, 4)])
def test_attention_forward_backward(dtype, B, T, H, dh, gain):
    """Fused causal attention against the plain definition (oracle/model.py) in float64, element by element.

    Bounds (u = 2^-8 for bf16: twice the unit roundoff of a bf16 rounding; 1e-5 for fp32, which accumulates T terms in fp32):
    the kernels round the probabilities P (forward, dV) and the score gradients dS (dQ, dK) to the storage type before the
    second product and the result once more, and the backward pass takes delta = rowsum(dO * O) from the stored O:
      |O  - ref| <= u (|O| + P|V|)                     |dV - ref| <= u (|dV| + P^T |dO|)
      E_i = u sum_d |dO_id| (|O_id| + (P|V|)_id)       (error of delta_i)
      |dQ - ref| <= u |dQ| + (E (P|K|) + u |dS||K|) / sqrt(dh)
      |dK - ref| <= u |dK| + ((P*E)^T |Q| + u |dS|^T |Q|) / sqrt(dh)"""
    import torch
    import paper_2506_06472_amd as tio
    from oracle import model as om
    print(f"attention {dtype} B={B} T={T} H={H} dh={dh} gain={gain}", flush=True)
    rng = np.random.default_rng(B * 1000 + T + H + dh)
    d = H * dh
    qkv = rng.standard_normal((B * T, 3 * d)).astype(np.float32)
    qkv[:, :2 * d] *= gain
    dO = rng.standard_normal((B * T, d)).astype(np.float32)
    tq, tg = _dev(qkv, dtype), _dev(dO, dtype)
    to = torch.full((B * T, d), 7.0, device="cuda", dtype=tq.dtype)
    tdq = torch.full((B * T, 3 * d), 7.0, device="cuda", dtype=tq.dtype)
    lse = torch.zeros(B * H * T, device="cuda", dtype=torch.float32)
    delta = torch.zeros(B * H * T, device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()
    tio.tio_op_attention(0, dtype, B, T, H, dh, tq.data_ptr(), to.data_ptr(), lse.data_ptr(), tg.data_ptr(),
                         delta.data_ptr(), tdq.data_ptr())
    torch.cuda.synchronize()
    x = _host(tq); g = _host(tg)
    heads = lambda a: a.reshape(B, T, H, dh).transpose(0, 2, 1, 3)
    unheads = lambda a: a.transpose(0, 2, 1, 3).reshape(B * T, d)
    q, k, v = (heads(x[:, i * d:(i + 1) * d]) for i in range(3))
    gh = heads(g)
    o_ref, p = om.attention_fwd(q, k, v)
    s = np.matmul(q, np.swapaxes(k, -1, -2)) / np.sqrt(dh)
    s = np.where(np.triu(np.ones((T, T), bool), 1), -np.inf, s)
    lse_ref = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    del s
    dq, dk, dv = om.attention_bwd(gh, q, k, v, p)
    u = 2.0 ** -8 if dtype == "bf16" else 1e-5
    pT = np.swapaxes(p, -1, -2)
    pv = np.matmul(p, np.abs(v))
    o_got = _host(to)
    err = np.abs(o_got - unheads(o_ref))
    bound = unheads(u * (np.abs(o_ref) + pv))
    assert np.all(err <= bound), ("o", float((err / bound).max()))
    assert np.abs(lse.cpu().numpy().reshape(B, H, T) - lse_ref).max() <= (1e-2 if dtype == "bf16" else 1e-4)
    # dS = P * (dO V^T - delta), by the definition
    dP = np.matmul(gh, np.swapaxes(v, -1, -2))
    dS = p * (dP - (gh * o_ref).sum(-1, keepdims=True))
    del dP
    E = u * (np.abs(gh) * (np.abs(o_ref) + pv)).sum(-1, keepdims=True)
    aS = np.abs(dS)
    rs = 1.0 / np.sqrt(dh)
    bounds = (u * np.abs(dq) + (E * np.matmul(p, np.abs(k)) + u * np.matmul(aS, np.abs(k))) * rs,
              u * np.abs(dk) + (np.matmul(pT * np.swapaxes(E, -1, -2), np.abs(q)) + u * np.matmul(np.swapaxes(aS, -1, -2), np.abs(q))) * rs,
              u * (np.abs(dv) + np.matmul(pT, np.abs(gh))))
    got = _host(tdq)
    for i, (ref, bnd) in enumerate(zip((dq, dk, dv), bounds)):
        err = np.abs(got[:, i * d:(i + 1) * d] - unheads(ref))
        assert np.all(err <= unheads(bnd)), ("dq dk dv".split()[i], float((err / unheads(bnd)).max()))
        print("  worst error / bound", "dq dk dv".split()[i], float((err / unheads(bnd)).max()), flush=True)


@pytest.mark.parametrize("T,H,dh", [(200, 2, 64), (330, 1, 128), (70, 1, 128)])
def test_attention_ignores_what_lies_behind_its_buffers(T, H, dh):
    """Tiles of 64 rows reach past the last row of a sequence whose length is not a multiple of 64; the kernels' buffer
    descriptors end with the sequence, so what lies behind qkv and dO in memory must not matter.  Both buffers are views at
    the start of larger allocations: once followed by zeros, once by NaN.  Every output has to be finite and bitwise the
    same in both runs (0 x NaN in a product of a masked probability with a row past the end would show at once)."""
    import torch
    import paper_2506_06472_amd as tio
    print(f"attention behind the buffer T={T} H={H} dh={dh}", flush=True)
    B, d = 1, H * dh
    rng = np.random.default_rng(T + dh)
    qkv = rng.standard_normal((B * T, 3 * d)).astype(np.float32)
    dO = rng.standard_normal((B * T, d)).astype(np.float32)
    outs = []
    for fill in (0.0, float("nan")):
        big_q = torch.full(((B * T + 192) * 3 * d,), fill, device="cuda", dtype=torch.bfloat16)
        big_g = torch.full(((B * T + 192) * d,), fill, device="cuda", dtype=torch.bfloat16)
        big_q[:B * T * 3 * d] = _dev(qkv, "bf16").reshape(-1)
        big_g[:B * T * d] = _dev(dO, "bf16").reshape(-1)
        o = torch.full((B * T, d), 7.0, device="cuda", dtype=torch.bfloat16)
        dq = torch.full((B * T, 3 * d), 7.0, device="cuda", dtype=torch.bfloat16)
        lse = torch.zeros(B * H * T, device="cuda", dtype=torch.float32)
        delta = torch.zeros(B * H * T, device="cuda", dtype=torch.float32)
        torch.cuda.synchronize()
        tio.tio_op_attention(0, "bf16", B, T, H, dh, big_q.data_ptr(), o.data_ptr(), lse.data_ptr(), big_g.data_ptr(),
                             delta.data_ptr(), dq.data_ptr())
        torch.cuda.synchronize()
        outs.append([t.float().cpu().numpy() for t in (o, dq, lse, delta)])
    for a, b in zip(*outs):
        assert np.isfinite(b).all()
        assert a.tobytes() == b.tobytes()


@pytest.mark.parametrize("a_km,b_km", [(0, 0), (0, 1), (1, 1), (1, 0)])
def test_gemm_ignores_what_lies_behind_its_operands(a_km, b_km):
    """Ragged M, N and K: the last tiles of both operands reach past their last row and, in the contraction, past their
    last column.  The operands are views at the start of larger allocations followed by NaN; the product has to equal
    the one computed with zeros behind them, bit for bit, and be finite."""
    import torch
    import paper_2506_06472_amd as tio
    M, N, K = 333, 200, 136
    print(f"gemm behind the operands a_km={a_km} b_km={b_km}", flush=True)
    rng = np.random.default_rng(5 + 2 * a_km + b_km)
    r8 = lambda n: (n + 7) // 8 * 8
    lda, ldb, ldc = (r8(M) if a_km else r8(K)), (r8(N) if b_km else r8(K)), r8(N)
    A = rng.standard_normal((K if a_km else M, lda)).astype(np.float32)
    Bm = rng.standard_normal((K if b_km else N, ldb)).astype(np.float32)
    outs = []
    for fill in (0.0, float("nan")):
        bufs = []
        for X in (A, Bm):
            t = torch.full((X.size + 300 * X.shape[1],), fill, device="cuda", dtype=torch.bfloat16)
            t[:X.size] = _dev(X, "bf16").reshape(-1)
            bufs.append(t)
        C = torch.full((M, ldc), 7.0, device="cuda", dtype=torch.bfloat16)
        torch.cuda.synchronize()
        tio.tio_op_gemm(0, "bf16", a_km, b_km, M, N, K, bufs[0].data_ptr(), lda, bufs[1].data_ptr(), ldb, 0, 0, 0,
                        C.data_ptr(), ldc, 0, 0, 1)
        torch.cuda.synchronize()
        outs.append(C.float().cpu().numpy())
    assert np.isfinite(outs[1][:, :N]).all()
    assert outs[0].tobytes() == outs[1].tobytes()
