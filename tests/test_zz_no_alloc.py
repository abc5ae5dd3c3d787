"""The entry point that allocates nothing (tio_op_gemm_static_ws) against tio_op_gemm with a caller workspace.

Both run the same kernels, so the outputs must be equal bit for bit; the static array keeps the previous call's
contents, so the second call is a smaller product that would show stale partial tiles if any were read.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _bits(t):
    import torch
    return t.view(torch.int16).cpu().numpy()


def _one(tio, torch, M, N, K, splits, seed):
    print(f"static-workspace gemm M={M} N={N} K={K} splits={splits}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(seed)
    r8 = lambda n: (n + 7) // 8 * 8
    lda, ldb, ldc = r8(M), r8(N), r8(N)
    dA = torch.randn((K, lda), device="cuda", generator=g).to(torch.bfloat16)
    dB = torch.randn((K, ldb), device="cuda", generator=g).to(torch.bfloat16)
    out = []
    for which in ("workspace", "static"):
        dC = torch.full((M, ldc), 7.0, device="cuda", dtype=torch.bfloat16)
        dsum = torch.full((r8(M) + 8,), 7.0, device="cuda", dtype=torch.bfloat16)
        torch.cuda.synchronize()
        if which == "workspace":
            ws = torch.full((splits * (M * N + M),), float("nan"), device="cuda", dtype=torch.float32)
            tio.tio_op_gemm(0, "bf16", 1, 1, M, N, K, dA.data_ptr(), lda, dB.data_ptr(), ldb, 0, 0, 0, dC.data_ptr(), ldc,
                            dsum.data_ptr(), ws.data_ptr(), splits)
        else:
            tio.tio_op_gemm_static_ws(0, "bf16", 1, 1, M, N, K, dA.data_ptr(), lda, dB.data_ptr(), ldb, dC.data_ptr(), ldc,
                                      dsum.data_ptr(), splits)
        torch.cuda.synchronize()
        out.append((_bits(dC), _bits(dsum)))
    (c0, s0), (c1, s1) = out
    assert np.array_equal(c0, c1), "outputs differ between caller workspace and static workspace"
    assert np.array_equal(s0, s1), "row sums differ between caller workspace and static workspace"
    # and the product itself is right (float64 product of the bf16 operands)
    A64 = dA.float().cpu().numpy().astype(np.float64)[:, :M].T
    B64 = dB.float().cpu().numpy().astype(np.float64)[:, :N].T
    ref = A64 @ B64.T
    got = torch.from_numpy(c1.copy()).view(torch.bfloat16).float().numpy().astype(np.float64)
    assert np.all(got[:, N:] == 7.0)
    assert np.all(np.abs(got[:, :N] - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-3 * np.sqrt(K))


def test_static_workspace_gemm_two_calls_in_a_row():
    import torch
    import paper_2506_06472_amd as tio
    _one(tio, torch, 1024, 768, 4096, 8, 1)      # 25 MiB of partial tiles
    _one(tio, torch, 200, 136, 1000, 3, 2)       # smaller, ragged: earlier partials stay in the array around it


def test_static_workspace_gemm_rejects_what_does_not_fit():
    import torch
    import paper_2506_06472_amd as tio
    x = torch.zeros(64, 64, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(tio.TioError, match="static workspace"):
        # 8 * (4096*4096 + 4096) floats = 512 MiB
        tio.tio_op_gemm_static_ws(0, "bf16", 1, 1, 4096, 4096, 64, x.data_ptr(), 4096, x.data_ptr(), 4096, x.data_ptr(), 4096, 0, 8)
    with pytest.raises(tio.TioError):
        tio.tio_op_gemm_static_ws(0, "bf16", 1, 1, 64, 64, 64, x.data_ptr(), 64, x.data_ptr(), 64, x.data_ptr(), 64, 0, 0)
