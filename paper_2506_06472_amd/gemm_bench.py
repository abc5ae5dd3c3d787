"""Times tio_op_gemm (bf16) on the GEMM shapes of a workload's training step, through the C ABI.

  python -m paper_2506_06472_amd.gemm_bench --shapes llama_7b --data normal small_int zero

For every linear layer of the model (QKV, attention output, FFN up/gate and down, vocabulary head) the three
products of a step are timed: forward y = x W^T, input gradient dx = dy W, weight gradient dW = dy^T x, with
S = 8192 tokens.  Operands are resident in device memory; the time is the average over --reps back-to-back launches
between two HIP events on the launch stream.  --data chooses the operand values: standard normal (what random-init
training sees), multiples of 1/4 in [-1, 1) (few mantissa bits set), or zeros.  The rate depends on it because the
chip's clock under matrix-core load depends on how many bits toggle: the same launches run faster on zeros.
--vendor times the same products through torch.matmul (the vendor's GEMM library) instead: a yardstick measured on the
same box with the same operands, nothing the library or its tests use.
"""
import argparse

SHAPES = {  # name -> [(layer, n_out, n_in, leading dimension of y or None, launches per step)]
    "gpt2_small": [("qkv", 2304, 768, None, 12), ("o", 768, 768, None, 12), ("fc1", 3072, 768, None, 12),
                   ("fc2", 768, 3072, None, 12), ("head", 50257, 768, 50304, 1)],
    "llama_7b": [("qkv", 12288, 4096, None, 32), ("o", 4096, 4096, None, 32), ("gate_up", 22016, 4096, None, 32),
                 ("down", 4096, 11008, None, 32), ("head", 32000, 4096, None, 1)],
    "llama_13b": [("qkv", 15360, 5120, None, 40), ("o", 5120, 5120, None, 40), ("gate_up", 27648, 5120, None, 40),
                  ("down", 5120, 13824, None, 40), ("head", 32000, 5120, None, 1)],
}


def products(shapes, S):
    for name, nout, nin, ldy, w in shapes:
        ldy = ldy or nout
        yield name + ".fwd", 0, 0, S, nout, nin, nin, nin, ldy, w
        yield name + ".dx", 0, 1, S, nin, nout, ldy, nin, nin, w
        yield name + ".dw", 1, 1, nout, nin, S, ldy, nin, nin, w


def operand(torch, rows, cols, data):
    if data == "normal":
        return torch.randn((rows, cols), device="cuda", dtype=torch.bfloat16)
    if data == "small_int":
        return (torch.randint(-4, 4, (rows, cols), device="cuda").float() * 0.25).to(torch.bfloat16)
    return torch.zeros((rows, cols), device="cuda", dtype=torch.bfloat16)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shapes", default="llama_7b", choices=sorted(SHAPES))
    ap.add_argument("--data", nargs="+", default=["normal"], choices=["normal", "small_int", "zero"])
    ap.add_argument("--tokens", type=int, default=8192)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--vendor", action="store_true", help="time torch.matmul on the same products instead of tio_op_gemm")
    args = ap.parse_args()
    import torch
    import paper_2506_06472_amd as tio
    st = torch.cuda.current_stream().cuda_stream
    for data in args.data:
        tot_f = tot_t = 0.0
        print(f"shapes {args.shapes}, {args.tokens} tokens, operands: {data}" + (", torch.matmul" if args.vendor else ""), flush=True)
        for name, akm, bkm, M, N, K, lda, ldb, ldc, weight in products(SHAPES[args.shapes], args.tokens):
            A = operand(torch, K if akm else M, lda, data)
            B = operand(torch, K if bkm else N, ldb, data)
            C = torch.empty((M, ldc), device="cuda", dtype=torch.bfloat16)
            splits = 1
            if akm and bkm:        # the split the training schedule uses for weight gradients with few tiles
                tiles = ((M + 127) // 128) * ((N + 127) // 128)
                while splits < 8 and tiles * splits * 2 <= 512 and K // (splits * 2) >= 256:
                    splits *= 2
            ws = torch.empty((splits * (M * N + M),), device="cuda", dtype=torch.float32) if splits > 1 else None

            def launch():
                if args.vendor:       # C[M, N] = op(A) op(B)^T on the same buffers: a k-major operand is stored [K, rows]
                    a = A[:, :M].t() if akm else A[:, :K]
                    b = B[:, :N] if bkm else B[:, :K].t()
                    torch.matmul(a, b, out=C[:, :N]) if ldc == N else C[:, :N].copy_(torch.matmul(a, b))
                    return
                tio.tio_op_gemm(st, "bf16", akm, bkm, M, N, K, A.data_ptr(), lda, B.data_ptr(), ldb, 0, 0, 0,
                                C.data_ptr(), ldc, 0, ws.data_ptr() if ws is not None else 0, splits)
            # untimed launches first: the clock takes some tenths of a second of load to ramp up after idling, so the
            # first product of a run gets more of them
            for _ in range(max(3, args.reps // 2) if tot_t else 300):
                launch()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.reps):
                launch()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / args.reps
            fl = 2.0 * M * N * K
            tot_f += fl * weight
            tot_t += us * weight
            print(f"  {name:12s} M={M:6d} N={N:6d} K={K:6d} {us:9.1f} us {fl / us / 1e6:8.1f} TFLOP/s"
                  + (f"  split-K {splits}" if splits > 1 and not args.vendor else ""), flush=True)
        print(f"  all GEMM launches of a step: {tot_t / 1e3:.2f} ms, {tot_f / tot_t / 1e6:.1f} TFLOP/s "
              f"({tot_f / tot_t / 1e6 / 2500:.3f} of 2.5 PFLOP/s)", flush=True)


if __name__ == "__main__":
    main()
