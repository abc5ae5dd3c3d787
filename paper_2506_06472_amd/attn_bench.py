"""Times tio_op_attention (bf16, causal) on the attention shapes of the workloads, through the C ABI.

  python -m paper_2506_06472_amd.attn_bench --shapes gpt2_small llama_7b llama_13b llama_30b

Forward alone, and forward plus backward (row-sum pre-pass, dQ launch, dK/dV launches): operands resident in device
memory, standard normal values, the average over --reps back-to-back calls between two HIP events on the launch
stream.  The rates count the algorithmic flops of causal attention: 4 B H T^2 dh / 2 forward, 2.5 times that backward
(what the kernels execute is more: the backward launches recompute the scores, and tiles on the diagonal are computed
whole).  --vendor times torch's scaled_dot_product_attention (the vendor's fused attention) on the same shapes instead,
on contiguous [B, H, T, dh] operands made outside the timed region: a yardstick, nothing the library or its tests use.
"""
import argparse

SHAPES = {  # name -> (B, T, H, dh): batch x sequence = 8192 tokens
    "gpt2_small": (8, 1024, 12, 64),
    "llama_7b": (4, 2048, 32, 128),
    "llama_13b": (4, 2048, 40, 128),
    "llama_30b": (2, 4096, 52, 128),
}


def flops_forward(B, T, H, dh):
    return 4.0 * B * H * T * T * dh / 2


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shapes", nargs="+", default=list(SHAPES), choices=sorted(SHAPES))
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--vendor", action="store_true", help="time torch's scaled_dot_product_attention instead of tio_op_attention")
    args = ap.parse_args()
    import torch
    import paper_2506_06472_amd as tio
    st = torch.cuda.current_stream().cuda_stream
    for name in args.shapes:
        B, T, H, dh = SHAPES[name]
        d = H * dh
        qkv = torch.randn((B * T, 3 * d), device="cuda", dtype=torch.bfloat16)
        dO = torch.randn((B * T, d), device="cuda", dtype=torch.bfloat16)
        o = torch.empty((B * T, d), device="cuda", dtype=torch.bfloat16)
        dqkv = torch.empty_like(qkv)
        lse = torch.empty((B * H * T,), device="cuda", dtype=torch.float32)
        delta = torch.empty_like(lse)

        def forward():
            tio.tio_op_attention(st, "bf16", B, T, H, dh, qkv.data_ptr(), o.data_ptr(), lse.data_ptr())

        def both():
            tio.tio_op_attention(st, "bf16", B, T, H, dh, qkv.data_ptr(), o.data_ptr(), lse.data_ptr(), dO.data_ptr(),
                                 delta.data_ptr(), dqkv.data_ptr())
        if args.vendor:
            import torch.nn.functional as F
            q, k, v = (qkv[:, i * d:(i + 1) * d].reshape(B, T, H, dh).permute(0, 2, 1, 3).contiguous().requires_grad_(True)
                       for i in range(3))
            g = dO.reshape(B, T, H, dh).permute(0, 2, 1, 3).contiguous()

            def forward():
                with torch.no_grad():
                    F.scaled_dot_product_attention(q, k, v, is_causal=True)

            def both():
                out = F.scaled_dot_product_attention(q, k, v, is_causal=True)
                out.backward(g)
                q.grad = k.grad = v.grad = None
        us = []
        for call in (forward, both):
            # untimed calls first: the clock takes tenths of a second of load to ramp up after idling
            for _ in range(3 if name != args.shapes[0] or us else 200):
                call()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.reps):
                call()
            e1.record()
            torch.cuda.synchronize()
            us.append(e0.elapsed_time(e1) * 1e3 / args.reps)
        fwd, bwd = us[0], us[1] - us[0]
        fl = flops_forward(B, T, H, dh)
        print(("torch sdpa " if args.vendor else "") + f"{name:11s} B={B} T={T} H={H} dh={dh}: forward {fwd:8.1f} us {fl / fwd / 1e6:7.1f} TFLOP/s | "
              f"backward {bwd:8.1f} us {2.5 * fl / bwd / 1e6:7.1f} TFLOP/s", flush=True)


if __name__ == "__main__":
    main()
