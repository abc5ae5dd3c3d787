"""The GEMM benchmark tool's shape table against the workloads' parameter counts (no GPU)."""
from paper_2506_06472_amd.gemm_bench import SHAPES, products
from synth import CONFIGS


def _gemm_params(cfg):
    d, f, L, V = cfg["d"], cfg["f"], cfg["L"], cfg["V"]
    ffn = 3 * d * f if cfg["arch"] == "llama" else 2 * d * f
    return L * (3 * d * d + d * d + ffn) + V * d


def test_products_of_a_step_add_up_to_six_flops_per_gemm_parameter_and_token():
    """Forward, input gradient and weight gradient of every linear layer are 2 M N K each: 6 flops per parameter in a GEMM
    and token, the count the roofline of the bench line uses."""
    S = 8192
    for name, key in (("gpt2_small", "gpt2_small_bf16"), ("llama_7b", "llama_7b_bf16"), ("llama_13b", "llama_13b_bf16")):
        rows = list(products(SHAPES[name], S))
        assert len(rows) == 15
        flops = sum(2 * M * N * K * w for _, _, _, M, N, K, _, _, _, w in rows)
        assert flops == 6 * _gemm_params(CONFIGS[key]) * S, name
        for pname, akm, bkm, M, N, K, lda, ldb, ldc, _ in rows:
            # leading dimensions cover the row length of each operand in its layout
            assert lda >= (M if akm else K) and ldb >= (N if bkm else K) and ldc >= N, pname
