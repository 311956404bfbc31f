"""Reference points for the int8 GEMM on the same chip and the same kind of data: the vendor library's int8
GEMM as PyTorch exposes it (torch._int_mm: int8 x int8 -> int32, no epilogue) and a bf16 GEMM of the same shape,
timed with events over back-to-back launches.  Context for the roofline figure of k_gemm_mixed, not a target:
    python3 paper_2407_19775_amd/microbench/int8_gemm_reference_points.py
Operands are Gaussian int8 codes with sigma 32, which is what row / column absmax scaling of Gaussian
activations and weights produces (the clock of this chip under its power limit depends on the operand data)."""
import torch


def timed(fn, iters):
    for _ in range(5):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3        # us


def run(M, K, N, iters):
    g = torch.Generator(device="cuda")
    g.manual_seed(1)
    a = (torch.randn((M, K), device="cuda", generator=g) * 32).clamp(-127, 127).round().to(torch.int8)
    b = (torch.randn((N, K), device="cuda", generator=g) * 32).clamp(-127, 127).round().to(torch.int8)
    for name, bb in (("K-contiguous weights", b.t()), ("N-contiguous weights", b.t().contiguous())):
        us = timed(lambda: torch._int_mm(a, bb), iters)
        print("int8 x int8 -> int32, %s  M=%d K=%d N=%d: %8.1f us  %7.1f TOP/s (%.1f %% of 5000)"
              % (name, M, K, N, us, 2 * M * K * N / us / 1e6, 2 * M * K * N / us / 1e6 / 50), flush=True)
    x = torch.randn((M, K), device="cuda", generator=g).bfloat16()
    w = torch.randn((N, K), device="cuda", generator=g).bfloat16()
    us = timed(lambda: x @ w.t(), iters)
    print("bf16 x bf16 -> bf16                          M=%d K=%d N=%d: %8.1f us  %7.1f TFLOP/s (%.1f %% of 2500)"
          % (M, K, N, us, 2 * M * K * N / us / 1e6, 2 * M * K * N / us / 1e6 / 25), flush=True)


if __name__ == "__main__":
    torch.cuda.set_device(0)
    run(4096, 8192, 8192, 50)       # 70B-shaped output projection
    run(4096, 8192, 57344, 10)      # 70B-shaped gate / up
    run(2048, 4096, 22016, 50)      # 7B-shaped gate / up
    run(8192, 8192, 8192, 20)
