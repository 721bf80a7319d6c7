"""Times the library's bf16 MFMA GEMM entry point (pg_gemm_bf16) on one shape.

    python -m paper_2512_15347_amd.gemm_probe --m 8192 --n 8192 --k 8192 --operands random

--operands zeros / ints / random chooses the operand values: the throughput of this part depends on them
(the switching activity of the operand bits moves the shader clock), so a figure is only meaningful together
with the operand distribution.  Prints one line per repetition block.
"""
import argparse


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--m", type=int, default=8192)
    ap.add_argument("--n", type=int, default=8192)
    ap.add_argument("--k", type=int, default=8192)
    ap.add_argument("--operands", choices=["random", "zeros", "ints"], default="random")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--blocks", type=int, default=3)
    args = ap.parse_args()
    import torch
    from . import binding as pg
    M, N, K = args.m, args.n, args.k
    if args.operands == "random":
        A = torch.randn(M, K, device="cuda"); W = torch.randn(N, K, device="cuda") * 0.02
    elif args.operands == "ints":
        A = torch.randint(-2, 3, (M, K), device="cuda").float(); W = torch.randint(-2, 3, (N, K), device="cuda").float()
    else:
        A = torch.zeros(M, K, device="cuda"); W = torch.zeros(N, K, device="cuda")
    A = A.to(torch.bfloat16).view(torch.int16); W = W.to(torch.bfloat16).view(torch.int16)
    C = torch.empty(M, N, device="cuda")
    for _ in range(3):
        pg.pg_gemm_bf16(A, K, W, K, None, C, N, M, N, K)
    torch.cuda.synchronize()
    for b in range(args.blocks):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.reps):
            pg.pg_gemm_bf16(A, K, W, K, None, C, N, M, N, K)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.reps
        print(f"gemm {M}x{N}x{K} {args.operands}: {ms * 1e3:.1f} us  {2.0 * M * N * K / ms / 1e9:.1f} TFLOP/s", flush=True)


if __name__ == "__main__":
    main()
