"""Time the library's GEMM (zo2_op_gemm) alone, with HIP events on torch's current stream.

    python3 paper_2503_12668_amd/gemm_bench.py [--n 2048] [--k 2048] [--dtype bf16] [--const]

For M = 512 .. 16384 rows (2 .. 64 rows of 256 x 256 tiles; with N = 2048 that is 16 .. 512 tiles, i.e. up to 256
of them one tile per compute unit) it prints the time of a launch and the rate per active compute unit.  Every
tile does the same work on its own compute unit, so what changes along the table is only how many compute units
work at the same time.  --const fills the operands with one value instead of random ones."""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=2048)
    ap.add_argument("--k", type=int, default=2048)
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f16"])
    ap.add_argument("--const", action="store_true")
    ap.add_argument("--launches", type=int, default=50)
    args = ap.parse_args()

    import torch

    from paper_2503_12668_amd import binding
    td = torch.bfloat16 if args.dtype == "bf16" else torch.float16
    g = torch.Generator(device="cuda").manual_seed(3)
    print(f"N {args.n}  K {args.k}  {args.dtype}  operands {'constant' if args.const else 'random N(0, 1)'}  ({args.launches} launches each)")
    print("| M | tiles | active CUs | us per launch | TFLOP/s | TFLOP/s per active CU |")
    print("|---|---|---|---|---|---|")
    for m in (512, 1024, 2048, 4096, 8192, 16384):
        if args.const:
            X = torch.full((m, args.k), 0.5, dtype=td, device="cuda")
            W = torch.full((args.n, args.k), 0.25, dtype=td, device="cuda")
        else:
            X = torch.randn(m, args.k, device="cuda", generator=g).to(td)
            W = torch.randn(args.n, args.k, device="cuda", generator=g).to(td)
        Y = torch.empty(m, args.n, dtype=td, device="cuda")
        for _ in range(5):
            binding.op_gemm(X, W, Y=Y)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.launches):
            binding.op_gemm(X, W, Y=Y)
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / args.launches
        tiles = ((m + 255) // 256) * ((args.n + 255) // 256)
        cus = min(tiles, torch.cuda.get_device_properties(0).multi_processor_count)
        tf = 2.0 * m * args.n * args.k / us / 1e6
        print(f"| {m} | {tiles} | {cus} | {us:.1f} | {tf:.0f} | {tf / cus:.2f} |", flush=True)


if __name__ == "__main__":
    main()
