"""Plain copy of known size through the library's format-conversion kernel (float32 -> float32), used to
calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE counters:

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d <out> -- python3 paper_2503_12668_amd/pmc_calibrate.py

Each launch reads 1 GiB and writes 1 GiB."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    import torch

    from paper_2503_12668_amd import binding
    n = (1 << 30) // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        binding.op_convert(src, dst)
    torch.cuda.synchronize()
    print("copied 3 x 1 GiB")


if __name__ == "__main__":
    main()
