"""The one measurement entry of the package: times single library kernels through the C ABI and turns rocprofv3
counter output into the traffic figures bench.py reports.

    python3 paper_2503_12668_amd/measure.py gemm [--dtype bf16|f16|f32] [--n N] [--k K] [--const] [--cold] [--library]
        zo2_op_gemm alone for M = 512 .. 16384: time per launch, TFLOP/s, TFLOP/s per active compute unit.
        --const: operands filled with one value instead of random ones; --cold: every launch takes operands from a
        ring of buffers larger than the memory-side cache (the situation inside a step) instead of the same ones;
        --library: a last column with torch.matmul (the vendor BLAS) on the same buffers, as a yardstick.
    python3 paper_2503_12668_amd/measure.py gemm-phases [--n N] [--k K] [--m M] [--f32-residual]
        needs libzo2_stamps.so (python3 paper_2503_12668_amd/build.py --gemm-stamps).  The large-tile GEMM with one
        workgroup's shader-clock stamps: cycles per tile for the wait for its first k-slab, the k loop (and, inside it, the
        waits for loads and at the barriers in the middle of the slabs) and the epilogue, for four or eight wavefronts per
        workgroup and with both operands, only X, or only W taken from a ring of cold buffers; the launch time next to
        it gives the clock the chip ran at.
    python3 paper_2503_12668_amd/measure.py streams
        what this machine delivers for plain HBM streams issued by the library's own kernels, nothing computed:
        copy (zo2_op_convert float32 -> float32: read 1, write 1), next to the perturbation alone (zo2_op_update_perturb
        with no update: read 1 / write 2, one Gaussian per element) and the fused update + perturb (read 1 / write 3,
        two Gaussians per element); GB/s of algorithmic bytes.
    python3 paper_2503_12668_amd/measure.py small-steps [--model opt-1.3b] [--steps 20] [--shape BxS ...] [--only off|on]
        whole steps of few tokens (default 1 x 16 .. 1 x 512, 4 x 64, 8 x 64), resident bf16: ms per step with the
        perturbation generated in the projections' loader switched off (the sweep writes W+ and W- for every tensor)
        and on, the ratio, and the time the K1 and projection kernels take per step in each mode.  --shape / --only
        restrict the run to some shapes and one mode (for a profiler run).
    python3 paper_2503_12668_amd/measure.py link
        what the host link delivers for 640 MB copies between pinned host memory and HBM (the size of an OPT-13B block
        bucket): host to device alone, device to host alone, and both at once on two streams - the situation of the
        upload and offload streams of a streamed step.
    python3 paper_2503_12668_amd/measure.py copy
        three 1 GiB copies and nothing else: the calibration run for rocprofv3's FETCH_SIZE / WRITE_SIZE counters.
    python3 paper_2503_12668_amd/measure.py traffic --fetch F.csv --write W.csv --cal-fetch CF.csv --cal-write CW.csv \\
            --steps S --out profiles/hbm_traffic_opt1.3b_bf16_resident.json
        reads the counter_collection CSVs of two `rocprofv3 --pmc` runs of bench.py (FETCH_SIZE, WRITE_SIZE) and of
        the two calibration runs of `measure.py copy`, and writes HBM bytes per step and per launch for the GEMM and K1
        kernels (last step of the run), with the scale factors and the commit they were measured at.
"""
import argparse
import csv
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _time_launches(fn, launches):
    import torch
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(launches):
        fn(i)
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) * 1e3 / launches          # microseconds per launch


def cmd_gemm(args):
    import torch

    from paper_2503_12668_amd import binding
    td = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}[args.dtype]
    g = torch.Generator(device="cuda").manual_seed(3)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    tile = 128 if args.dtype == "f32" else 256
    print(f"N {args.n}  K {args.k}  {args.dtype}  operands {'constant' if args.const else 'random N(0, 1)'}, "
          f"{'cold (ring of buffers)' if args.cold else 'hot (same buffers every launch)'}  ({args.launches} launches each)"
          + (f"  {args.waves} wavefronts per workgroup" if args.waves else ""))
    print("| M | tiles | active CUs | us per launch | TFLOP/s | TFLOP/s per active CU |" + (" torch.matmul TFLOP/s |" if args.library else ""))
    print("|---|---|---|---|---|---|" + ("---|" if args.library else ""))
    binding.op_set_gemm_wavefronts(args.waves)
    for m in (args.rows or (512, 1024, 2048, 4096, 8192, 16384)):
        esz = 4 if args.dtype == "f32" else 2
        nbuf = max(1, min(16, int(600e6 // ((m + args.n) * args.k * esz)) + 1)) if args.cold else 1
        if args.const:
            Xs = [torch.full((m, args.k), 0.5, dtype=td, device="cuda") for _ in range(nbuf)]
            Ws = [torch.full((args.n, args.k), 0.25, dtype=td, device="cuda") for _ in range(nbuf)]
        else:
            Xs = [torch.randn(m, args.k, device="cuda", generator=g).to(td) for _ in range(nbuf)]
            Ws = [torch.randn(args.n, args.k, device="cuda", generator=g).to(td) for _ in range(nbuf)]
        Y = torch.empty(m, args.n, dtype=td, device="cuda")
        for i in range(5):
            binding.op_gemm(Xs[i % nbuf], Ws[i % nbuf], Y=Y)
        us = _time_launches(lambda i: binding.op_gemm(Xs[i % nbuf], Ws[i % nbuf], Y=Y), args.launches)
        tiles = ((m + tile - 1) // tile) * ((args.n + tile - 1) // tile)
        active = min(tiles, cus * (2 if args.dtype == "f32" else 1))
        tf = 2.0 * m * args.n * args.k / us / 1e6
        extra = ""
        if args.library:
            WT = [w.t() for w in Ws]
            for i in range(5):
                torch.matmul(Xs[i % nbuf], WT[i % nbuf], out=Y)
            us_l = _time_launches(lambda i: torch.matmul(Xs[i % nbuf], WT[i % nbuf], out=Y), args.launches)
            extra = f" {2.0 * m * args.n * args.k / us_l / 1e6:.1f} |"
        print(f"| {m} | {tiles} | {min(active, cus)} | {us:.1f} | {tf:.1f} | {tf / min(active, cus):.2f} |" + extra, flush=True)


def cmd_gemm_phases(args):
    import torch

    from paper_2503_12668_amd import binding, build
    if not os.path.exists(build.LIB_STAMPS):
        sys.exit("measure.py gemm-phases: libzo2_stamps.so is not built (python3 paper_2503_12668_amd/build.py --gemm-stamps)")
    binding.LIB_PATH = build.LIB_STAMPS
    M, N, K = args.m, args.n, args.k
    g = torch.Generator(device="cuda").manual_seed(3)
    ring = max(2, int(600e6 // ((M + N) * K * 2)) + 1)
    Xs = [torch.randn(M, K, device="cuda", generator=g).bfloat16() for _ in range(ring)]
    Ws = [torch.randn(N, K, device="cuda", generator=g).bfloat16() for _ in range(ring)]
    out32 = args.f32_residual
    Y = torch.empty(M, N, device="cuda", dtype=torch.float32 if out32 else torch.bfloat16)
    R = torch.zeros(M, N, device="cuda") if out32 else None
    stamps = torch.zeros(64, dtype=torch.int64, device="cuda")
    tiles_per_cu = ((M + 255) // 256) * ((N + 255) // 256) / torch.cuda.get_device_properties(0).multi_processor_count
    print(f"M {M}  N {N}  K {K}  bf16, random N(0, 1) operands, {'float32 output + residual' if out32 else 'bf16 output'}; "
          f"{tiles_per_cu:.2f} tiles of 256 x 256 per compute unit; pure MFMA issue of a tile's k loop: {K // 32 * 64 * 16} cycles per SIMD")
    print("| wavefronts | X | W | us per launch | TFLOP/s | cycles per tile: wait for first slab | k loop | of it: waiting for loads | at the mid-slab barrier | epilogue | clock GHz |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for i in range(1000):        # the first launches of a process run at another clock: let it settle before the first row
        binding.op_gemm_phases(Xs[0], Ws[0], Y, stamps, residual=R)
    for waves in (4, 8):
        binding.op_set_gemm_wavefronts(waves)
        for cx, cw in ((False, False), (False, True), (True, False), (True, True)):
            f = lambda i: binding.op_gemm_phases(Xs[i % ring if cx else 0], Ws[i % ring if cw else 0], Y, stamps, residual=R)
            for i in range(5):
                f(i)
            us = _time_launches(f, args.launches)
            st = stamps.cpu().numpy().astype("int64")
            nt = int(st[62])
            ph = [[int(st[4 * t + k + 1] - st[4 * t + k]) for k in range(3)] for t in range(nt)]
            mean = [sum(p[k] for p in ph) / nt for k in range(3)]
            total = int(st[4 * nt - 1] - st[0])
            print(f"| {waves} | {'cold' if cx else 'hot'} | {'cold' if cw else 'hot'} | {us:.1f} | {2.0 * M * N * K / us / 1e6:.0f} | {mean[0]:.0f} | {mean[1]:.0f} | "
                  f"{st[60] / nt:.0f} | {st[61] / nt:.0f} | {mean[2]:.0f} | {total / us / 1e3:.2f} |", flush=True)
    binding.op_set_gemm_wavefronts(0)


def cmd_streams(args):
    import torch

    from paper_2503_12668_amd import binding
    n = args.elements
    g = torch.Generator(device="cuda").manual_seed(5)
    print(f"{n} elements per launch, {args.launches} launches each, buffers rotated over {args.ring} sets")
    print("| stream | bytes per element | us per launch | GB/s |")
    print("|---|---|---|---|")
    ring = args.ring
    # copy: float32 -> float32
    src = [torch.randn(n // 2, device="cuda", generator=g) for _ in range(ring)]
    dst = [torch.empty(n // 2, device="cuda") for _ in range(ring)]
    for i in range(3):
        binding.op_convert(src[i % ring], dst[i % ring])
    us = _time_launches(lambda i: binding.op_convert(src[i % ring], dst[i % ring]), args.launches)
    print(f"| copy (convert float32 -> float32), read 1 / write 1 | 8 (over {n // 2} elements) | {us:.1f} | {n // 2 * 8 / us / 1e3:.0f} |", flush=True)
    del src, dst
    th = [(torch.randn(n, device="cuda", generator=g) * 0.02).bfloat16() for _ in range(ring)]
    wp = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(ring)]
    wm = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(ring)]
    cases = [("perturb only: read 1 / write 2, one Gaussian per element (bf16)", 6, dict(has_pending=False, eps=1e-3)),
             ("fused update + perturb: read 1 / write 3, two Gaussians per element", 8, dict(has_pending=True, eps=1e-3))]
    for name, bpe, kw in cases:
        f = lambda i: binding.op_update_perturb(th[i % ring], wp[i % ring], wm[i % ring], 7, 0, kw["has_pending"], 41, 1e-9, 42, kw["eps"])
        for i in range(3):
            f(i)
        us = _time_launches(f, args.launches)
        print(f"| {name} | {bpe} | {us:.1f} | {n * bpe / us / 1e3:.0f} |", flush=True)


def cmd_small_steps(args):
    import time
    import torch
    import synth_inputs as si
    from paper_2503_12668_amd import binding
    cfg = si.opt_config(args.model)
    P = si.make_weights(cfg, seed=1)
    ctx = binding.Zo2Context(cfg, P, wire="bf16", compute="bf16", arena_bytes=args.arena_gib << 30)
    print(f"# {args.model} shape, bf16 resident; ms per step (mean of {args.steps}); k1 / gemm = their kernels' ms per step",
          flush=True)
    print("| batch x seq | off: ms | k1 | gemm | on: ms | k1 | gemm | off / on |", flush=True)
    print("|---|---|---|---|---|---|---|---|", flush=True)
    shapes = [tuple(int(v) for v in sh.lower().split("x")) for sh in args.shape] if args.shape else \
        [(1, 16), (1, 64), (1, 128), (1, 256), (4, 64), (8, 64), (1, 512)]
    modes = {"off": (-1,), "on": (1,), None: (-1, 1)}[args.only]
    for (B, S) in shapes:
        tok = si.make_tokens(cfg["vocab"], B, S, seed=2, dist="zipf")
        lab = si.next_token_labels(tok)
        row = []
        for mode in modes:
            ctx.set_loader_fusion(mode)
            for j in range(3):
                ctx.step(tok, lab, 42 + j, 1e-3, 1e-7)
            active = ctx.plan()["loader_fusion"]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for j in range(args.steps):
                ctx.step(tok, lab, 50 + j, 1e-3, 1e-7)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) / args.steps * 1e3
            ctx.set_profiling(("gemm", "k1"))
            acc = {"gemm": 0.0, "k1": 0.0}
            for j in range(5):
                ctx.step(tok, lab, 80 + j, 1e-3, 1e-7)
                for k, (m, n) in ctx.kernel_times().items():
                    if k in acc:
                        acc[k] += m / 5
            ctx.set_profiling(())
            row.append((ms, acc["k1"], acc["gemm"], active))
        if len(row) == 1:
            m, k, g, a = row[0]
            print(f"| {B} x {S} | {args.only}{'' if a or args.only == 'off' else ' (not applicable)'}: {m:.2f} | {k:.2f} | {g:.2f} |", flush=True)
            continue
        (m0, k0, g0, a0), (m1, k1, g1, a1) = row
        on = f"{m1:.2f} | {k1:.2f} | {g1:.2f}" if a1 else "not applicable | | "
        print(f"| {B} x {S} | {m0:.2f} | {k0:.2f} | {g0:.2f} | {on} | {m0 / m1:.2f} |", flush=True)
    ctx.close()


def cmd_link(args):
    import time
    import torch
    n = 160 * 1024 * 1024                              # float32 elements: 640 MB
    h_up = torch.ones(n, dtype=torch.float32).pin_memory()
    h_down = torch.empty(n, dtype=torch.float32).pin_memory()
    d_up = torch.empty(n, dtype=torch.float32, device="cuda")
    d_down = torch.ones(n, dtype=torch.float32, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    def both():
        with torch.cuda.stream(s1):
            d_up.copy_(h_up, non_blocking=True)
        with torch.cuda.stream(s2):
            h_down.copy_(d_down, non_blocking=True)

    gb = n * 4 / 1e9
    print("| copy of 640 MB (pinned host memory, asynchronous copies) | GB/s |")
    print("|---|---|")
    print(f"| host to device alone | {gb / timed(lambda: d_up.copy_(h_up, non_blocking=True)):.1f} |")
    print(f"| device to host alone | {gb / timed(lambda: h_down.copy_(d_down, non_blocking=True)):.1f} |")
    print(f"| both at once, two streams | {gb / timed(both):.1f} each way |")


def cmd_copy(args):
    import torch

    from paper_2503_12668_amd import binding
    n = (1 << 30) // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        binding.op_convert(src, dst)
    torch.cuda.synchronize()
    print("copied 3 x 1 GiB")


def _counter_rows(path, counter):
    """(kernel name, counter value) per dispatch, in dispatch order, from a rocprofv3 counter_collection CSV."""
    out = []
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            if row.get("Counter_Name") == counter:
                out.append((int(row["Dispatch_Id"]), row["Kernel_Name"], float(row["Counter_Value"])))
    out.sort()
    return [(k, v) for _, k, v in out]


def cmd_traffic(args):
    GIB_KIB = float(1 << 20)                       # the calibration copy moves 1 GiB each way; counters are in KiB
    def cal(path, counter):
        vals = [v for k, v in _counter_rows(path, counter) if "convert" in k]
        return GIB_KIB / (sum(vals) / len(vals))
    kf, kw = cal(args.cal_fetch, "FETCH_SIZE"), cal(args.cal_write, "WRITE_SIZE")
    res = {}
    for cls, pat in (("gemm", "gemm_mfma256_kernel"), ("k1", "k1_kernel")):
        per = {}
        for counter, path, k in (("FETCH_SIZE", args.fetch, kf), ("WRITE_SIZE", args.write, kw)):
            vals = [v for name, v in _counter_rows(path, counter) if pat in name]
            n = int(round(len(vals) / args.steps))   # launches per step (the first step, with nothing pending, has one fewer K1 launch); the last step of the run is the steady state
            last = vals[-n:]
            per[counter] = (sum(last) * 1024.0 * k, n)
        launches = per["FETCH_SIZE"][1]
        total = per["FETCH_SIZE"][0] + per["WRITE_SIZE"][0]
        res[cls] = {"kernel": pat, "launches_per_step": launches, "fetch_bytes_per_step": per["FETCH_SIZE"][0],
                    "write_bytes_per_step": per["WRITE_SIZE"][0], "bytes_per_step": total, "bytes_per_launch": total / launches}
    try:
        commit = subprocess.check_output(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], text=True).strip()
    except Exception:
        commit = None
    out = {"workload": args.workload, "measured_at_commit": commit, "steps_in_run": args.steps,
           "scale": {"FETCH_SIZE": kf, "WRITE_SIZE": kw,
                     "note": "bytes moved by a 1 GiB copy / KiB the counter reported for it"},
           "kernels": res}
    with open(args.out, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(json.dumps(out, indent=1))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    g = sub.add_parser("gemm")
    g.add_argument("--n", type=int, default=2048)
    g.add_argument("--k", type=int, default=2048)
    g.add_argument("--dtype", default="bf16", choices=["bf16", "f16", "f32"])
    g.add_argument("--const", action="store_true")
    g.add_argument("--cold", action="store_true")
    g.add_argument("--library", action="store_true")
    g.add_argument("--launches", type=int, default=50)
    g.add_argument("--waves", type=int, default=0, choices=[0, 4, 8], help="wavefronts per workgroup for 256-row tiles (0: chosen per launch)")
    g.add_argument("--rows", type=int, nargs="*", default=None, help="row counts M to run (default: 512 .. 16384)")
    gp = sub.add_parser("gemm-phases")
    gp.add_argument("--m", type=int, default=8192)
    gp.add_argument("--n", type=int, default=8192)
    gp.add_argument("--k", type=int, default=2048)
    gp.add_argument("--f32-residual", action="store_true", help="float32 output with a residual (the attention-output / FC2 epilogue)")
    gp.add_argument("--launches", type=int, default=100)
    s = sub.add_parser("streams")
    s.add_argument("--elements", type=int, default=100 * 1024 * 1024)
    s.add_argument("--ring", type=int, default=4)
    s.add_argument("--launches", type=int, default=40)
    sub.add_parser("copy")
    sub.add_parser("link")
    ss = sub.add_parser("small-steps")
    ss.add_argument("--model", default="opt-1.3b")
    ss.add_argument("--steps", type=int, default=20)
    ss.add_argument("--arena-gib", type=int, default=20)
    ss.add_argument("--shape", action="append", help="BxS, e.g. 1x16 (repeatable)")
    ss.add_argument("--only", choices=["off", "on"], default=None)
    t = sub.add_parser("traffic")
    for k in ("fetch", "write", "cal-fetch", "cal-write", "out"):
        t.add_argument("--" + k, required=True)
    t.add_argument("--steps", type=int, required=True)
    t.add_argument("--workload", default="opt-1.3b shape, bf16 resident, batch 16 x seq 256 (bench.py)")
    args = ap.parse_args()
    {"gemm": cmd_gemm, "gemm-phases": cmd_gemm_phases, "streams": cmd_streams, "copy": cmd_copy, "link": cmd_link, "small-steps": cmd_small_steps, "traffic": cmd_traffic}[args.cmd](args)


if __name__ == "__main__":
    main()
