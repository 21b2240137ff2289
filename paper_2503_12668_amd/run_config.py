"""Run the ZO2 step on one of the OPT-shaped workloads and print one JSON line of measurements.

    python -m paper_2503_12668_amd.run_config --model opt-13b --batch 8 --seq 512 --wire bf16 \\
        --slots 3 --steps 5

Weights are synthetic (N(0, 0.02), LayerNorm gain 1 / bias 0), generated on the GPU with torch's generator
and copied to pinned host buckets in the transfer format (--no-pin: pageable ones, for fully resident runs of the
larger shapes: the host copy is then only read once, at set-up).  --slots N caps the HBM budget so that exactly N
blocks fit (streamed mode, Alg. 3); --budget-bytes sets the cap directly; neither = everything resident.
--layers trims the depth (per-block numbers stay those of the full-width model)."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def gpu_weight_source(seed=1, std=0.02):
    import torch
    gen = torch.Generator(device="cuda").manual_seed(seed)

    def source(name, shape):
        is_ln = ".ln" in name or name.startswith("final_ln")
        if is_ln:
            return torch.ones(shape, device="cuda") if name.endswith(".w") else torch.zeros(shape, device="cuda")
        return torch.randn(shape, device="cuda", generator=gen) * std
    return source


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="opt-13b")
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--seq", type=int, default=512)
    ap.add_argument("--wire", default="bf16")
    ap.add_argument("--compute", default="bf16")
    ap.add_argument("--slots", type=int, default=None)
    ap.add_argument("--budget-bytes", type=float, default=None)
    ap.add_argument("--arena-gb", type=float, default=None)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--eps", type=float, default=1e-3)
    ap.add_argument("--lr", type=float, default=1e-7)
    ap.add_argument("--fp8-scale", type=float, default=64.0)
    ap.add_argument("--directions", type=int, default=1, help="directions per update (1 = the paper's estimator; q > 1: one step + q - 1 extra directions per round, eta / q each)")
    ap.add_argument("--no-overlap", action="store_true", help="ablation: upload, compute, offload of a block strictly in sequence")
    ap.add_argument("--flush-each-step", action="store_true", help="ablation: no deferred update (every block travels twice per step)")
    ap.add_argument("--one-pass", action="store_true", help="with --directions q > 1: the whole round in one pass over the model (zo2_step_multi: a streamed block is uploaded once per round)")
    ap.add_argument("--writeback-interval", type=int, default=1, help="streamed blocks go back to the host once their host copy would lack this many updates (1: after every update, as in the paper's schedule)")
    ap.add_argument("--no-split-k", action="store_true", help="never split a projection along k (for comparison)")
    ap.add_argument("--no-pin", action="store_true", help="pageable host buckets: for fully resident runs of models whose buckets exceed what the box lets a process pin")
    args = ap.parse_args()

    import numpy as np
    import torch

    import synth_inputs as si
    from paper_2503_12668_amd import binding

    cfg = si.opt_config(args.model, n_layers=args.layers)
    cfg["max_pos"] = max(cfg["max_pos"], args.seq)        # sequence sweeps beyond 2048 extend the position table
    L = cfg["n_layers"]
    tok = si.make_tokens(cfg["vocab"], args.batch, args.seq, seed=2, dist="zipf")
    lab = si.next_token_labels(tok)
    scales = None
    if args.wire.startswith("fp8"):
        scales = np.full(4 + 16 * L + (0 if cfg["tied"] else 1), args.fp8_scale, dtype=np.float32)
    t0 = time.time()
    wsz = binding.lib().zo2_dtype_size(binding.DTYPE_ID[args.wire])
    bucket_bytes = binding.block_tensor_offsets(binding.make_config(cfg, args.wire, args.compute))[16] * wsz
    arena = int(args.arena_gb * 2 ** 30) if args.arena_gb else None
    if arena is None and (args.slots or args.budget_bytes):
        arena = int(args.budget_bytes) if args.budget_bytes else 64 << 30
    ctx = binding.Zo2Context(cfg, gpu_weight_source(), wire=args.wire, compute=args.compute, arena_bytes=arena, scales=scales, pin=not args.no_pin)
    setup_s = time.time() - t0
    if args.no_split_k:
        ctx.set_split_k(-1)
    ctx.set_writeback_interval(args.writeback_interval)
    if args.budget_bytes:
        ctx.set_resident_budget(int(args.budget_bytes))
    T = args.batch * args.seq
    q = max(1, args.directions)
    one_pass = args.one_pass and q > 1
    if one_pass:                                             # plans with the whole arena (and the residual streams of q directions)
        res = ctx.step_multi(tok, lab, [41 + i for i in range(q)], args.eps, args.lr / q)[-1]
    else:
        res = ctx.step(tok, lab, 41, args.eps, args.lr)      # plans with the whole arena
    if args.slots:
        used = ctx.plan()["bytes_used"]
        # a resident plan holds L slots; keep exactly `slots` of them
        ctx.set_resident_budget(used - (L - args.slots) * bucket_bytes)
    if args.no_overlap:
        ctx.set_stream_overlap(False)
    for j in range(args.warmup):
        res = ctx.step(tok, lab, 42 + j, args.eps, args.lr)
        if args.flush_each_step:
            ctx.flush()
    plan = ctx.plan()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    up = down = 0
    ms_u = ms_o = ms_c = 0.0
    for j in range(args.steps):      # a "step" of the output below is one round of q directions
        for i in range(1 if one_pass else q):
            if one_pass:
                res = ctx.step_multi(tok, lab, [100 + 16 * j + k for k in range(q)], args.eps, args.lr / q)[-1]
            else:
                res = (ctx.step if i == 0 else ctx.step_extra)(tok, lab, 100 + 16 * j + i, args.eps, args.lr / q)
            st = ctx.step_stats()
            up += st["bytes_up"]; down += st["bytes_down"]
            ms_u += st["ms_upload"]; ms_o += st["ms_offload"]; ms_c += st["ms_compute"]
        if args.flush_each_step:
            ctx.flush()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    out = {"model": args.model, "layers": L, "batch": args.batch, "seq": args.seq, "wire": args.wire, "compute": args.compute,
           "resident": plan["resident"], "n_slots": plan["n_slots"], "directions": q, "one_pass": one_pass, "writeback_interval": args.writeback_interval, "no_overlap": args.no_overlap, "flush_each_step": args.flush_each_step, "arena_bytes_used": plan["bytes_used"],
           "ms_per_step": dt * 1e3, "tokens_per_s": T / dt, "ms_per_block": dt * 1e3 / max(L, 1),
           "bucket_MB": bucket_bytes / 1e6,
           "upload_GBps": (up / 1e9) / (ms_u / 1e3) if ms_u else None,
           "offload_GBps": (down / 1e9) / (ms_o / 1e3) if ms_o else None,
           "link_GBps_over_step": (up / args.steps / 1e9) / dt if up else None,
           "compute_stream_ms": ms_c / args.steps, "last": [float(x) for x in res], "setup_s": setup_s}
    print(json.dumps(out), flush=True)
    ctx.close()


if __name__ == "__main__":
    main()
