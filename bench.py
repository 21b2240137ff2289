"""Benchmark of the ZO2 step on one MI355X.

A "step" is one whole zeroth-order iteration (Alg. 2): embedding, every decoder block's
fused update + perturb and dual forward, LM head + loss for both streams, g.  The workload is
the OPT-1.3B-shaped configuration: 24 layers, d 2048, 32 heads, FFN 8192, vocab 50272, bf16
weights fully resident in HBM, batch 16 x seq 256, Zipf(1.1) token ids, eps 1e-3, lr 1e-7.

Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MODEL, BATCH, SEQ = "opt-1.3b", 16, 256
EPS, LR, SEED0 = 1e-3, 1e-7, 42
PEAK_BF16_MFMA = 2500.0      # TFLOP/s, dense
PEAK_HBM = 8000.0            # GB/s
# HBM bytes per launch come from two rocprofv3 --pmc passes (FETCH_SIZE, WRITE_SIZE) over this same command, scaled by
# a 1 GiB copy through the same counters: `paper_2503_12668_amd/measure.py traffic` turns the profiler's CSVs into this
# file (with the commit it was measured at); it is read here, not measured live
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "hbm_traffic_opt1.3b_bf16_resident.json")


def measured_traffic():
    try:
        with open(TRAFFIC_JSON) as f:
            return json.load(f)
    except (OSError, ValueError):
        return None


def gemm_flops_per_step(cfg, T):
    """Dense projection flops of one step: both streams, every block, plus the LM head."""
    d, f, L, V = cfg["d_model"], cfg["d_ffn"], cfg["n_layers"], cfg["vocab"]
    per_forward = L * 2 * T * (4 * d * d + 2 * d * f) + 2 * T * V * d
    return 2 * per_forward


def k1_bytes_per_step(cfg, wire_bytes, comp_bytes):
    """Algorithmic HBM bytes of the fused update + perturb: read theta, write theta', W+, W-
    for every block parameter, the (tied) vocabulary matrix and the final LayerNorm."""
    d, f, L, V = cfg["d_model"], cfg["d_ffn"], cfg["n_layers"], cfg["vocab"]
    n = L * (4 * d * d + 2 * d * f + 9 * d + f) + V * d + 2 * d
    return n * (2 * wire_bytes + 2 * comp_bytes)


def cpu_baseline(cfg_full, T_batch, T_seq):
    """The oracle, as it stands, on a bounded sample of the same workload: the embedding + LM
    head alone (0 layers) and with three decoder blocks at the full width, vocabulary and
    batch, one step with a pending update each (about 12 s of CPU work); tokens/s extrapolated to the full depth."""
    import copy

    import torch

    import synth_inputs as si
    from oracle import opt_model, zo_step

    tok = si.make_tokens(cfg_full["vocab"], T_batch, T_seq, seed=2, dist="zipf")
    lab = si.next_token_labels(tok)
    times = {}
    kSampleBlocks = 3
    for nl in (0, kSampleBlocks):
        cfg = dict(cfg_full, n_layers=nl)
        P = si.make_weights(cfg, seed=1)
        oz = zo_step.Zo2Blockwise(opt_model.OptShape(**cfg), P)
        oz.pending = (1.0, SEED0 - 1, LR)          # as in steady state: an update is pending
        t0 = time.time()
        oz.step(tok, lab, SEED0, EPS, LR)
        times[nl] = time.time() - t0
    t_rest, t_block = times[0], max((times[kSampleBlocks] - times[0]) / kSampleBlocks, 1e-9)
    total = t_rest + cfg_full["n_layers"] * t_block
    return {"value": T_batch * T_seq / total, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"oracle step on embedding+LM head ({t_rest:.1f} s) and on {kSampleBlocks} of {cfg_full['n_layers']} decoder blocks "
                      f"({t_block:.1f} s each) at full width, vocabulary and batch {T_batch}x{T_seq}; extrapolated to "
                      f"{cfg_full['n_layers']} blocks ({total:.0f} s per step)"}


def _release(ctx):
    """Close a context and give its device arena and its pinned host buffers back (torch caches both)."""
    import gc

    import torch
    ctx.close()
    for name in ("h_buckets", "h_tok", "h_pos", "h_flnw", "h_flnb", "h_lm", "arena"):
        setattr(ctx, name, None)
    gc.collect()
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()


def budget_leg(model, layers, batch, seq, wire, compute, steps):
    """A streamed configuration under a fixed HBM budget of 18e9 bytes (everything the library touches: embeddings,
    block slots, W+ / W- scratch, activations): weights held on the host in the 8-bit transfer format (Sec. 5.5) and
    unpacked to bf16 on the device.  `layers`: None = the model's own depth; a number = that many blocks of the true
    shape (what fits the host memory this process may pin), reported per block."""
    import numpy as np
    import torch

    import synth_inputs as si
    from paper_2503_12668_amd import binding, run_config

    cfg = si.opt_config(model, n_layers=layers)
    L = cfg["n_layers"]
    scales = np.full(4 + 16 * L, 64.0, dtype=np.float32)
    ctx = binding.Zo2Context(cfg, run_config.gpu_weight_source(), wire=wire, compute=compute, arena_bytes=int(18e9), scales=scales)
    tok = si.make_tokens(cfg["vocab"], batch, seq, seed=2, dist="zipf")
    lab = si.next_token_labels(tok)
    ctx.step(tok, lab, 40, EPS, LR)
    ctx.step(tok, lab, 41, EPS, LR)
    plan = ctx.plan()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    up = 0
    for j in range(steps):
        ctx.step(tok, lab, 100 + j, EPS, LR)
        up += ctx.step_stats()["bytes_up"]
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    full = si.opt_config(model)["n_layers"]
    out = {"model": model, "layers_run": L, "layers_of_model": full, "batch": batch, "seq": seq, "wire": wire, "compute": compute,
           "budget_bytes": int(18e9), "arena_bytes_used": plan["bytes_used"], "resident": plan["resident"], "n_slots": plan["n_slots"],
           "sweeps_per_block": plan["sweeps_per_block"], "block_MB": ctx.offs[16] * binding.lib().zo2_dtype_size(ctx.wire_id) / 1e6,
           "ms_per_step": dt * 1e3, "ms_per_block": dt * 1e3 / L, "link_GBps_each_way_over_step": up / steps / dt / 1e9}
    if L == full:
        out["tokens_per_s"] = batch * seq / dt
    _release(ctx)
    return out


def offload_leg(steps=3, budget_legs=True):
    """The streamed mode on the driver's clock: OPT-13B shape (40 layers, d 5120, 40 heads, FFN 20480, bf16 weights in
    pinned host memory), blocks streamed through exactly 3 slots on three HIP streams (Alg. 3).  Batch 8 x seq 512 is
    the configuration as given (host-link bound on this machine); batch 32 x seq 512 is the point where a block's dual
    forward outlasts its copy, measured streamed and fully resident on the same context."""
    import torch

    import synth_inputs as si
    from paper_2503_12668_amd import binding, run_config

    cfg = si.opt_config("opt-13b")
    L = cfg["n_layers"]
    ctx = binding.Zo2Context(cfg, run_config.gpu_weight_source(), wire="bf16", compute="bf16", arena_bytes=36 << 30)
    bucket = ctx.offs[16] * 2

    def timed(batch, seq, slots, writeback_interval=1, dirs=1):
        tok = si.make_tokens(cfg["vocab"], batch, seq, seed=2, dist="zipf")
        lab = si.next_token_labels(tok)
        ctx.set_writeback_interval(writeback_interval)
        ctx.set_resident_budget(36 << 30)
        one = (lambda s0: ctx.step(tok, lab, s0, EPS, LR)) if dirs == 1 else \
              (lambda s0: ctx.step_multi(tok, lab, [s0 * 16 + k for k in range(dirs)], EPS, LR / dirs))   # a round of directions in one pass
        one(40)                                               # plans with everything resident: tells the bytes in use
        if slots:
            ctx.set_resident_budget(ctx.plan()["bytes_used"] - (L - slots) * bucket)
        one(41)
        plan = ctx.plan()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        up = down = 0
        ms_u = ms_o = 0.0
        for j in range(steps):
            one(100 + j)
            st = ctx.step_stats()
            up += st["bytes_up"]; down += st["bytes_down"]; ms_u += st["ms_upload"]; ms_o += st["ms_offload"]
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        return {"batch": batch, "seq": seq, "resident": plan["resident"], "n_slots": plan["n_slots"],
                "writeback_interval": writeback_interval, "directions_per_pass": dirs, "steps": steps, "ms_per_step": dt * 1e3,
                "tokens_per_s": batch * seq / dt, "forward_tokens_per_s": 2 * dirs * batch * seq / dt, "arena_bytes_used": plan["bytes_used"],
                "link_up_GBps_over_step": up / steps / dt / 1e9, "link_down_GBps_over_step": down / steps / dt / 1e9,
                "upload_stream_GBps": (up / 1e9) / (ms_u / 1e3) if ms_u else None,
                "offload_stream_GBps": (down / 1e9) / (ms_o / 1e3) if ms_o else None}

    res32 = timed(32, 512, None)
    str32 = timed(32, 512, 3)
    str8 = timed(8, 512, 3)
    # the host copies of the streamed blocks written back on every 8th update only (the updates they lack are replayed
    # from their seeds on upload; same results bit for bit): 8 steps, so that exactly one of them writes back
    steps, keep = 8, steps
    str8_wb8 = timed(8, 512, 3, writeback_interval=8)
    steps = keep
    # a round of two directions in one pass (zo2_step_multi): each block is uploaded once and runs four forwards
    str8_q2 = timed(8, 512, 3, dirs=2)
    _release(ctx)
    assert str8["n_slots"] == 3 and not str8["resident"] and str32["n_slots"] == 3 and res32["resident"], (str8, str32, res32)
    big = {}
    if budget_legs:
        big["opt30b_fp8_wire_18e9"] = budget_leg("opt-30b", None, 4, 1024, "fp8_e4m3", "bf16", steps)
        big["opt175b_fp8_wire_18e9"] = budget_leg("opt-175b", 12, 1, 2048, "fp8_e4m3", "bf16", steps)
    return {**big, "workload": f"opt-13b-shaped decoder ({L} layers, d {cfg['d_model']}, ffn {cfg['d_ffn']}), bf16 weights in pinned host "
                        f"memory ({bucket / 1e6:.0f} MB per block), streamed through 3 block slots on upload / compute / offload streams",
            "batch8_seq512_streamed": str8, "batch8_seq512_streamed_writeback_every_8": str8_wb8,
            "batch8_seq512_streamed_two_directions_one_pass": str8_q2, "batch32_seq512_streamed": str32, "batch32_seq512_resident": res32,
            "streamed_over_resident_at_32x512": str32["ms_per_step"] / res32["ms_per_step"], "steps": steps}


def small_steps_leg(ctx, cfg, steps=10):
    """Steps of few tokens on the benchmark's resident context: the perturbation written by the sweep kernel (as in the
    benchmark step) against generated in the projections' weight loader (what the library does by default up to 64
    tokens per stream).  ms per step, wall clock around `steps` steps each."""
    import torch

    import synth_inputs as si
    out = {"note": "same resident bf16 context; 'sweep_copies' = zo2_set_loader_fusion(-1), 'loader' = the default", "steps": steps}
    for (b, s_) in ((1, 16), (1, 64)):
        tok = si.make_tokens(cfg["vocab"], b, s_, seed=2, dist="zipf")
        lab = si.next_token_labels(tok)
        row = {}
        for name, mode in (("sweep_copies", -1), ("loader", 0)):
            ctx.set_loader_fusion(mode)
            for j in range(2):
                ctx.step(tok, lab, SEED0 + 500 + j, EPS, LR)
            row[name + "_active"] = ctx.plan()["loader_fusion"]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for j in range(steps):
                ctx.step(tok, lab, SEED0 + 510 + j, EPS, LR)
            torch.cuda.synchronize()
            row["ms_per_step_" + name] = (time.perf_counter() - t0) / steps * 1e3
        row["ratio"] = row["ms_per_step_sweep_copies"] / row["ms_per_step_loader"]
        out[f"{b}x{s_}"] = row
    ctx.set_loader_fusion(0)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-offload", action="store_true", help="skip the streamed (offload-mode) leg")
    ap.add_argument("--no-small-steps", action="store_true", help="skip the leg with steps of 16 and 64 tokens")
    ap.add_argument("--layers", type=int, default=None, help="debug: fewer layers (invalid as a benchmark number)")
    ap.add_argument("--gemm-wavefronts", type=int, default=0, choices=[0, 4, 8],
                    help="measurement aid: run every 256-row GEMM tile with this many wavefronts (0: chosen per launch, the library's default)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the ZO2 step is single-GPU; the design notes say how it "
              "would shard); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import synth_inputs as si
    from paper_2503_12668_amd import binding

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    binding.lib()
    binding.op_set_gemm_wavefronts(args.gemm_wavefronts)
    cfg = si.opt_config(MODEL, n_layers=args.layers)
    T = BATCH * SEQ
    t0 = time.time()
    P = si.make_weights(cfg, seed=1)
    tok = si.make_tokens(cfg["vocab"], BATCH, SEQ, seed=2, dist="zipf")
    lab = si.next_token_labels(tok)
    ctx = binding.Zo2Context(cfg, P, wire="bf16", compute="bf16", arena_bytes=20 << 30)
    del P
    print(f"[bench] setup {time.time() - t0:.1f} s", file=sys.stderr, flush=True)

    for j in range(args.warmup):
        ctx.step(tok, lab, SEED0 + j, EPS, LR)
    plan = ctx.plan()

    # timed region: exactly K steps, nothing else on the GPU
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for j in range(args.steps):
        ctx.step(tok, lab, SEED0 + args.warmup + j, EPS, LR)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / args.steps * 1e3

    # second pass over the same K steps with a pair of HIP events around every GEMM / K1 / attention launch on the
    # library's compute stream.  Kept out of the timed region: each event costs about 5 us of idle GPU between two
    # kernels (about 250 of them per step, +6 % step time), the kernels themselves run as in the timed region.
    ctx.set_profiling(("gemm", "k1", "attn"))
    acc = {k: [0.0, 0] for k in ctx.KERNEL_CLASSES}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for j in range(args.steps):
        ctx.step(tok, lab, SEED0 + args.warmup + args.steps + j, EPS, LR)
        for k, (ms, n) in ctx.kernel_times().items():
            acc[k][0] += ms
            acc[k][1] += n
    torch.cuda.synchronize()
    ms_step_profiled = (time.perf_counter() - t0) / args.steps * 1e3
    ctx.set_profiling(())

    gemm_ms, gemm_n = acc["gemm"]
    k1_ms, k1_n = acc["k1"]
    att_ms, att_n = acc["attn"]
    flops = gemm_flops_per_step(cfg, T) * args.steps
    tflops = flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    k1_bytes = k1_bytes_per_step(cfg, 2, 2) * args.steps
    k1_gbs = k1_bytes / (k1_ms * 1e-3) / 1e9 if k1_ms > 0 else 0.0
    traffic = measured_traffic()
    out = {
        "metric": "zo_step_tokens_per_s", "value": T / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{MODEL}-shaped decoder ({cfg['n_layers']} layers, d {cfg['d_model']}, {cfg['n_heads']} heads, "
                               f"ffn {cfg['d_ffn']}, vocab {cfg['vocab']}), bf16 weights resident in HBM, batch {BATCH} x seq {SEQ}, "
                               f"Zipf(1.1) tokens, eps {EPS}, lr {LR}",
                   "global_batch": BATCH, "seq_len": SEQ, "resident": plan["resident"], "arena_bytes_used": plan["bytes_used"],
                   **({"gemm_wavefronts_forced": args.gemm_wavefronts} if args.gemm_wavefronts else {})},
        "roofline": {"kernel": "gemm_mfma256_kernel (QKV / output / FFN / LM-head projections)", "bound": "mfma",
                     "achieved": tflops, "peak": PEAK_BF16_MFMA, "unit": "TFLOP/s", "frac": tflops / PEAK_BF16_MFMA,
                     "traffic": traffic["kernels"]["gemm"]["bytes_per_launch"] if (traffic and args.layers is None) else None,
                     "traffic_unit": "bytes per launch (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, calibrated, offline)",
                     "traffic_measured_at_commit": traffic["measured_at_commit"] if traffic else None,
                     "algorithmic_flops_per_launch": flops / gemm_n if gemm_n else None,
                     "launches_per_step": gemm_n / args.steps, "ms_per_step": gemm_ms / args.steps},
        "roofline_k1": {"kernel": "k1_kernel (fused regenerate + update + perturb)", "bound": "hbm", "achieved": k1_gbs,
                        "peak": PEAK_HBM, "unit": "GB/s", "frac": k1_gbs / PEAK_HBM,
                        "traffic": traffic["kernels"]["k1"]["bytes_per_launch"] if (traffic and args.layers is None) else None,
                        "traffic_unit": "bytes per launch (rocprofv3 --pmc, calibrated, offline)",
                        "algorithmic_bytes_per_launch": k1_bytes / k1_n if k1_n else None,
                        "launches_per_step": k1_n / args.steps, "ms_per_step": k1_ms / args.steps},
        "kernel_ms_per_step": {"gemm": gemm_ms / args.steps, "k1": k1_ms / args.steps, "attention": att_ms / args.steps,
                               "note": "from a second pass of the same number of steps with HIP events around every launch",
                               "ms_per_step_with_events": ms_step_profiled},
    }
    if not args.no_small_steps:
        out["small_steps"] = small_steps_leg(ctx, cfg)
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    if not args.no_offload and args.layers is None:
        out["offload"] = offload_leg()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, BATCH, SEQ)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
