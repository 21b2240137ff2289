"""The library's host code under UndefinedBehaviorSanitizer.

`build.py --host-sanitize` builds libzo2_hostsan.so: the same sources and device code, the host side instrumented
(signed overflow, shifts, misaligned or null accesses, array bounds), not recovering - the first finding aborts the
process.  Each test runs a child process that loads that library instead of libzo2.so, so a finding shows up as a
non-zero exit status with the sanitizer's report on stderr.  The planner, the offset tables and the workspace-size
calls are pure host arithmetic on sizes up to the OPT-175B shape (products beyond 2^31 elements), which is where such
findings would be; the GPU test drives the schedulers of all step variants through the instrumented host code and
compares the losses with those of the ordinary build.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PRELUDE = f"""
import sys
sys.path.insert(0, {ROOT!r})
from paper_2503_12668_amd import binding, build
if sys.argv[1] == "hostsan":
    binding.LIB_PATH = build.LIB_HOSTSAN
"""


def _hostsan_lib():
    sys.path.insert(0, ROOT)
    from paper_2503_12668_amd import build
    if not os.path.exists(build.LIB_HOSTSAN) or os.path.getmtime(build.LIB_HOSTSAN) < os.path.getmtime(build.LIB):
        if os.environ.get("GRAFT_REPO_ROOT"):        # on a GPU machine nothing is built: the library travels with the tree
            pytest.skip("libzo2_hostsan.so not in the tree (python paper_2503_12668_amd/build.py --host-sanitize)")
        build.build(verbose=False)
        build.build_host_sanitized(verbose=False)
    return build.LIB_HOSTSAN


def _run(code, which, timeout=600):
    p = subprocess.run([sys.executable, "-c", PRELUDE + code, which], capture_output=True, text=True, timeout=timeout, cwd=ROOT)
    assert "runtime error" not in p.stderr, p.stderr[-4000:]
    assert p.returncode == 0, (p.returncode, p.stderr[-4000:])
    return p.stdout


HOST_ONLY = """
import ctypes as C
L = binding.lib()
import synth_inputs as si
out = []
for name in ("opt-125m", "opt-1.3b", "opt-13b", "opt-30b", "opt-66b", "opt-175b"):
    cfg = si.opt_config(name)
    for wire, comp in (("f32", "f32"), ("bf16", "bf16"), ("fp8_e4m3", "bf16")):
        zc = binding.make_config(cfg, wire, comp)
        offs = (C.c_int64 * 17)()
        assert L.zo2_block_tensor_offsets(C.byref(zc), offs) == 0
        out.append(int(offs[16]))
for dt in range(-1, 8):
    out.append(int(L.zo2_dtype_size(dt)))
for (M, N, K) in ((1, 64, 64), (128, 49152, 12288), (256, 12288, 49152), (16, 50272, 12288), (0, 0, 0), (256, 2**30, 2**20)):
    out.append(int(L.zo2_op_gemm_perturbed_workspace_bytes(M, N, K)))
for (M, N) in ((1, 4), (4096, 50272), (2659, 50272), (2**20, 2**20), (0, 0)):
    out.append(int(L.zo2_op_lm_head_ce_workspace_bytes(M, N)))
print(out)
"""


def test_host_arithmetic_under_the_sanitizer_up_to_the_175b_shape():
    _hostsan_lib()
    a = _run(HOST_ONLY, "hostsan")
    b = _run(HOST_ONLY, "plain")
    assert a == b and len(a) > 20


GPU_STEPS = """
import numpy as np
import synth_inputs as si
cfg = si.tiny_config(n_layers=5, d_model=64, n_heads=4, d_ffn=128, vocab=211, max_pos=64)
out = []
for wire, comp in (("f32", "f32"), ("bf16", "bf16"), ("fp8_e4m3", "bf16")):
    P = si.make_weights(cfg, seed=11, std=0.08, ln_jitter=True)
    ctx = binding.Zo2Context(cfg, P, wire=wire, compute=comp, arena_bytes=64 << 20)
    tok = si.make_tokens(cfg["vocab"], 2, 19, seed=12)
    lab = si.next_token_labels(tok)
    r = [ctx.step(tok, lab, 1, 1e-3, 1e-3)]
    full = ctx.plan()["bytes_used"]
    ctx.set_resident_budget(full - 2 * ctx.offs[16] * binding.lib().zo2_dtype_size(ctx.wire_id))      # streamed through 3 slots
    r.append(ctx.step(tok, lab, 2, 1e-3, 1e-3))
    r.append(ctx.step_extra(tok, lab, 3, 1e-3, 5e-4))
    r.append(ctx.step(tok, lab, 4, 1e-3, 1e-3))
    ev = ctx.eval(tok, lab)
    for sweeps in (2, 4, 0):
        ctx.set_scratch_plan(sweeps)
        r.append(ctx.step(tok, lab, 5 + sweeps, 1e-3, 1e-3))
    ctx.set_writeback_interval(3)
    for j in range(4):
        r.append(ctx.step(tok, lab, 12 + j, 1e-3, 1e-3))
    r.append(ctx.step_extra(tok, lab, 16, 1e-3, 5e-4))
    r += ctx.step_multi(tok, lab, [17, 18, 19], 1e-3, 3e-4)
    ctx.set_loader_fusion(-1)
    r.append(ctx.step(tok, lab, 20, 1e-3, 1e-3))
    r += ctx.step_multi(tok, lab, [22, 23], 1e-3, 3e-4)
    ctx.set_writeback_interval(1)
    ctx.set_loader_fusion(0)
    ctx.set_resident_budget(full)
    r.append(ctx.step(tok, lab, 21, 1e-3, 1e-3))
    pl = ctx.plan()
    ctx.flush(); ctx.sync_to_host()
    out.append([[float(v) for v in x] for x in r] + [float(ev), pl["n_slots"], pl["resident"]])
    ctx.close()
print(out)
"""


@pytest.mark.gpu
def test_all_step_variants_run_clean_under_the_host_sanitizer_and_give_the_same_losses():
    _hostsan_lib()
    a = _run(GPU_STEPS, "hostsan")
    b = _run(GPU_STEPS, "plain")
    assert a == b, (a, b)
