"""Build libzo2.so (HIP, gfx950) in-tree with hipcc.  Cross-compiles without a GPU."""
import glob
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libzo2.so")
LIB_STAMPS = os.path.join(HERE, "libzo2_stamps.so")       # the large-tile GEMM with cycle stamps compiled in (measure.py gemm-phases)
LIB_HOSTSAN = os.path.join(HERE, "libzo2_hostsan.so")     # same device code, host code under UndefinedBehaviorSanitizer (a test aid)

HIPCC_FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wno-unused-command-line-argument", "-Wno-unused-value", "-Wno-unused-result",
               # keep the compiler from forming packed-fp32 instructions
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _needs_build(obj, src, deps):
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(p) > t for p in [src] + deps)


# csrc/gemm256.hip issues its MFMAs from inline assembly (to pin the accumulators to accumulation registers), so the
# compiler neither knows that they are MFMAs nor inserts the wait states an MFMA result needs before another kind of
# instruction may touch it.  The kernel keeps that distance itself; this scan of the generated assembly fails the build
# if a compiler-generated access to an accumulation register ever lands closer than kMfmaDistance instructions behind
# an MFMA (each instruction is at least one wait state; s_nop N counts N + 1).
kMfmaDistance = 20
_ACC_REG = re.compile(r"\ba(\d+|\[\d+:\d+\])")


def scan_mfma_hazards(asm_text):
    """Returns a list of (kernel, line number, instruction, distance) for every accumulation-register access that
    follows an MFMA too closely in program order."""
    bad, kernel, dist = [], None, 10 ** 9
    for n, line in enumerate(asm_text.splitlines(), 1):
        m = re.match(r"^(_Z\w+):", line)
        if m:
            kernel, dist = m.group(1), 10 ** 9
            continue
        ins = line.split(";")[0].strip()
        if not ins or ins.startswith(".") or ins.endswith(":"):
            continue
        op = ins.split()[0]
        if op.startswith("v_mfma"):
            dist = 0
            continue
        if op == "s_nop":
            dist += int(ins.split()[1], 0) + 1
            continue
        if dist < kMfmaDistance and ("accvgpr" in op or _ACC_REG.search(ins)):
            bad.append((kernel, n, ins, dist))
        dist += 1
    return bad


def _check_gemm256(hipcc, src, bdir, verbose):
    asm = os.path.join(bdir, "gemm256.s")
    cmd = [hipcc] + [f for f in HIPCC_FLAGS if f != "-fPIC"] + ["--offload-device-only", "-S", src, "-o", asm]
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    with open(asm) as f:
        text = f.read()
    if "v_mfma" not in text:
        raise RuntimeError("gemm256: no MFMA in the generated assembly - the hazard scan is looking at the wrong file")
    bad = scan_mfma_hazards(text)
    if bad:
        head = "\n".join("  %s line %d: %s (%d behind an MFMA)" % b for b in bad[:8])
        raise RuntimeError("gemm256: %d accumulation-register accesses too close behind an inline-assembly MFMA:\n%s" % (len(bad), head))
    if verbose:
        print("[build] gemm256 MFMA hazard scan: clean", flush=True)


def build(force=False, verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    deps = sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(HERE, "..", "include", "zo2.h")]
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs, procs = [], []
    for s in srcs:
        o = os.path.join(bdir, os.path.basename(s) + ".o")
        objs.append(o)
        if force or _needs_build(o, s, deps):
            cmd = [hipcc] + HIPCC_FLAGS + ["-c", s, "-o", o]
            if verbose:
                print("[build]", " ".join(cmd), flush=True)
            procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    ok = True
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            ok = False
            print(f"[build] FAILED {s}\n{out}", file=sys.stderr)
        elif out.strip() and verbose:
            print(out)
    if not ok:
        raise RuntimeError("hipcc failed")
    g256 = os.path.join(CSRC, "gemm256.hip")
    if any(src == g256 for src, _ in procs):
        _check_gemm256(hipcc, g256, bdir, verbose)
    if force or procs or not os.path.exists(LIB):
        cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
        if verbose:
            print("[build]", " ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return LIB


def build_gemm_stamps(verbose=True):
    """libzo2_stamps.so: the library with -DZO2_GEMM_STAMPS in the two sources that know the macro (the large-tile GEMM
    records one workgroup's shader clock around the phases of its tiles; zo2_op_gemm_phases hands the buffer in).  A
    measurement aid for `measure.py gemm-phases`; nothing else loads it."""
    build(verbose=verbose)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    bdir = os.path.join(HERE, "_build", "stamps")
    os.makedirs(bdir, exist_ok=True)
    objs = []
    for s in sorted(glob.glob(os.path.join(CSRC, "*.hip"))):
        name = os.path.basename(s)
        if name in ("gemm256.hip", "zo2_lib.hip"):
            o = os.path.join(bdir, name + ".o")
            cmd = [hipcc] + HIPCC_FLAGS + ["-DZO2_GEMM_STAMPS", "-c", s, "-o", o]
            if verbose:
                print("[build]", " ".join(cmd), flush=True)
            subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
        else:
            o = os.path.join(HERE, "_build", name + ".o")
        objs.append(o)
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB_STAMPS] + objs
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB_STAMPS


def build_host_sanitized(verbose=True):
    """libzo2_hostsan.so: the same sources and device code, the host side compiled with -fsanitize=undefined (and bounds),
    not recovering: the first finding ends the process.  A test aid (tests/test_host_sanitizer.py loads it in a child
    process); device code cannot be sanitized on the test machines, host code can."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    rt = sorted(glob.glob("/opt/rocm*/lib/llvm/lib/clang/*/lib/linux/libclang_rt.ubsan_standalone-x86_64.so"))
    if not rt:
        raise RuntimeError("no shared UndefinedBehaviorSanitizer runtime under /opt/rocm*/lib/llvm")
    rt_dir = os.path.dirname(os.path.realpath(rt[-1]))
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    bdir = os.path.join(HERE, "_build", "hostsan")
    os.makedirs(bdir, exist_ok=True)
    # (without the indirect-call check: under -fsanitize=function a kernel launched through a function-pointer variable,
    # as the two kernels with dynamic LDS are, is pushed but never launched by this toolchain's host stub)
    san = ["-g1", "-Xarch_host", "-fsanitize=undefined,bounds", "-Xarch_host", "-fno-sanitize=function",
           "-Xarch_host", "-fno-sanitize-recover=undefined,bounds"]
    objs, procs = [], []
    for s in srcs:
        o = os.path.join(bdir, os.path.basename(s) + ".o")
        objs.append(o)
        cmd = [hipcc] + HIPCC_FLAGS + san + ["-c", s, "-o", o]
        if verbose:
            print("[build]", " ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for s, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {s}\n{out}")
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-fsanitize=undefined", "-shared-libsan", "-Wno-option-ignored",
           "-Wl,-rpath," + rt_dir, "-o", LIB_HOSTSAN] + objs
    if verbose:
        print("[build]", " ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB_HOSTSAN


if __name__ == "__main__":
    build(force="--force" in sys.argv)
    if "--host-sanitize" in sys.argv:
        build_host_sanitized()
    if "--gemm-stamps" in sys.argv:
        build_gemm_stamps()
