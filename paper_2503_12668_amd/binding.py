"""ctypes binding of libzo2 (argument marshalling only).

torch is used for device / pinned memory and stream handles; every step of the
zeroth-order iteration runs inside the library's HIP kernels.
"""
import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libzo2.so")

F32, BF16, F16, FP8_E4M3, FP8_E5M2 = 0, 1, 2, 3, 4
DTYPE_ID = {"f32": F32, "bf16": BF16, "f16": F16, "fp8_e4m3": FP8_E4M3, "fp8_e5m2": FP8_E5M2}
TORCH_DTYPE = {F32: torch.float32, BF16: torch.bfloat16, F16: torch.float16,
               FP8_E4M3: torch.float8_e4m3fn, FP8_E5M2: torch.float8_e5m2}
STATUS = {0: "ZO2_OK", 1: "ZO2_EINVAL", 2: "ZO2_ENOMEM", 3: "ZO2_EBUDGET", 4: "ZO2_EHIP", 5: "ZO2_ESTATE",
          6: "ZO2_ENONFINITE"}
BLOCK_TENSORS = ("ln1.w", "ln1.b", "q.w", "q.b", "k.w", "k.b", "v.w", "v.b",
                 "o.w", "o.b", "ln2.w", "ln2.b", "fc1.w", "fc1.b", "fc2.w", "fc2.b")


class Zo2Error(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


class Config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("max_pos", C.c_int32), ("pos_offset", C.c_int32), ("tied_lm_head", C.c_int32),
                ("wire_dtype", C.c_int32), ("compute_dtype", C.c_int32), ("ln_eps", C.c_float)]


class HostWeights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("pos_emb", C.c_void_p), ("final_ln_w", C.c_void_p), ("final_ln_b", C.c_void_p),
                ("lm_head", C.c_void_p), ("block_bucket", C.POINTER(C.c_void_p)), ("tensor_scale", C.POINTER(C.c_float))]


class Device(C.Structure):
    _fields_ = [("arena", C.c_void_p), ("arena_bytes", C.c_size_t), ("stream_compute", C.c_void_p),
                ("stream_upload", C.c_void_p), ("stream_offload", C.c_void_p), ("stream_k1", C.c_void_p)]


_lib = None


def lib():
    """Load libzo2.so; raises if it has not been built (python -m paper_2503_12668_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_2503_12668_amd/build.py` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, u32, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64, C.c_float
    sigs = {
        "zo2_block_tensor_offsets": (i32, [C.POINTER(Config), C.POINTER(i64)]),
        "zo2_dtype_size": (C.c_size_t, [i32]),
        "zo2_init": (i32, [C.POINTER(vp), C.POINTER(Config), C.POINTER(HostWeights), C.POINTER(Device)]),
        "zo2_set_resident_budget": (i32, [vp, C.c_size_t]),
        "zo2_step": (i32, [vp, vp, vp, i32, i32, u64, f32, f32, C.POINTER(f32), C.POINTER(f32), C.POINTER(f32)]),
        "zo2_step_extra": (i32, [vp, vp, vp, i32, i32, u64, f32, f32, C.POINTER(f32), C.POINTER(f32), C.POINTER(f32)]),
        "zo2_step_multi": (i32, [vp, vp, vp, i32, i32, i32, vp, f32, f32, vp]),
        "zo2_flush": (i32, [vp]),
        "zo2_eval": (i32, [vp, vp, vp, i32, i32, C.POINTER(f32)]),
        "zo2_get_pending": (i32, [vp, C.POINTER(i32), C.POINTER(u64), C.POINTER(f32)]),
        "zo2_set_pending": (i32, [vp, i32, u64, f32]),
        "zo2_pending_count": (i32, [vp, C.POINTER(i32)]),
        "zo2_get_pending_at": (i32, [vp, i32, C.POINTER(u64), C.POINTER(f32)]),
        "zo2_add_pending": (i32, [vp, u64, f32]),
        "zo2_sync_to_host": (i32, [vp]),
        "zo2_get_plan": (i32, [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_size_t)]),
        "zo2_get_scratch_plan": (i32, [vp, C.POINTER(i32), C.POINTER(i64), C.POINTER(i32)]),
        "zo2_set_scratch_plan": (i32, [vp, i32]),
        "zo2_set_loader_fusion": (i32, [vp, i32]),
        "zo2_get_loader_fusion": (i32, [vp, C.POINTER(i32)]),
        "zo2_set_split_k": (i32, [vp, i32]),
        "zo2_set_writeback_interval": (i32, [vp, i32]),
        "zo2_get_writeback_state": (i32, [vp, C.POINTER(i32), C.POINTER(i32)]),
        "zo2_get_step_stats": (i32, [vp, C.POINTER(f32), C.POINTER(f32), C.POINTER(f32), C.POINTER(u64), C.POINTER(u64)]),
        "zo2_set_profiling": (i32, [vp, u32]),
        "zo2_set_stream_overlap": (i32, [vp, i32]),
        "zo2_set_wire_rounding": (i32, [vp, i32]),
        "zo2_get_kernel_times": (i32, [vp, C.POINTER(f32), C.POINTER(i32)]),
        "zo2_debug_set_stream_delay": (i32, [vp, i32, u32]),
        "zo2_debug_set_slot_poison": (i32, [vp, i32]),
        "zo2_last_error": (C.c_char_p, [vp]),
        "zo2_destroy": (None, [vp]),
        "zo2_op_last_error": (C.c_char_p, []),
        "zo2_op_philox_words": (i32, [u64, u32, u64, u64, vp, vp]),
        "zo2_op_gaussian": (i32, [u64, u32, u64, u64, vp, vp]),
        "zo2_op_update_perturb": (i32, [vp, i32, vp, vp, i32, u32, u64, u64, i32, u64, f32, u64, f32, f32, i32, vp]),
        "zo2_op_update_perturb_block": (i32, [C.POINTER(Config), i32, vp, vp, vp, i32, u64, f32, u64, f32, C.POINTER(f32), i32, vp]),
        "zo2_op_convert": (i32, [vp, i32, f32, vp, i32, f32, u64, vp]),
        "zo2_op_gemm": (i32, [i32, i32, i32, i32, vp, i64, vp, i64, vp, vp, vp, i32, i64, f32, i32, vp]),
        "zo2_op_gemm_split_k": (i32, [i32, i32, i32, i32, vp, i64, vp, i64, vp, vp, vp, i32, i64, f32, i32, i32, vp, C.c_size_t, vp]),
        "zo2_op_gemm_split_k_workspace_bytes": (C.c_size_t, [i32, i32, i32]),
        "zo2_op_gemm_split_k_pieces": (i32, [i32, i32, i32, i32, i32]),
        "zo2_op_set_gemm_tile_rows": (i32, [i32]),
        "zo2_op_set_gemm_wavefronts": (i32, [i32]),
        "zo2_op_gemm_phases": (i32, [i32, i32, i32, i32, vp, i64, vp, i64, vp, vp, i32, i64, vp, vp]),
        "zo2_op_gemm_perturbed": (i32, [i32, i32, i32, i32, vp, vp, i64, vp, u32, u64, f32, vp, vp, vp, vp, vp, vp, i32, i64, f32, i32, vp, C.c_size_t, vp]),
        "zo2_op_gemm_perturbed_workspace_bytes": (C.c_size_t, [i32, i32, i32]),
        "zo2_op_perturbed_rows": (i32, [i32, vp, i64, i64, i64, u32, u64, f32, vp, vp, vp]),
        "zo2_op_attention": (i32, [i32, vp, vp, vp, vp, i32, i32, i32, i32, i64, i32, vp]),
        "zo2_op_layernorm": (i32, [i32, vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, vp]),
        "zo2_op_cross_entropy_rows": (i32, [vp, i64, vp, i32, i32, vp, vp]),
        "zo2_op_lm_head_ce": (i32, [i32, i32, i32, i32, vp, i64, vp, i64, vp, vp, vp, C.c_size_t, vp]),
        "zo2_op_lm_head_ce_workspace_bytes": (C.c_size_t, [i32, i32]),
        "zo2_op_lm_head_ce_static": (i32, [i32, i32, i32, i32, vp, i64, vp, i64, vp, vp, vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


EXPORTED = ["zo2_block_tensor_offsets", "zo2_dtype_size", "zo2_init", "zo2_set_resident_budget", "zo2_step", "zo2_step_extra", "zo2_step_multi", "zo2_flush", "zo2_eval", "zo2_get_pending", "zo2_set_pending",
            "zo2_pending_count", "zo2_get_pending_at", "zo2_add_pending",
            "zo2_sync_to_host", "zo2_get_plan", "zo2_get_scratch_plan", "zo2_set_scratch_plan", "zo2_set_loader_fusion", "zo2_get_loader_fusion", "zo2_set_split_k", "zo2_set_writeback_interval", "zo2_get_writeback_state", "zo2_get_step_stats", "zo2_set_profiling", "zo2_set_stream_overlap", "zo2_set_wire_rounding", "zo2_get_kernel_times", "zo2_debug_set_stream_delay", "zo2_debug_set_slot_poison", "zo2_last_error", "zo2_destroy", "zo2_op_last_error",
            "zo2_op_philox_words", "zo2_op_gaussian", "zo2_op_update_perturb", "zo2_op_update_perturb_block", "zo2_op_convert", "zo2_op_gemm", "zo2_op_gemm_split_k", "zo2_op_gemm_split_k_workspace_bytes", "zo2_op_gemm_split_k_pieces", "zo2_op_set_gemm_tile_rows", "zo2_op_set_gemm_wavefronts", "zo2_op_gemm_phases", "zo2_op_gemm_perturbed", "zo2_op_gemm_perturbed_workspace_bytes", "zo2_op_perturbed_rows",
            "zo2_op_attention", "zo2_op_layernorm", "zo2_op_cross_entropy_rows", "zo2_op_lm_head_ce",
            "zo2_op_lm_head_ce_workspace_bytes", "zo2_op_lm_head_ce_static"]


def _op_check(st):
    if st != 0:
        raise Zo2Error(st, lib().zo2_op_last_error().decode())


def _stream_ptr(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _dt(t):
    for k, v in TORCH_DTYPE.items():
        if v == t.dtype:
            return k
    raise TypeError(t.dtype)


def make_config(cfg, wire="f32", compute="f32"):
    return Config(cfg["n_layers"], cfg["d_model"], cfg["n_heads"], cfg["d_ffn"], cfg["vocab"], cfg["max_pos"],
                  cfg["pos_offset"], 1 if cfg["tied"] else 0, DTYPE_ID[wire], DTYPE_ID[compute], cfg.get("ln_eps", 1e-5))


def block_tensor_offsets(ccfg):
    offs = (C.c_int64 * 17)()
    _op_check(lib().zo2_block_tensor_offsets(C.byref(ccfg), offs))
    return list(offs)


def block_tensor_shape(cfg, t):
    d, f = cfg["d_model"], cfg["d_ffn"]
    return {"q.w": (d, d), "k.w": (d, d), "v.w": (d, d), "o.w": (d, d), "fc1.w": (f, d), "fc2.w": (d, f),
            "fc1.b": (f,)}.get(t, (d,))


# ------------------------------------------------------------------------------------------------
# kernel-level wrappers (torch device tensors in, enqueue on the current stream)
# ------------------------------------------------------------------------------------------------
def op_philox_words(seed, tensor_id, e0, n, stream=None):
    out = torch.empty(n, dtype=torch.int32, device="cuda")
    _op_check(lib().zo2_op_philox_words(seed, tensor_id, e0, n, _ptr(out), _stream_ptr(stream)))
    return out


def op_gaussian(seed, tensor_id, e0, n, stream=None):
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    _op_check(lib().zo2_op_gaussian(seed, tensor_id, e0, n, _ptr(out), _stream_ptr(stream)))
    return out


def op_update_perturb(theta, w_plus, w_minus, tensor_id, e0, has_pending, seed_prev, c, seed, eps, scale=1.0,
                      compute_dtype=None, n=None, stochastic=False, stream=None):
    """theta: device tensor in wire dtype (rewritten in place); w_plus / w_minus: device tensors or None."""
    n = theta.numel() if n is None else n
    cdt = _dt(w_plus) if w_plus is not None else (compute_dtype if compute_dtype is not None else F32)
    _op_check(lib().zo2_op_update_perturb(_ptr(theta), _dt(theta), _ptr(w_plus), _ptr(w_minus), cdt, tensor_id, e0, n,
                                          1 if has_pending else 0, seed_prev, c, seed, eps, scale, 1 if stochastic else 0,
                                          _stream_ptr(stream)))


def op_update_perturb_block(ccfg, layer, bucket, w_plus, w_minus, has_pending, seed_prev, c, seed, eps, scales=None,
                            stochastic=False, stream=None):
    """All 16 tensors of one block bucket in one launch (bucket: device tensor in the wire dtype, rewritten in place)."""
    sc = None
    if scales is not None:
        sc = (C.c_float * 16)(*[float(x) for x in scales])
    _op_check(lib().zo2_op_update_perturb_block(C.byref(ccfg), layer, _ptr(bucket), _ptr(w_plus), _ptr(w_minus),
                                                1 if has_pending else 0, seed_prev, c, seed, eps, sc, 1 if stochastic else 0,
                                                _stream_ptr(stream)))


def op_convert(src, dst, src_scale=1.0, dst_scale=1.0, stream=None):
    assert src.numel() == dst.numel()
    _op_check(lib().zo2_op_convert(_ptr(src), _dt(src), src_scale, _ptr(dst), _dt(dst), dst_scale, src.numel(),
                                   _stream_ptr(stream)))


def op_gemm(X, W, bias=None, residual=None, out_dtype=None, out_scale=1.0, relu=False, Y=None, stream=None):
    M, K = X.shape
    N = W.shape[0]
    odt = _dt(X) if out_dtype is None else out_dtype
    if Y is None:
        Y = torch.empty(M, N, dtype=TORCH_DTYPE[odt], device="cuda")
    _op_check(lib().zo2_op_gemm(_dt(X), M, N, K, _ptr(X), X.stride(0), _ptr(W), W.stride(0), _ptr(bias), _ptr(residual),
                                _ptr(Y), odt, Y.stride(0), out_scale, 1 if relu else 0, _stream_ptr(stream)))
    return Y


def op_gemm_split_k(X, W, splits, bias=None, residual=None, out_dtype=None, out_scale=1.0, relu=False, stream=None):
    M, K = X.shape
    N = W.shape[0]
    odt = _dt(X) if out_dtype is None else out_dtype
    Y = torch.empty(M, N, dtype=TORCH_DTYPE[odt], device="cuda")
    nbytes = lib().zo2_op_gemm_split_k_workspace_bytes(M, N, splits)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    _op_check(lib().zo2_op_gemm_split_k(_dt(X), M, N, K, _ptr(X), X.stride(0), _ptr(W), W.stride(0), _ptr(bias), _ptr(residual),
                                        _ptr(Y), odt, Y.stride(0), out_scale, 1 if relu else 0, splits, _ptr(ws), nbytes, _stream_ptr(stream)))
    return Y


def op_gemm_split_k_pieces(dtype_id, M, N, K, nprob):
    return int(lib().zo2_op_gemm_split_k_pieces(dtype_id, M, N, K, nprob))


def op_gemm_perturbed(Xp, Xm, theta, tensor_id, seed, eps, bias_p=None, bias_m=None, res_p=None, res_m=None, out_dtype=None,
                      out_scale=1.0, relu=False, stream=None):
    """Both streams' projection with W+- generated in the weight loader; returns (Y+, Y-)."""
    M, K = Xp.shape
    N = theta.shape[0]
    odt = _dt(Xp) if out_dtype is None else out_dtype
    Yp = torch.empty(M, N, dtype=TORCH_DTYPE[odt], device="cuda")
    Ym = torch.empty(M, N, dtype=TORCH_DTYPE[odt], device="cuda")
    nb = lib().zo2_op_gemm_perturbed_workspace_bytes(M, N, K)
    ws = torch.empty(max(nb, 16), dtype=torch.uint8, device="cuda")
    _op_check(lib().zo2_op_gemm_perturbed(_dt(Xp), M, N, K, _ptr(Xp), _ptr(Xm), Xp.stride(0), _ptr(theta), tensor_id, seed, eps,
                                          _ptr(bias_p), _ptr(bias_m), _ptr(res_p), _ptr(res_m), _ptr(Yp), _ptr(Ym), odt, Yp.stride(0),
                                          out_scale, 1 if relu else 0, _ptr(ws), nb, _stream_ptr(stream)))
    return Yp, Ym


def op_perturbed_rows(theta_rows, K, n0, tensor_id, seed, eps, stream=None):
    """W+ and W- of rows n0 .. of a dense [N, K] tensor (theta_rows: those rows) through the loader's code path."""
    wp, wm = torch.empty_like(theta_rows), torch.empty_like(theta_rows)
    _op_check(lib().zo2_op_perturbed_rows(_dt(theta_rows), _ptr(theta_rows), K, n0, theta_rows.numel() // K, tensor_id, seed, eps,
                                          _ptr(wp), _ptr(wm), _stream_ptr(stream)))
    return wp, wm


def op_set_gemm_tile_rows(rows):
    """0: the GEMM picks 128- or 256-row tiles per launch; 128 / 256: forced (tests, measurements)."""
    _op_check(lib().zo2_op_set_gemm_tile_rows(int(rows)))


def op_set_gemm_wavefronts(waves):
    """0: 256-row tiles run with 4 or 8 wavefronts as the length of k suggests; 4 / 8: forced (tests, measurements)."""
    _op_check(lib().zo2_op_set_gemm_wavefronts(int(waves)))


def op_gemm_phases(X, W, Y, stamps, residual=None, stream=None):
    """The large-tile GEMM with one workgroup's cycle stamps (instrumented build only; see zo2_op_gemm_phases)."""
    M, K = X.shape
    N = W.shape[0]
    _op_check(lib().zo2_op_gemm_phases(_dt(X), M, N, K, _ptr(X), X.stride(0), _ptr(W), W.stride(0), _ptr(residual) if residual is not None else None,
                                       _ptr(Y), _dt(Y), Y.stride(0), _ptr(stamps), _stream_ptr(stream)))


def op_attention(q, k, v, n_seq, seq, n_heads, d_head, vector_kernel=False, stream=None):
    out = torch.empty_like(q)
    _op_check(lib().zo2_op_attention(_dt(q), _ptr(q), _ptr(k), _ptr(v), _ptr(out), n_seq, seq, n_heads, d_head,
                                     q.stride(0), 1 if vector_kernel else 0, _stream_ptr(stream)))
    return out


def op_layernorm(x, w, b, eps=1e-5, w2=None, b2=None, rows_first=None, stream=None):
    rows, d = x.shape
    y = torch.empty(rows, d, dtype=w.dtype, device="cuda")
    rf = rows if rows_first is None else rows_first
    _op_check(lib().zo2_op_layernorm(_dt(w), _ptr(x), _ptr(w), _ptr(b), _ptr(w2), _ptr(b2), _ptr(y), rows, rf, d, eps,
                                     _stream_ptr(stream)))
    return y


def op_cross_entropy_rows(logits, labels, vocab=None, stream=None):
    rows = logits.shape[0]
    vocab = logits.shape[1] if vocab is None else vocab
    out = torch.empty(rows, dtype=torch.float32, device="cuda")
    _op_check(lib().zo2_op_cross_entropy_rows(_ptr(logits), logits.stride(0), _ptr(labels), rows, vocab, _ptr(out),
                                              _stream_ptr(stream)))
    return out


def op_lm_head_ce(X, W, labels, stream=None):
    M, K = X.shape
    N = W.shape[0]
    nb = lib().zo2_op_lm_head_ce_workspace_bytes(M, N)
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device="cuda")
    out = torch.empty(M, dtype=torch.float32, device="cuda")
    _op_check(lib().zo2_op_lm_head_ce(_dt(X), M, N, K, _ptr(X), X.stride(0), _ptr(W), W.stride(0), _ptr(labels), _ptr(out),
                                      _ptr(ws), nb, _stream_ptr(stream)))
    return out


def op_lm_head_ce_static(X, W, labels, out=None, stream=None):
    """op_lm_head_ce without a workspace: the library's built-in scratch buffer is used; nothing is allocated by the
    call itself (pass `out` to keep the binding from allocating the result either)."""
    M, K = X.shape
    N = W.shape[0]
    if out is None:
        out = torch.empty(M, dtype=torch.float32, device="cuda")
    _op_check(lib().zo2_op_lm_head_ce_static(_dt(X), M, N, K, _ptr(X), X.stride(0), _ptr(W), W.stride(0), _ptr(labels),
                                             _ptr(out), _stream_ptr(stream)))
    return out


# ------------------------------------------------------------------------------------------------
# training context
# ------------------------------------------------------------------------------------------------
def _to_wire(a, wire_id, scale=1.0):
    """float32 numpy / torch tensor -> flat torch CPU tensor in the wire dtype, packed by the library's own
    conversion kernel (zo2_op_convert: round to nearest even, 8-bit formats saturating, stored = theta * scale)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)) if isinstance(a, np.ndarray) else a
    t = t.to(device="cuda", dtype=torch.float32).contiguous().reshape(-1)
    if wire_id == F32:
        return t.cpu()
    dst = torch.empty(t.numel(), dtype=TORCH_DTYPE[wire_id], device="cuda")
    op_convert(t, dst, 1.0, float(scale))
    return dst.cpu()


def _from_wire(t, scale=1.0):
    """flat torch CPU tensor in a wire dtype -> float32 CPU tensor, unpacked by the library (theta = stored / scale)."""
    if t.dtype == torch.float32:
        return t.clone()
    src = t.to("cuda")
    dst = torch.empty(src.numel(), dtype=torch.float32, device="cuda")
    op_convert(src, dst, float(scale), 1.0)
    return dst.cpu()


class Zo2Context:
    """Host buffers + arena + streams + the library context for one model.

    weights: name -> float32 array ("tok_emb", "pos_emb", "blocks.{l}.{t}", "final_ln.w", "final_ln.b"[, "lm_head.w"]),
    or a callable (name, shape) -> float32 torch tensor on any device (for models too large to build as a dict).
    They are converted once to the wire dtype and packed into per-block host buckets (pinned when possible);
    from then on the library owns their contents.
    overlap_k1: hand the library a fourth stream so that the update + perturb pass of block l+1 runs concurrently
    with the forwards of block l (off by default: on MI355X the cross-stream waits cost more than the overlap wins)."""

    def __init__(self, cfg, weights, wire="f32", compute="f32", arena_bytes=None, budget_bytes=None, scales=None,
                 pin=True, overlap_k1=False):
        self.cfg = dict(cfg)
        self.ccfg = make_config(cfg, wire, compute)
        self.wire_id, self.compute_id = DTYPE_ID[wire], DTYPE_ID[compute]
        self.offs = block_tensor_offsets(self.ccfg)
        L = cfg["n_layers"]
        wsz = lib().zo2_dtype_size(self.wire_id)
        self.n_tensors = 4 + 16 * L + (0 if cfg["tied"] else 1)
        self.scales = np.ones(self.n_tensors, dtype=np.float32) if scales is None else np.asarray(scales, np.float32)
        pin = pin and torch.cuda.is_available()
        tdt = TORCH_DTYPE[self.wire_id]

        def host(n):
            return torch.zeros(n, dtype=tdt, pin_memory=pin)

        def get(name, shape):
            return weights(name, shape) if callable(weights) else weights[name]

        def fill(dst, a, tid):
            dst.copy_(_to_wire(a, self.wire_id, float(self.scales[tid])))

        self.h_tok = host(cfg["vocab"] * cfg["d_model"]); fill(self.h_tok, get("tok_emb", (cfg["vocab"], cfg["d_model"])), 0)
        self.h_pos = host((cfg["max_pos"] + cfg["pos_offset"]) * cfg["d_model"]); fill(self.h_pos, get("pos_emb", (cfg["max_pos"] + cfg["pos_offset"], cfg["d_model"])), 1)
        self.h_flnw = host(cfg["d_model"]); fill(self.h_flnw, get("final_ln.w", (cfg["d_model"],)), 2 + 16 * L)
        self.h_flnb = host(cfg["d_model"]); fill(self.h_flnb, get("final_ln.b", (cfg["d_model"],)), 3 + 16 * L)
        self.h_lm = None
        if not cfg["tied"]:
            self.h_lm = host(cfg["vocab"] * cfg["d_model"]); fill(self.h_lm, get("lm_head.w", (cfg["vocab"], cfg["d_model"])), 4 + 16 * L)
        self.h_buckets = []
        for l in range(L):
            b = host(self.offs[16])
            for k, t in enumerate(BLOCK_TENSORS):
                a = get(f"blocks.{l}.{t}", block_tensor_shape(cfg, t))
                n = int(np.prod(a.shape))
                fill(b[self.offs[k]:self.offs[k] + n], a, 2 + 16 * l + k)
            self.h_buckets.append(b)

        model_bytes = wsz * (self.h_tok.numel() * (1 if cfg["tied"] else 2) + self.h_pos.numel() + L * self.offs[16])
        if arena_bytes is None:
            arena_bytes = int(model_bytes * 1.05) + (3 << 30)
        self.arena = torch.empty(int(arena_bytes), dtype=torch.uint8, device="cuda")
        self.streams = [torch.cuda.Stream() for _ in range(4)]
        self._bucket_ptrs = (C.c_void_p * max(L, 1))(*[b.data_ptr() for b in self.h_buckets])
        self._scales_c = self.scales.ctypes.data_as(C.POINTER(C.c_float)) if scales is not None else None
        hw = HostWeights(self.h_tok.data_ptr(), self.h_pos.data_ptr(), self.h_flnw.data_ptr(), self.h_flnb.data_ptr(),
                         self.h_lm.data_ptr() if self.h_lm is not None else None,
                         C.cast(self._bucket_ptrs, C.POINTER(C.c_void_p)), self._scales_c)
        dev = Device(self.arena.data_ptr(), self.arena.numel(), self.streams[0].cuda_stream, self.streams[1].cuda_stream,
                     self.streams[2].cuda_stream, self.streams[3].cuda_stream if overlap_k1 else None)
        self.handle = C.c_void_p()
        st = lib().zo2_init(C.byref(self.handle), C.byref(self.ccfg), C.byref(hw), C.byref(dev))
        if st != 0:
            msg = lib().zo2_last_error(self.handle).decode() if self.handle else lib().zo2_op_last_error().decode()
            if self.handle:
                lib().zo2_destroy(self.handle)
                self.handle = C.c_void_p()
            raise Zo2Error(st, msg)
        if budget_bytes is not None:
            self.set_resident_budget(budget_bytes)

    def _check(self, st, allow=()):
        if st != 0 and st not in allow:
            raise Zo2Error(st, lib().zo2_last_error(self.handle).decode())
        return st

    def set_resident_budget(self, nbytes):
        self._check(lib().zo2_set_resident_budget(self.handle, int(nbytes)))

    def step(self, tokens, labels, seed, eps, lr, allow_nonfinite=False):
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        lab = np.ascontiguousarray(labels, dtype=np.int32)
        assert tok.shape == lab.shape and tok.ndim == 2
        lp, lm, g = C.c_float(), C.c_float(), C.c_float()
        self._check(lib().zo2_step(self.handle, tok.ctypes.data, lab.ctypes.data, tok.shape[0], tok.shape[1], int(seed),
                                   float(eps), float(lr), C.byref(lp), C.byref(lm), C.byref(g)),
                    allow=(6,) if allow_nonfinite else ())
        return np.float32(lp.value), np.float32(lm.value), np.float32(g.value)

    def step_extra(self, tokens, labels, seed, eps, lr, allow_nonfinite=False):
        """One more direction of the current round (after step): same parameters, its update deferred with the others."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        lab = np.ascontiguousarray(labels, dtype=np.int32)
        assert tok.shape == lab.shape and tok.ndim == 2
        lp, lm, g = C.c_float(), C.c_float(), C.c_float()
        self._check(lib().zo2_step_extra(self.handle, tok.ctypes.data, lab.ctypes.data, tok.shape[0], tok.shape[1], int(seed),
                                         float(eps), float(lr), C.byref(lp), C.byref(lm), C.byref(g)),
                    allow=(6,) if allow_nonfinite else ())
        return np.float32(lp.value), np.float32(lm.value), np.float32(g.value)

    def step_multi(self, tokens, labels, seeds, eps, lr, allow_nonfinite=False):
        """A whole round of len(seeds) directions in one pass; returns a list of (l+, l-, g), one per direction."""
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        lab = np.ascontiguousarray(labels, dtype=np.int32)
        assert tok.shape == lab.shape and tok.ndim == 2
        sd = np.ascontiguousarray([int(x) for x in seeds], dtype=np.uint64)
        res = np.zeros(3 * len(sd), dtype=np.float32)
        self._check(lib().zo2_step_multi(self.handle, tok.ctypes.data, lab.ctypes.data, tok.shape[0], tok.shape[1], len(sd),
                                         sd.ctypes.data, float(eps), float(lr), res.ctypes.data),
                    allow=(6,) if allow_nonfinite else ())
        return [(np.float32(res[3 * j]), np.float32(res[3 * j + 1]), np.float32(res[3 * j + 2])) for j in range(len(sd))]

    def flush(self):
        self._check(lib().zo2_flush(self.handle))

    def eval(self, tokens, labels):
        tok = np.ascontiguousarray(tokens, dtype=np.int32)
        lab = np.ascontiguousarray(labels, dtype=np.int32)
        assert tok.shape == lab.shape and tok.ndim == 2
        loss = C.c_float()
        self._check(lib().zo2_eval(self.handle, tok.ctypes.data, lab.ctypes.data, tok.shape[0], tok.shape[1], C.byref(loss)))
        return np.float32(loss.value)

    def pending(self):
        """(has_pending, seed, eta * g) of the deferred update."""
        has, seed, step = C.c_int32(), C.c_uint64(), C.c_float()
        self._check(lib().zo2_get_pending(self.handle, C.byref(has), C.byref(seed), C.byref(step)))
        return bool(has.value), int(seed.value), np.float32(step.value)

    def set_pending(self, has_pending, seed=0, step=0.0):
        self._check(lib().zo2_set_pending(self.handle, 1 if has_pending else 0, int(seed), float(step)))

    def pending_list(self):
        """[(seed, eta * g), ...] of all deferred updates, in the order of application."""
        n = C.c_int32()
        self._check(lib().zo2_pending_count(self.handle, C.byref(n)))
        out = []
        for i in range(n.value):
            seed, step = C.c_uint64(), C.c_float()
            self._check(lib().zo2_get_pending_at(self.handle, i, C.byref(seed), C.byref(step)))
            out.append((int(seed.value), np.float32(step.value)))
        return out

    def set_pending_list(self, items):
        self.set_pending(False)
        for seed, step in items:
            self._check(lib().zo2_add_pending(self.handle, int(seed), float(step)))

    def sync_to_host(self):
        self._check(lib().zo2_sync_to_host(self.handle))

    def plan(self):
        n, r, b = C.c_int32(), C.c_int32(), C.c_size_t()
        self._check(lib().zo2_get_plan(self.handle, C.byref(n), C.byref(r), C.byref(b)))
        pg, se, ss = C.c_int32(), C.c_int64(), C.c_int32()
        self._check(lib().zo2_get_scratch_plan(self.handle, C.byref(pg), C.byref(se), C.byref(ss)))
        lf = C.c_int32()
        self._check(lib().zo2_get_loader_fusion(self.handle, C.byref(lf)))
        return dict(n_slots=n.value, resident=bool(r.value), bytes_used=b.value, sweeps_per_block=pg.value,
                    scratch_elems=se.value, scratch_sets=ss.value, loader_fusion=bool(lf.value))

    def set_loader_fusion(self, mode):
        """0: the projections perturb in their weight loader for steps of few tokens; 1: whenever possible; -1: never."""
        self._check(lib().zo2_set_loader_fusion(self.handle, int(mode)))

    def set_writeback_interval(self, updates):
        """Streamed blocks go back to the host once their host copy would lack this many updates (1: after every update)."""
        self._check(lib().zo2_set_writeback_interval(self.handle, int(updates)))

    def writeback_state(self):
        a, b_ = C.c_int32(), C.c_int32()
        self._check(lib().zo2_get_writeback_state(self.handle, C.byref(a), C.byref(b_)))
        return dict(interval=a.value, lacking=b_.value)

    def set_split_k(self, mode):
        """0: projections that would leave most compute units idle are split along k; -1: never."""
        self._check(lib().zo2_set_split_k(self.handle, int(mode)))

    def set_scratch_plan(self, sweeps):
        """1, 2 or 4 update + perturb sweeps per block (W+ / W- scratch for a whole block, a half, a tensor group);
        0: the planner chooses."""
        self._check(lib().zo2_set_scratch_plan(self.handle, int(sweeps)))

    def step_stats(self):
        a, b, c_ = C.c_float(), C.c_float(), C.c_float()
        u, d = C.c_uint64(), C.c_uint64()
        self._check(lib().zo2_get_step_stats(self.handle, C.byref(a), C.byref(b), C.byref(c_), C.byref(u), C.byref(d)))
        return dict(ms_compute=a.value, ms_upload=b.value, ms_offload=c_.value, bytes_up=u.value, bytes_down=d.value)

    def set_wire_rounding(self, stochastic):
        self._check(lib().zo2_set_wire_rounding(self.handle, 1 if stochastic else 0))

    def set_stream_overlap(self, enabled):
        self._check(lib().zo2_set_stream_overlap(self.handle, 1 if enabled else 0))

    def debug_set_stream_delay(self, which, microseconds):
        self._check(lib().zo2_debug_set_stream_delay(self.handle, {"compute": 0, "upload": 1, "offload": 2}[which], int(microseconds)))

    def debug_set_slot_poison(self, enabled):
        self._check(lib().zo2_debug_set_slot_poison(self.handle, 1 if enabled else 0))

    KERNEL_CLASSES = ("k1", "gemm", "attn", "ln", "embed", "ce")

    def set_profiling(self, classes=()):
        mask = 0
        for c_ in classes:
            mask |= 1 << self.KERNEL_CLASSES.index(c_)
        self._check(lib().zo2_set_profiling(self.handle, mask))

    def kernel_times(self):
        """class -> (milliseconds, launches) of the last step, for the classes being profiled."""
        ms = (C.c_float * 6)()
        n = (C.c_int32 * 6)()
        self._check(lib().zo2_get_kernel_times(self.handle, ms, n))
        return {k: (ms[i], n[i]) for i, k in enumerate(self.KERNEL_CLASSES)}

    def parameters(self):
        """name -> float32 numpy array decoded from the host buffers (call sync_to_host first)."""
        cfg, L = self.cfg, self.cfg["n_layers"]
        d = cfg["d_model"]
        out = {"tok_emb": _from_wire(self.h_tok, self.scales[0]).reshape(cfg["vocab"], d).numpy(),
               "pos_emb": _from_wire(self.h_pos, self.scales[1]).reshape(-1, d).numpy()}
        for l in range(L):
            for k, t in enumerate(BLOCK_TENSORS):
                shp = block_tensor_shape(cfg, t)
                n = int(np.prod(shp))
                out[f"blocks.{l}.{t}"] = _from_wire(self.h_buckets[l][self.offs[k]:self.offs[k] + n],
                                                    self.scales[2 + 16 * l + k]).reshape(shp).numpy()
        out["final_ln.w"] = _from_wire(self.h_flnw, self.scales[2 + 16 * L]).numpy()
        out["final_ln.b"] = _from_wire(self.h_flnb, self.scales[3 + 16 * L]).numpy()
        if self.h_lm is not None:
            out["lm_head.w"] = _from_wire(self.h_lm, self.scales[4 + 16 * L]).reshape(cfg["vocab"], d).numpy()
        return out

    def close(self):
        if getattr(self, "handle", None):
            lib().zo2_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
