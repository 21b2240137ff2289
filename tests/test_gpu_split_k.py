"""GPU tests of the projections split along k (launches with few rows per stream): the op against the oracle's linear
layer in float64 and against the unsplit launch; whole steps with the split active against the oracle's Alg. 2,
against the same steps without it, and streamed against resident bit for bit."""
import copy

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import codec, opt_model, zo_step
from oracle import opt_model as om

pytestmark = pytest.mark.gpu

TD = {"bf16": torch.bfloat16, "f16": torch.float16}
ACC_TOL = 2e-5
HALF_ULP = {"f32": 0.0, "bf16": 2.0 ** -9, "f16": 2.0 ** -12}


def _b():
    from paper_2503_12668_amd import binding
    return binding


def _within(got, ref, out_fmt):
    d = (got.double().cpu() - ref).abs()
    bound = ACC_TOL * max(1.0, float(ref.abs().max())) + 2 * HALF_ULP[out_fmt] * ref.abs()
    return bool((d <= bound).all())


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K,splits", [(512, 2048, 2048, 4), (300, 520, 1024, 2), (160, 256, 1024, 2), (1024, 2048, 8192, 2),
                                         (257, 260, 2048, 4), (40, 64, 512, 4)])
def test_split_k_gemm_against_the_oracle_linear_and_the_unsplit_launch(dt, M, N, K, splits):
    b = _b()
    g = torch.Generator().manual_seed(M + N + K)
    X = (torch.randn(M, K, generator=g) * 0.5).to(TD[dt])
    W = (torch.randn(N, K, generator=g) * 0.05).to(TD[dt])
    bias = torch.randn(N, generator=g).to(TD[dt])
    R = torch.randn(M, N, generator=g)
    ref = om.linear(X.double(), W.double(), bias.double()) * 0.125
    Xc, Wc, bc, Rc = X.cuda(), W.cuda(), bias.cuda(), R.cuda()
    # compute-dtype output with ReLU
    Y = b.op_gemm_split_k(Xc, Wc, splits, bias=bc, out_scale=0.125, relu=True)
    assert _within(Y, torch.clamp(ref, min=0.0), dt)
    # float32 output + residual
    Y32 = b.op_gemm_split_k(Xc, Wc, splits, bias=bc, residual=Rc, out_dtype=b.F32, out_scale=0.125)
    assert _within(Y32, ref + R.double(), "f32")
    Y1 = b.op_gemm(Xc, Wc, bc, residual=Rc, out_dtype=b.F32, out_scale=0.125)
    assert float((Y32 - Y1).abs().max()) <= ACC_TOL * max(1.0, float(ref.abs().max()))
    # deterministic
    Y32b = b.op_gemm_split_k(Xc, Wc, splits, bias=bc, residual=Rc, out_dtype=b.F32, out_scale=0.125)
    assert torch.equal(Y32, Y32b)


def test_split_k_rejects_what_it_cannot_do():
    b = _b()
    X = torch.zeros(64, 512, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(64, 512, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(b.Zo2Error):
        b.op_gemm_split_k(X, W, 3)                               # 2 or 4 pieces
    with pytest.raises(b.Zo2Error):
        b.op_gemm_split_k(X.float(), W.float(), 2, out_dtype=b.F32)      # 16-bit formats only
    W2 = torch.zeros(66, 512, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(b.Zo2Error):
        b.op_gemm_split_k(X, W2, 2)                              # N % 4
    assert b.op_gemm_split_k_pieces(b.DTYPE_ID["bf16"], 4096, 2048, 2048, 2) == 1      # the benchmark's launches are not split
    assert b.op_gemm_split_k_pieces(b.DTYPE_ID["bf16"], 512, 2048, 8192, 2) == 4
    assert b.op_gemm_split_k_pieces(b.DTYPE_ID["f32"], 512, 2048, 8192, 2) == 1


def _model():
    # d 256 / ffn 2048 at 2 x 80 tokens: FC2 (k = 2048) is split into 4 pieces; the other projections have k = 256, too short to split
    cfg = si.tiny_config(n_layers=4, d_model=256, n_heads=4, d_ffn=2048, vocab=331, max_pos=96)
    P = si.make_weights(cfg, seed=11, std=0.05, ln_jitter=True)
    tok = si.make_tokens(cfg["vocab"], 2, 80, seed=12)
    lab = si.next_token_labels(tok)
    lab[1, 7] = -100
    return cfg, P, tok, lab


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_steps_with_split_projections_track_the_oracle_and_the_unsplit_steps(dt):
    b = _b()
    cfg, P, tok, lab = _model()
    T = tok.size
    assert b.op_gemm_split_k_pieces(b.DTYPE_ID[dt], T, cfg["d_model"], cfg["d_ffn"], 2) > 1      # FC2 is split at this shape
    Po = {n: codec.round_to(a, dt) for n, a in P.items()}
    oz = zo_step.Zo2Blockwise(opt_model.OptShape(**cfg), copy.deepcopy(Po), store=dt, compute=dt)
    split = b.Zo2Context(cfg, P, wire=dt, compute=dt, arena_bytes=256 << 20)
    plain = b.Zo2Context(cfg, P, wire=dt, compute=dt, arena_bytes=256 << 20)
    plain.set_split_k(-1)
    for j in range(3):
        a = oz.step(tok, lab, 42 + j, 1e-3, 1e-2)
        s = split.step(tok, lab, 42 + j, 1e-3, 1e-2)
        p = plain.step(tok, lab, 42 + j, 1e-3, 1e-2)
        for k in (0, 1):
            assert abs(float(s[k]) - float(a[k])) <= 2e-2 * abs(float(a[k])), (j, k)
            assert abs(float(s[k]) - float(p[k])) <= (2e-3 if j == 0 else 2e-2) * abs(float(p[k])), (j, k)
    ev_s, ev_p, ev_o = split.eval(tok, lab), plain.eval(tok, lab), oz.eval_loss(tok, lab)
    assert abs(float(ev_s) - float(ev_p)) <= 2e-2 * abs(float(ev_p))
    assert abs(float(ev_s) - float(ev_o)) <= 2e-2 * abs(float(ev_o))
    split.close(); plain.close()


def test_split_projections_streamed_equals_resident_bitwise():
    b = _b()
    cfg, P, tok, lab = _model()
    runs = {}
    for name in ("resident", "streamed"):
        ctx = b.Zo2Context(cfg, P, wire="bf16", compute="bf16", arena_bytes=256 << 20)
        r = [ctx.step(tok, lab, 5, 1e-3, 1e-3)]
        if name == "streamed":
            ctx.set_resident_budget(ctx.plan()["bytes_used"] - 1 * ctx.offs[16] * 2)        # 3 slots for 4 blocks
            ctx.debug_set_slot_poison(True)
        r.append(ctx.step(tok, lab, 6, 1e-3, 1e-3))
        r.append(ctx.step_extra(tok, lab, 7, 1e-3, 5e-4))
        r.append(ctx.step(tok, lab, 8, 1e-3, 1e-3))
        ev = ctx.eval(tok, lab)
        pl = ctx.plan()
        assert pl["resident"] == (name == "resident") and not pl["loader_fusion"], pl
        ctx.flush(); ctx.sync_to_host()
        runs[name] = ([tuple(map(float, x)) for x in r] + [float(ev)], ctx.parameters())
        ctx.close()
    assert runs["streamed"][0] == runs["resident"][0]
    for n in runs["resident"][1]:
        assert np.array_equal(runs["streamed"][1][n], runs["resident"][1][n]), n
