"""GPU parity of the forward kernels (GEMM, attention, LayerNorm, cross-entropy) against the oracle's own
operations (oracle/opt_model.py: linear, causal_attention, layer_norm, row_cross_entropy), evaluated in float64
on the CPU from the same inputs.

Bounds.  Inputs are exact in their storage format, so what separates the kernel from the float64 value is the
float32 accumulation of K products (observed ~1e-6 of the largest output; bound 2e-5) and, for 16-bit outputs, one
rounding of the result to the format (half a unit in the last place: 2^-9 of the value for bf16, 2^-12 for fp16,
here with a factor two of slack)."""
import numpy as np
import pytest
import torch

from oracle import opt_model as om

pytestmark = pytest.mark.gpu

TD = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def _b():
    from paper_2503_12668_amd import binding
    return binding


ACC_TOL = 2e-5                                   # float32 accumulation, relative to the largest output
HALF_ULP = {"f32": 0.0, "bf16": 2.0 ** -9, "f16": 2.0 ** -12}


def _within(got, ref, out_fmt):
    """|got - ref| <= ACC_TOL max(1, max|ref|) + 2 * (half a unit in the last place of the output format at |ref|)."""
    d = (got.double().cpu() - ref).abs()
    bound = ACC_TOL * max(1.0, float(ref.abs().max())) + 2 * HALF_ULP[out_fmt] * ref.abs()
    return bool((d <= bound).all())


@pytest.mark.parametrize("dt", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (22, 32, 32), (200, 136, 72), (257, 515, 264), (128, 97 * 8, 40), (4, 8, 8),
                                   (256, 256, 64), (512, 768, 128), (300, 515, 192), (1024, 384, 2048), (700, 1030, 320),
                                   # the 256 x 256 kernel (K % 128 == 0) with ragged rows and columns, two to six k-slabs
                                   (257, 260, 128), (300, 520, 256), (700, 1032, 384),
                                   # the same kernel with fewer rows than a tile has (128-row tiles, rows clamped and masked)
                                   (1, 256, 128), (16, 512, 256), (100, 264, 128), (130, 2048, 2048), (200, 520, 384)])
def test_gemm_against_float64(dt, M, N, K):
    b = _b()
    g = torch.Generator().manual_seed(M * 1000 + N + K)
    X = (torch.randn(M, K, generator=g) * 0.5).to(TD[dt])
    W = (torch.randn(N, K, generator=g) * 0.5).to(TD[dt])
    bias = (torch.randn(N, generator=g)).to(TD[dt])
    R = torch.randn(M, N, generator=g)
    ref = om.linear(X.double(), W.double(), bias.double()) * 0.125
    # plain, compute-dtype output
    out_dt = b.F32 if dt == "f32" else None
    Y = b.op_gemm(X.cuda(), W.cuda(), bias.cuda(), out_scale=0.125, out_dtype=out_dt)
    assert _within(Y, ref, dt)
    # relu + residual, float32 output
    Y2 = b.op_gemm(X.cuda(), W.cuda(), bias.cuda(), residual=R.cuda(), out_scale=0.125, relu=True, out_dtype=b.F32)
    assert _within(Y2, torch.relu(ref) + R.double(), "f32")
    # no bias, strided operands
    Xs = torch.zeros(M, K + 8, dtype=TD[dt]); Xs[:, :K] = X
    Y3 = b.op_gemm(Xs.cuda()[:, :K], W.cuda(), out_dtype=b.F32)
    assert _within(Y3, om.linear(X.double(), W.double()), "f32")


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K", [(257, 260, 128), (300, 520, 256), (700, 1032, 384), (1024, 384, 2048), (2048, 512, 512)])
def test_gemm_tile_heights_and_wavefront_counts(dt, M, N, K):
    """The large-tile kernel with 128-row tiles and with 256-row tiles run by four and by eight wavefronts: each against
    float64, and against each other bit for bit (the order in which a dot product is accumulated depends on neither)."""
    b = _b()
    g = torch.Generator().manual_seed(M + N + K)
    X = (torch.randn(M, K, generator=g) * 0.5).to(TD[dt]).cuda()
    W = (torch.randn(N, K, generator=g) * 0.5).to(TD[dt]).cuda()
    bias = (torch.randn(N, generator=g)).to(TD[dt]).cuda()
    R = torch.randn(M, N, generator=g).cuda()
    ref = om.linear(X.double().cpu(), W.double().cpu(), bias.double().cpu()) * 0.125
    ref2 = torch.relu(ref) + R.double().cpu()
    out = {}
    try:
        for rows, waves in ((128, 0), (256, 4), (256, 8)):
            b.op_set_gemm_tile_rows(rows)
            b.op_set_gemm_wavefronts(waves)
            Y = b.op_gemm(X, W, bias, out_scale=0.125)
            Y2 = b.op_gemm(X, W, bias, residual=R, out_scale=0.125, relu=True, out_dtype=b.F32)
            assert _within(Y, ref, dt), (rows, waves)
            assert _within(Y2, ref2, "f32"), (rows, waves)
            out[rows, waves] = (Y.cpu(), Y2.cpu())
        with pytest.raises(b.Zo2Error):
            b.op_set_gemm_tile_rows(64)
        with pytest.raises(b.Zo2Error):
            b.op_set_gemm_wavefronts(2)
    finally:
        b.op_set_gemm_tile_rows(0)
        b.op_set_gemm_wavefronts(0)
    for key in ((256, 4), (256, 8)):
        assert torch.equal(out[128, 0][0].view(torch.int16), out[key][0].view(torch.int16)), key
        assert torch.equal(out[128, 0][1], out[key][1]), key


def test_gemm_rejects_bad_arguments():
    b = _b()
    X = torch.zeros(8, 12, device="cuda", dtype=torch.bfloat16)
    W = torch.zeros(8, 12, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(b.Zo2Error):
        b.op_gemm(X, W)                      # K not a multiple of 8


def _attention_ref(q, k, v, n_seq, seq, H, dh):
    sh = lambda t: t.double().view(n_seq, seq, H * dh)
    return om.causal_attention(sh(q), sh(k), sh(v), H).reshape(n_seq * seq, H * dh)


@pytest.mark.parametrize("dt", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("n_seq,seq,H,dh", [(2, 11, 4, 8), (3, 64, 2, 64), (2, 130, 3, 32), (1, 257, 2, 128), (4, 1, 2, 16),
                                           (2, 256, 3, 64), (2, 23, 2, 64), (1, 300, 2, 128), (3, 33, 1, 128), (2, 200, 3, 80), (1, 31, 2, 80)])
@pytest.mark.parametrize("vector_kernel", [False, True])
def test_attention_against_float64(dt, n_seq, seq, H, dh, vector_kernel):
    b = _b()
    g = torch.Generator().manual_seed(seq * 7 + dh)
    mk = lambda s: (torch.randn(n_seq * seq, H * dh, generator=g) * s).to(TD[dt])
    q, k, v = mk(0.3), mk(1.0), mk(1.0)
    out = b.op_attention(q.cuda(), k.cuda(), v.cuda(), n_seq, seq, H, dh, vector_kernel=vector_kernel)
    ref = _attention_ref(q, k, v, n_seq, seq, H, dh)
    tol = 2e-6 if dt == "f32" else 1.5e-2
    assert (out.double().cpu() - ref).abs().max() <= tol * max(1.0, ref.abs().max())


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("rows,d", [(5, 32), (64, 768), (9, 2048), (7, 2056), (6, 5120), (5, 7168), (4, 9216), (3, 12288), (3, 12296), (2, 16384), (3, 1028)])
def test_layernorm_two_parameter_sets(dt, rows, d):
    b = _b()
    g = torch.Generator().manual_seed(d)
    x = torch.randn(rows, d, generator=g) * 2 + 0.5
    w1, b1, w2, b2 = [(torch.randn(d, generator=g) * 0.1 + o).to(TD[dt]) for o in (1, 0, 1, 0)]
    first = rows // 2
    y = b.op_layernorm(x.cuda(), w1.cuda(), b1.cuda(), 1e-5, w2.cuda(), b2.cuda(), rows_first=first)
    xd = x.double()
    ref = torch.cat([om.layer_norm(xd[:first], w1.double(), b1.double(), 1e-5), om.layer_norm(xd[first:], w2.double(), b2.double(), 1e-5)])
    d_ = (y.double().cpu() - ref).abs()
    assert bool((d_ <= 2e-6 * max(1.0, float(ref.abs().max())) + 2 * HALF_ULP[dt] * ref.abs()).all())


@pytest.mark.parametrize("rows,V", [(7, 97), (33, 50272), (2, 256)])
def test_cross_entropy_rows(rows, V):
    b = _b()
    g = torch.Generator().manual_seed(V)
    lg = torch.randn(rows, V, generator=g) * 3
    lab = torch.randint(0, V, (rows,), generator=g, dtype=torch.int32)
    lab[rows // 2] = -100
    out = b.op_cross_entropy_rows(lg.cuda(), lab.cuda())
    ref = om.row_cross_entropy(lg.double(), lab.numpy())
    assert float(ref[rows // 2]) == 0.0
    assert (out.double().cpu() - ref).abs().max() <= 2e-6 * ref.abs().max()


def test_lm_head_ce_small_and_bad_shapes():
    b = _b()
    g = torch.Generator().manual_seed(1)
    M, N, K = 300, 520, 128                                  # ragged in both directions, several spans per row
    X = (torch.randn(M, K, generator=g)).to(torch.float16)
    W = (torch.randn(N, K, generator=g) * 0.2).to(torch.float16)
    lab = torch.randint(0, N, (M,), generator=g, dtype=torch.int32)
    lab[0] = -100
    ref = om.row_cross_entropy(om.linear(X.double(), W.double()), lab.numpy())
    assert float(ref[0]) == 0.0
    try:
        for rows, waves in ((128, 0), (256, 4), (256, 8), (0, 0)):      # the three forms of the GEMM, then its own choice
            b.op_set_gemm_tile_rows(rows)
            b.op_set_gemm_wavefronts(waves)
            out = b.op_lm_head_ce(X.cuda(), W.cuda(), lab.cuda()).cpu()
            assert (out.double() - ref).abs().max() <= ACC_TOL * max(1.0, float(ref.abs().max())), (rows, waves)
    finally:
        b.op_set_gemm_tile_rows(0)
        b.op_set_gemm_wavefronts(0)
    with pytest.raises(b.Zo2Error):
        b.op_lm_head_ce(X[:100].cuda(), W.cuda(), lab[:100].cuda())          # fewer than 256 rows
    with pytest.raises(b.Zo2Error):
        b.op_lm_head_ce(X.float().cuda(), W.float().cuda(), lab.cuda())      # float32 has no fused path
    with pytest.raises(b.Zo2Error):
        b.op_lm_head_ce(X[:, :64].contiguous().cuda(), W[:, :64].contiguous().cuda(), lab.cuda())   # K is not a multiple of 128


def test_gemm_phases_needs_the_instrumented_build():
    """The ordinary library carries no cycle stamps: the measurement entry point says so instead of running."""
    b = _b()
    X = torch.zeros(256, 128, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(256, 128, dtype=torch.bfloat16, device="cuda")
    Y = torch.empty(256, 256, dtype=torch.bfloat16, device="cuda")
    stamps = torch.zeros(64, dtype=torch.int64, device="cuda")
    with pytest.raises(b.Zo2Error):
        b.op_gemm_phases(X, W, Y, stamps)
