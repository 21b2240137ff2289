"""GPU parity of the projection that perturbs in its weight loader (few tokens per step): the bits of W+- against the
sweep kernel's, the outputs against the oracle's linear() on oracle-made W+-, and against the ordinary path."""
import numpy as np
import pytest
import torch

from oracle import codec, philox
from oracle import opt_model as om
from oracle.zo_step import _fma32, _store

pytestmark = pytest.mark.gpu

TD = {"bf16": torch.bfloat16, "f16": torch.float16}


def _b():
    from paper_2503_12668_amd import binding
    return binding


@pytest.mark.parametrize("dt", ["bf16", "f16"])
def test_loader_perturbation_has_the_bits_of_the_sweep_kernel_and_of_the_oracle(dt):
    b = _b()
    N, K, tid, seed, eps = 200, 320, 2 + 16 * 5 + 12, 42, 1e-3
    g = torch.Generator().manual_seed(1)
    theta = (torch.randn(N, K, generator=g) * 0.02).to(TD[dt])
    n0, rows = 24, 130
    wp, wm = b.op_perturbed_rows(theta[n0:n0 + rows].contiguous().cuda(), K, n0, tid, seed, eps)
    # the sweep kernel on the same window (no update)
    t = theta[n0:n0 + rows].contiguous().cuda().reshape(-1)
    kp, km = torch.empty_like(t), torch.empty_like(t)
    b.op_update_perturb(t, kp, km, tid, n0 * K, False, 0, 0.0, seed, eps)
    torch.cuda.synchronize()
    assert torch.equal(wp.reshape(-1).view(torch.int16), kp.view(torch.int16)) and torch.equal(wm.reshape(-1).view(torch.int16), km.view(torch.int16))
    # and the oracle (z agrees to 2e-6, so a few values may sit across a rounding boundary)
    z = philox.gaussian(seed, tid, n0 * K, rows * K)
    th = theta[n0:n0 + rows].float().numpy().reshape(-1)
    want = _store(_fma32(np.float32(eps), z, th), dt)
    got = wp.float().cpu().numpy().reshape(-1)
    assert np.mean(got == want) > 0.98 and np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -7 + 1e-9)


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K,res,relu", [(1, 64, 64, False, False), (19, 136, 192, True, False), (32, 128, 64, False, False), (33, 200, 448, True, True), (64, 2048, 2048, False, True),
                                            (100, 520, 8192, True, False), (128, 260, 256, False, False), (129, 64, 128, True, True),
                                            (256, 768, 3072, True, False), (200, 6144, 2048, False, False)])
def test_perturbed_gemm_against_oracle_linear(dt, M, N, K, res, relu):
    b = _b()
    tid, seed, eps = 7, 1234, 1e-3
    g = torch.Generator().manual_seed(M + N + K)
    Xp = (torch.randn(M, K, generator=g) * 0.5).to(TD[dt])
    Xm = (torch.randn(M, K, generator=g) * 0.5).to(TD[dt])
    theta = (torch.randn(N, K, generator=g) * 0.05).to(TD[dt])
    bp, bm = [(torch.randn(N, generator=g) * 0.1).to(TD[dt]) for _ in range(2)]
    Rp, Rm = (torch.randn(M, N, generator=g), torch.randn(M, N, generator=g)) if res else (None, None)
    cu = lambda t: None if t is None else t.cuda()
    Yp, Ym = b.op_gemm_perturbed(cu(Xp), cu(Xm), cu(theta), tid, seed, eps, cu(bp), cu(bm), cu(Rp), cu(Rm),
                                 out_dtype=b.F32 if res else None, out_scale=0.25, relu=relu)
    # reference: the oracle's z and rounding make W+-, the oracle's linear() does the rest in float64
    z = philox.gaussian(seed, tid, 0, N * K).reshape(N, K)
    th = theta.float().numpy()
    half_ulp = 0.0 if res else (2.0 ** -9 if dt == "bf16" else 2.0 ** -12)
    for Y, X, sign, bias, R in ((Yp, Xp, 1.0, bp, Rp), (Ym, Xm, -1.0, bm, Rm)):
        W = _store(_fma32(np.float32(sign * eps), z, th), dt)
        ref = om.linear(X.double(), torch.from_numpy(W).double(), bias.double()) * 0.25
        if relu:
            ref = torch.relu(ref)
        if res:
            ref = ref + R.double()
        d = (Y.double().cpu() - ref).abs()
        # float32 accumulation, the output's rounding, and the ~1 % of weights that sit one unit away (dz = 2e-6)
        bound = 2e-5 * max(1.0, float(ref.abs().max())) + 2 * half_ulp * ref.abs() + 0.25 * 0.02 * float(X.abs().max()) * 0.05 * 2.0 ** -7 * np.sqrt(K)
        assert bool((d <= bound).all()), float((d - bound).max())


def test_perturbed_gemm_equals_the_ordinary_path_and_is_deterministic():
    """Sweep kernel + ordinary GEMM on its W+- against the fused loader: same weights bit for bit, so the outputs differ by
    the order of the float32 additions only; and two runs of the fused kernel are identical (ordered slice sums)."""
    b = _b()
    M, N, K, tid, seed, eps = 96, 2048, 8192, 40, 9, 1e-3
    g = torch.Generator(device="cuda").manual_seed(3)
    Xp = torch.randn(M, K, device="cuda", generator=g).bfloat16()
    Xm = torch.randn(M, K, device="cuda", generator=g).bfloat16()
    theta = (torch.randn(N, K, device="cuda", generator=g) * 0.02).bfloat16()
    R = torch.randn(M, N, device="cuda", generator=g)
    Yp, Ym = b.op_gemm_perturbed(Xp, Xm, theta, tid, seed, eps, res_p=R, res_m=R, out_dtype=b.F32)
    Yp2, Ym2 = b.op_gemm_perturbed(Xp, Xm, theta, tid, seed, eps, res_p=R, res_m=R, out_dtype=b.F32)
    assert torch.equal(Yp, Yp2) and torch.equal(Ym, Ym2)
    t = theta.clone().reshape(-1)
    wp, wm = torch.empty_like(t), torch.empty_like(t)
    b.op_update_perturb(t, wp, wm, tid, 0, False, 0, 0.0, seed, eps)
    Zp = b.op_gemm(Xp, wp.reshape(N, K), residual=R, out_dtype=b.F32)
    Zm = b.op_gemm(Xm, wm.reshape(N, K), residual=R, out_dtype=b.F32)
    for Y, Z in ((Yp, Zp), (Ym, Zm)):
        assert (Y - Z).abs().max() <= 2e-5 * max(1.0, float(Z.abs().max()))
    assert not torch.equal(Yp, Ym)


@pytest.mark.parametrize("M,N,K,layer,k", [(48, 5120, 5120, 39, 2), (48, 20480, 5120, 39, 12), (48, 5120, 20480, 39, 14),
                                           (16, 49152, 12288, 95, 12), (16, 12288, 49152, 95, 14), (128, 7168, 7168, 47, 8)])
def test_perturbed_gemm_sampled_columns_at_the_13b_30b_175b_widths(M, N, K, layer, k):
    """Projections of the larger shapes (whole weight matrices of OPT-13B / 30B / 175B blocks, their real tensor ids): 96
    sampled output features, each against the oracle - z and the rounding of W+- from the oracle for that feature's row
    of the matrix (element offset n K inside the tensor), the dot products in float64."""
    b = _b()
    tid, seed, eps = 2 + 16 * layer + k, 77, 1e-3
    g = torch.Generator(device="cuda").manual_seed(N + K)
    theta = torch.empty(N, K, device="cuda", dtype=torch.bfloat16)
    step = max(1, (64 << 20) // K)
    for r0 in range(0, N, step):
        theta[r0:r0 + step] = (torch.randn(min(step, N - r0), K, device="cuda", generator=g) * 0.02).bfloat16()
    Xp = (torch.randn(M, K, device="cuda", generator=g) * 0.5).bfloat16()
    Xm = (torch.randn(M, K, device="cuda", generator=g) * 0.5).bfloat16()
    bias = (torch.randn(N, device="cuda", generator=g) * 0.1).bfloat16()
    Yp, Ym = b.op_gemm_perturbed(Xp, Xm, theta, tid, seed, eps, bias, bias, out_dtype=b.F32)
    torch.cuda.synchronize()
    rs = np.random.RandomState(N % 1000 + K % 1000)
    cols = np.unique(np.concatenate([[0, 1, 127, 128, N - 129, N - 2, N - 1], rs.randint(0, N, 89)]))
    xp, xm = Xp.double().cpu(), Xm.double().cpu()
    bcpu = bias.double().cpu()
    worst = 0.0
    for n in cols:
        th = theta[n].float().cpu().numpy()
        z = philox.gaussian(seed, tid, int(n) * K, K)
        for Y, X, sign in ((Yp, xp, 1.0), (Ym, xm, -1.0)):
            w = torch.from_numpy(_store(_fma32(np.float32(sign * eps), z, th), "bf16")).double()
            ref = X @ w + bcpu[n]
            d = (Y[:, n].double().cpu() - ref).abs()
            # float32 accumulation plus the ~1 % of weights that sit one unit away (z agrees to 2e-6)
            bound = 2e-5 * max(1.0, float(ref.abs().max())) + 0.02 * 0.5 * 4 * 0.02 * 2.0 ** -7 * np.sqrt(K)
            worst = max(worst, float((d - bound).max()))
    assert worst <= 0.0, worst


def test_perturbed_gemm_rejects_what_it_does_not_cover():
    b = _b()
    X = torch.zeros(300, 128, device="cuda", dtype=torch.bfloat16)
    W = torch.zeros(64, 128, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(b.Zo2Error):
        b.op_gemm_perturbed(X, X, W, 1, 1, 1e-3)                    # more than 256 rows
    with pytest.raises(b.Zo2Error):
        b.op_gemm_perturbed(X[:8, :96].contiguous(), X[:8, :96].contiguous(), W[:, :96].contiguous(), 1, 1, 1e-3)   # K % 64 != 0
    with pytest.raises(b.Zo2Error):
        b.op_gemm_perturbed(X[:8].float(), X[:8].float(), W.float(), 1, 1, 1e-3)   # float32
