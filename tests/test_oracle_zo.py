"""Pins for the oracle's ZO-SGD step (run without a GPU)."""
import copy

import numpy as np
import pytest

import synth_inputs as si
from oracle import opt_model, philox, zo_step

from hf_reference import hf_param_grads


def _setup(tied=True, std=0.1, seed=1):
    cfg = si.tiny_config(n_layers=2, d_model=32, n_heads=4, d_ffn=64, vocab=97, max_pos=24, tied=tied)
    P = si.make_weights(cfg, seed=seed, std=std, ln_jitter=True)
    tok = si.make_tokens(cfg["vocab"], 2, 11, seed=2)
    return cfg, opt_model.OptShape(**cfg), P, tok, si.next_token_labels(tok)


def _loss64_at(s, P, z, t, tok, lab):
    W = {n: P[n].astype(np.float64) + t * z[n].astype(np.float64) for n in P}
    return opt_model.loss(s, W, tok, lab)


@pytest.mark.parametrize("tied", [True, False])
def test_projected_gradient_is_directional_derivative(tied):
    """Eq. 2: g -> z . grad L as eps -> 0.  grad L comes from autograd through an
    independently written module.  The ReLU FFN makes L only piecewise smooth, so the
    generic case is checked at an eps small enough that no unit switches (float64),
    and the O(eps^2) law of the central difference is checked where L is smooth along
    the whole segment (FFN biases shifted so that every unit stays active)."""
    cfg, s, P, tok, lab = _setup(tied=tied)
    z = zo_step.z_of(s, 42)
    _, grads = hf_param_grads(cfg, P, tok, lab)
    dd = sum(float(np.sum(grads[n] * z[n].astype(np.float64))) for n in P)
    g = (_loss64_at(s, P, z, 1e-6, tok, lab) - _loss64_at(s, P, z, -1e-6, tok, lab)) / 2e-6
    assert abs(g - dd) < 1e-6 * abs(dd)          # the module's float32 softmax limits dd to ~1e-7

    for l in range(cfg["n_layers"]):
        P[f"blocks.{l}.fc1.b"] = P[f"blocks.{l}.fc1.b"] + np.float32(4.0)
    _, grads = hf_param_grads(cfg, P, tok, lab)
    dd = sum(float(np.sum(grads[n] * z[n].astype(np.float64))) for n in P)
    errs = []
    for eps in (4e-3, 2e-3, 1e-3):
        g = (_loss64_at(s, P, z, eps, tok, lab) - _loss64_at(s, P, z, -eps, tok, lab)) / (2 * eps)
        errs.append(abs(g - dd))
    assert errs[2] < 2e-3 * abs(dd)
    assert 3.8 < errs[0] / errs[1] < 4.2 and 3.8 < errs[1] / errs[2] < 4.2      # error ~ eps^2
    # the float32 step (canonical arithmetic) reports the same number up to the
    # cancellation in l+ - l-: |dg| <= ulp32(l) / (2 eps) ~ 5e-7 * 5 / 2e-3
    lp, lm, g32 = zo_step.step_whole(s, copy.deepcopy(P), tok, lab, 42, 1e-3, 0.0)
    assert abs(float(g32) - dd) < errs[2] + 2.5e-3


def test_update_uses_the_same_z_and_sign():
    """Eq. 3: theta_new = theta - eta g z with the z of Eq. 2."""
    cfg, s, P, tok, lab = _setup()
    P0 = copy.deepcopy(P)
    lp, lm, g = zo_step.step_whole(s, P, tok, lab, 42, 1e-3, 1e-4)
    assert g != 0
    z = zo_step.z_of(s, 42)
    for n in P:
        want = P0[n].astype(np.float64) - 1e-4 * float(g) * z[n].astype(np.float64)
        assert np.abs(P[n] - want).max() < 2e-7, n
    # a first-order check of descent direction: moving along -g z lowers the loss
    assert opt_model.loss(s, P, tok, lab) < opt_model.loss(s, P0, tok, lab)


def test_in_place_sequence_vs_exact_restore():
    """Eq. 1-3 evaluated by moving the parameters in place (by eps z times +1, -2, +1, then the update)
    against the canonical copy-based form: same losses up to float32 rounding of the perturbation, and
    parameters within a few float32 ulps per step."""
    cfg, s, P, tok, lab = _setup()
    Pa, Pb = copy.deepcopy(P), copy.deepcopy(P)
    for j in range(3):
        la = zo_step.step_in_place(s, Pa, tok, lab, 42 + j, 1e-3, 1e-3)
        lb = zo_step.step_whole(s, Pb, tok, lab, 42 + j, 1e-3, 1e-3)
        assert abs(float(la[0]) - float(lb[0])) < 2e-6 * abs(float(lb[0]))
        assert abs(float(la[1]) - float(lb[1])) < 2e-6 * abs(float(lb[1]))
        for n in P:
            ulp = np.spacing(np.abs(Pb[n]) + np.float32(6e-3))
            assert np.all(np.abs(Pa[n] - Pb[n]) <= 4 * (j + 1) * ulp), (j, n)


@pytest.mark.parametrize("tied", [True, False])
def test_blockwise_deferred_equals_whole_model(tied):
    """Alg. 2 with the deferred update (Sec. 5.4) reproduces Alg. 1 exactly: the same
    l+, l- at every iteration and, after the pending update is applied, the same theta."""
    cfg, s, P, tok, lab = _setup(tied=tied)
    Pa, Pb = copy.deepcopy(P), copy.deepcopy(P)
    zo = zo_step.Zo2Blockwise(s, Pb)
    for j in range(4):
        lr = 1e-3 * (j + 1)                     # eta_j travels with g_j
        a = zo_step.step_whole(s, Pa, tok, lab, 100 + j, 1e-3, lr)
        b = zo.step(tok, lab, 100 + j, 1e-3, lr)
        assert tuple(map(float, a)) == tuple(map(float, b)), j
    assert any(not np.array_equal(Pa[n], Pb[n]) for n in P)     # last update still pending
    zo.flush()
    for n in P:
        assert np.array_equal(Pa[n], Pb[n]), n


def test_eval_loss_is_the_loss_of_the_updated_parameters():
    """The single-forward evaluation sees theta with the deferred update applied: it equals the loss of
    Alg. 1's theta_{j+1} (whole-model form), it is the eps -> 0 limit of (l+ + l-) / 2 of a step taken from
    there (the odd terms cancel), and it leaves nothing pending."""
    cfg, s, P, tok, lab = _setup()
    tok2 = si.make_tokens(cfg["vocab"], 2, 11, seed=9)
    lab2 = si.next_token_labels(tok2)
    Pa, Pb = copy.deepcopy(P), copy.deepcopy(P)
    zo = zo_step.Zo2Blockwise(s, Pb)
    for j in range(3):
        zo_step.step_whole(s, Pa, tok, lab, 100 + j, 1e-3, 2e-3)
        zo.step(tok, lab, 100 + j, 1e-3, 2e-3)
    ev = zo.eval_loss(tok2, lab2)
    assert zo.pending is None
    assert float(ev) == float(np.float32(opt_model.loss(s, Pa, tok2, lab2)))       # Alg. 1's parameters, same loss
    gaps = []
    for eps in (2e-3, 1e-3):
        lp, lm, _ = zo_step.step_whole(s, copy.deepcopy(Pa), tok2, lab2, 7, eps, 0.0)
        gaps.append(abs(0.5 * (float(lp) + float(lm)) - float(ev)))
    assert gaps[0] < 1e-4 * float(ev) and gaps[1] < gaps[0]          # shrinks with eps (ReLU kinks keep it from a clean eps^2)
    # training continued after an evaluation is the training without it
    a = zo_step.step_whole(s, Pa, tok, lab, 200, 1e-3, 1e-3)
    b = zo.step(tok, lab, 200, 1e-3, 1e-3)
    assert tuple(map(float, a)) == tuple(map(float, b))


def test_zero_learning_rate_and_sign_symmetry():
    cfg, s, P, tok, lab = _setup()
    P0 = copy.deepcopy(P)
    zo = zo_step.Zo2Blockwise(s, P)
    r1 = zo.step(tok, lab, 5, 1e-3, 0.0)
    r2 = zo.step(tok, lab, 5, -1e-3, 0.0)
    zo.flush()
    for n in P:
        assert np.array_equal(P[n], P0[n])
    assert float(r1[0]) == float(r2[1]) and float(r1[1]) == float(r2[0])
    assert float(r1[2]) == float(r2[2])


def test_same_seed_same_step_different_seed_different_step():
    cfg, s, P, tok, lab = _setup()
    a = zo_step.step_whole(s, copy.deepcopy(P), tok, lab, 42, 1e-3, 1e-3)
    b = zo_step.step_whole(s, copy.deepcopy(P), tok, lab, 42, 1e-3, 1e-3)
    c = zo_step.step_whole(s, copy.deepcopy(P), tok, lab, 43, 1e-3, 1e-3)
    assert tuple(map(float, a)) == tuple(map(float, b))
    assert float(a[2]) != float(c[2])


def test_low_bit_storage_step_keeps_parameters_representable():
    """Sec. 5.5: with parameters held in bf16 the updated theta is again a bf16 value,
    W+- are bf16 values, and blockwise == whole-model still holds."""
    from oracle import codec
    cfg, s, P, tok, lab = _setup()
    P = {n: codec.round_to(a, "bf16") for n, a in P.items()}
    Pa, Pb = copy.deepcopy(P), copy.deepcopy(P)
    zo = zo_step.Zo2Blockwise(s, Pb, store="bf16", compute="bf16")
    for j in range(2):
        a = zo_step.step_whole(s, Pa, tok, lab, 9 + j, 1e-3, 5e-2, store="bf16", compute="bf16")
        b = zo.step(tok, lab, 9 + j, 1e-3, 5e-2)
        assert tuple(map(float, a)) == tuple(map(float, b))
    zo.flush()
    for n in P:
        assert np.array_equal(Pa[n], Pb[n])
        assert np.array_equal(codec.round_to(Pa[n], "bf16"), Pa[n])
    assert any(not np.array_equal(Pa[n], P[n]) for n in P)


@pytest.mark.parametrize("fmt,scale", [("fp8_e4m3", 64.0), ("fp8_e5m2", 4.0), ("fp8_e4m3", 48.0), ("fp8_e4m3", 0.5)])
def test_scaled_8bit_store_against_torch_cpu_casts(fmt, scale):
    """Sec. 5.5 with a per-tensor scale: the stored code is the 8-bit cast of float32(x s), the value read back is
    float32(code / s).  Pinned against torch's CPU casts on explicitly scaled inputs (in the format's finite range),
    for powers of two - where scaling is exact - and for a scale that is not one; and the stochastic rounding
    lands on one of the two neighbours of the same scaled value."""
    import torch
    from oracle import codec
    tdt = {"fp8_e4m3": torch.float8_e4m3fn, "fp8_e5m2": torch.float8_e5m2}[fmt]
    rng = np.random.default_rng(7)
    x = (rng.standard_normal(20000) * 0.05).astype(np.float32)
    x[:6] = [0.0, -0.0, 1e-9, -3e-7, 0.9, -1.3]
    got = zo_step._store(x, fmt, scale)
    xs = torch.from_numpy(x) * torch.tensor(scale, dtype=torch.float32)          # float32 product
    want = (xs.to(tdt).to(torch.float32) / torch.tensor(scale, dtype=torch.float32)).numpy()
    assert np.array_equal(got, want)
    # the codes are those of the explicitly scaled input, and unscaled storage is the scale-1 case of the same rule
    if np.frexp(scale)[0] == 0.5:                  # a power of two: un-scaling is exact, so the codes can be read back
        assert np.array_equal(codec.round_to(xs.numpy(), fmt), got * np.float32(scale))
    assert np.array_equal(zo_step._store(x, fmt, 1.0), torch.from_numpy(x).to(tdt).to(torch.float32).numpy())
    # a scale really changes what survives: small values flush to zero without it
    tiny = np.full(8, 6e-4, np.float32)
    assert np.all(zo_step._store(tiny, "fp8_e4m3", 1.0) == 0) and np.all(zo_step._store(tiny, "fp8_e4m3", 64.0) != 0)
    # stochastic: one of the two neighbours of float32(x s), divided by s; exact values stay
    r16 = rng.integers(0, 65536, x.size)
    sr = zo_step._store(x, fmt, scale, r16)
    xs64 = xs.numpy().astype(np.float64)
    lo = codec.round_stochastic(xs64, fmt, np.full(x.size, 65536))      # never below the fraction: the lower neighbour
    hi = codec.round_stochastic(xs64, fmt, np.zeros(x.size))
    s32 = np.float32(scale)
    assert np.all((sr == (lo / s32).astype(np.float32)) | (sr == (hi / s32).astype(np.float32)))
    assert np.all(np.abs(lo) <= np.abs(xs64)) and np.all(np.abs(hi) >= np.abs(xs64))
    assert 0.2 < np.mean(sr == (hi / s32).astype(np.float32)) < 0.8


@pytest.mark.parametrize("rounding", ["nearest", "stochastic"])
def test_blockwise_equals_whole_model_with_scaled_8bit_storage(rounding):
    """The deferred, module-by-module form with an 8-bit master and per-tensor scales: same losses as the
    whole-model form at every iteration and - for round-to-nearest, which the whole-model form implements -
    the same stored parameters after the flush; every stored value is a code of the format at its tensor's scale."""
    from oracle import codec
    cfg, s, P, tok, lab = _setup()
    names = [n for n, _, _ in opt_model.tensor_table(s)]
    scales = {n: (64.0 if i % 2 else 16.0) for i, n in enumerate(names)}
    P8 = {n: zo_step._store(P[n], "fp8_e4m3", scales[n]) for n in names}
    Pa, Pb = copy.deepcopy(P8), copy.deepcopy(P8)
    zo = zo_step.Zo2Blockwise(s, Pb, store="fp8_e4m3", compute="bf16", scales=scales, rounding=rounding)
    for j in range(3):
        b = zo.step(tok, lab, 60 + j, 1e-3, 2e-2)
        if rounding == "nearest":
            a = zo_step.step_whole(s, Pa, tok, lab, 60 + j, 1e-3, 2e-2, store="fp8_e4m3", compute="bf16", scales=scales)
            assert tuple(map(float, a)) == tuple(map(float, b)), j
    zo.flush()
    changed = 0
    for n in names:
        sc = np.float32(scales[n])
        assert np.array_equal(codec.round_to(Pb[n] * sc, "fp8_e4m3") / sc, Pb[n]), n
        if rounding == "nearest":
            assert np.array_equal(Pa[n], Pb[n]), n
        changed += int(np.sum(Pb[n] != P8[n]))
    assert changed > 0


def test_stochastic_rounding_lets_a_bf16_master_follow_small_updates():
    """With round-to-nearest a bfloat16 master ignores an update far below half its spacing (the situation at the
    paper's lr = 1e-7); with stochastic rounding the stored parameters follow the float32 trajectory on average."""
    from oracle import codec
    cfg, s, P, tok, lab = _setup()
    P16 = {n: codec.round_to(a, "bf16") for n, a in P.items()}
    runs = {}
    for mode in ("nearest", "stochastic"):
        zo = zo_step.Zo2Blockwise(s, copy.deepcopy(P16), store="bf16", compute="bf16", rounding=mode)
        for j in range(6):
            zo.step(tok, lab, 300 + j, 1e-3, 2e-6)
        zo.flush()
        runs[mode] = zo.P
    ref = zo_step.Zo2Blockwise(s, copy.deepcopy(P16), store="f32", compute="bf16")
    for j in range(6):
        ref.step(tok, lab, 300 + j, 1e-3, 2e-6)
    ref.flush()
    n = "blocks.0.fc1.w"
    moved = ref.P[n] - P16[n]                                   # the float32 master's total displacement
    sp = np.spacing(np.abs(P16[n]).astype(np.float32)).astype(np.float64) * 65536                  # bfloat16 spacing at each element
    assert np.median(np.abs(moved) / sp) < 0.1                  # typical displacement: far below one bf16 step
    d_near = runs["nearest"][n] - P16[n]
    d_sr = runs["stochastic"][n] - P16[n]
    print(np.count_nonzero(d_near), np.count_nonzero(d_sr), d_near.size)
    assert np.count_nonzero(d_near) < 0.03 * d_near.size       # nearest: only elements close to zero (fine spacing) move
    assert np.count_nonzero(d_sr) > 0
    # summed over many elements, the stochastic master's displacement tracks the float32 one (unbiased)
    proj = lambda d: float(np.sum(d.astype(np.float64) * np.sign(moved)))
    print(proj(d_sr), proj(d_near), proj(moved))
    assert abs(proj(d_sr) - proj(moved)) < 0.5 * proj(moved)
    assert proj(d_near) < 0.1 * proj(moved)


# --------------------------------------------------------------------------- q directions per update
def test_one_direction_of_the_multi_form_is_the_plain_step():
    cfg, s, P, tok, lab = _setup()
    Pa, Pb = copy.deepcopy(P), copy.deepcopy(P)
    a = zo_step.step_whole(s, Pa, tok, lab, 42, 1e-3, 1e-3)
    b = zo_step.step_whole_multi(s, Pb, tok, lab, [42], 1e-3, [1e-3])
    assert tuple(map(float, a)) == tuple(map(float, b[0]))
    for n in P:
        assert np.array_equal(Pa[n], Pb[n]), n


@pytest.mark.parametrize("tied", [True, False])
def test_blockwise_with_extra_directions_equals_whole_model(tied):
    """All directions of a round are evaluated at the same parameters (none of the round's own updates is visible
    to them), and the deferred, module-by-module application reproduces the whole-model form bit for bit."""
    cfg, s, P, tok, lab = _setup(tied=tied)
    Pa, Pb = copy.deepcopy(P), copy.deepcopy(P)
    zo = zo_step.Zo2Blockwise(s, Pb)
    for j in range(3):
        seeds = [1000 + 10 * j + i for i in range(3)]
        lrs = [1e-3 * (j + 1) / 3, 2e-3 / 3, 5e-4]             # every direction carries its own eta
        a = zo_step.step_whole_multi(s, Pa, tok, lab, seeds, 1e-3, lrs)
        b = [zo.step(tok, lab, seeds[0], 1e-3, lrs[0])]
        b += [zo.step_extra(tok, lab, seeds[i], 1e-3, lrs[i]) for i in (1, 2)]
        assert [tuple(map(float, x)) for x in a] == [tuple(map(float, x)) for x in b], j
        # the directions of one round see the same parameters: l+ and l- differ only through z
        assert len({float(x[0]) for x in a}) == 3
    zo.flush()
    for n in P:
        assert np.array_equal(Pa[n], Pb[n]), n
    with pytest.raises(ValueError):
        zo_step.Zo2Blockwise(s, copy.deepcopy(P)).step_extra(tok, lab, 1, 1e-3, 1e-3)


def test_average_over_directions_estimates_the_gradient():
    """E[g z] = grad L (Eq. 1-2): the average over q directions has projection (ghat . G) / |G|^2 -> 1 with relative
    spread sqrt(2 / q), and its cosine with G grows like sqrt(q / (q + d)); one direction alone is almost orthogonal."""
    cfg, s, P, tok, lab = _setup()
    for l in range(cfg["n_layers"]):                       # keep L smooth along every direction (see the first test)
        P[f"blocks.{l}.fc1.b"] = P[f"blocks.{l}.fc1.b"] + np.float32(4.0)
    _, G = hf_param_grads(cfg, P, tok, lab)
    gnorm2 = sum(float(np.sum(G[n] ** 2)) for n in P)
    d = sum(P[n].size for n in P)

    def estimate(q, seed0):
        Pq = copy.deepcopy(P)
        eta = 1e-3
        zo_step.step_whole_multi(s, Pq, tok, lab, list(range(seed0, seed0 + q)), 1e-3, [eta / q] * q)
        gh = {n: (P[n].astype(np.float64) - Pq[n].astype(np.float64)) / eta for n in P}
        dot = sum(float(np.sum(gh[n] * G[n])) for n in P)
        return dot / gnorm2, dot / np.sqrt(gnorm2 * sum(float(np.sum(gh[n] ** 2)) for n in P))

    q = 200
    proj, cos = estimate(q, 5000)
    assert abs(proj - 1.0) < 3.5 * np.sqrt(2.0 / q), proj
    assert 0.5 * np.sqrt(q / (q + d)) < cos < 2.0 * np.sqrt(q / (q + d)), (cos, d)
    _, cos1 = estimate(1, 7000)
    assert 0.0 <= cos1 < 0.4 * cos
