"""GPU tests of zo2_step_multi: a whole round of directions in one pass over the model.  Its results and the state it
leaves must equal those of zo2_step + zo2_step_extra (which the other tests hold against the oracle) bit for bit, on
every path of the step: resident and streamed, sweep copies and perturbation in the weight loader, per-group scratch,
stochastic rounding of the stored update, 8-bit wire format, write-back interval; plus one direct comparison with the
oracle's q-direction estimator."""
import copy

import numpy as np
import pytest

import synth_inputs as si
from oracle import opt_model, zo_step

pytestmark = pytest.mark.gpu


def _b():
    from paper_2503_12668_amd import binding
    return binding


def _case(n_layers=5, tied=True, batch=3, seq=23, d_ffn=136):
    cfg = si.tiny_config(n_layers=n_layers, d_model=64, n_heads=4, d_ffn=d_ffn, vocab=211, max_pos=80, tied=tied)
    P = si.make_weights(cfg, seed=11, std=0.08, ln_jitter=True)
    tok = si.make_tokens(cfg["vocab"], batch, seq, seed=12)
    lab = si.next_token_labels(tok)
    lab[1, 4] = -100
    return cfg, P, tok, lab


def _sequential_round(ctx, tok, lab, seeds, eps, lr):
    out = [ctx.step(tok, lab, seeds[0], eps, lr)]
    out += [ctx.step_extra(tok, lab, s, eps, lr) for s in seeds[1:]]
    return [tuple(float(v) for v in r) for r in out]


def _multi_round(ctx, tok, lab, seeds, eps, lr):
    return [tuple(float(v) for v in r) for r in ctx.step_multi(tok, lab, seeds, eps, lr)]


def _run(b, cfg, P, tok, lab, multi, wire, compute, streamed, sr=False, fusion=0, sweeps=0, interval=1):
    ctx = b.Zo2Context(cfg, P, wire=wire, compute=compute, arena_bytes=96 << 20)
    ctx.set_wire_rounding(sr)
    ctx.set_loader_fusion(fusion)
    rnd = _multi_round if multi else _sequential_round
    out = [rnd(ctx, tok, lab, [7, 8, 9], 1e-3, 1e-4)]                    # first round: resident, nothing pending
    if streamed:
        esz = b.lib().zo2_dtype_size(ctx.wire_id)
        # 3 or 4 slots for 5 blocks (the slack pays for the residual streams of the further directions)
        ctx.set_resident_budget(ctx.plan()["bytes_used"] - 2 * ctx.offs[16] * esz + 40_000)
        ctx.debug_set_slot_poison(True)
        ctx.set_writeback_interval(interval)
    if sweeps:
        ctx.set_scratch_plan(sweeps)
    out.append(rnd(ctx, tok, lab, [20, 21], 1e-3, 1e-4))
    out.append(rnd(ctx, tok, lab, [30, 31, 32, 33], 1e-3, 5e-5))
    out.append([tuple(float(v) for v in ctx.step(tok, lab, 40, 1e-3, 1e-4))])   # an ordinary step applies the round of four
    out.append(rnd(ctx, tok, lab, [50, 51], 1e-3, 1e-4))
    ev = float(ctx.eval(tok, lab))
    out.append(rnd(ctx, tok, lab, [60, 61, 62], 1e-3, 1e-4))
    pend = ctx.pending_list()
    pl = ctx.plan()
    assert pl["resident"] == (not streamed), pl
    ctx.flush(); ctx.sync_to_host()
    res = (out, ev, [(int(s), float(c)) for s, c in pend], ctx.parameters())
    ctx.close()
    return res


def _same(a, b):
    assert a[0] == b[0]
    assert a[1] == b[1]
    assert a[2] == b[2] and len(a[2]) == 3
    for n in a[3]:
        assert np.array_equal(a[3][n], b[3][n]), n
    assert all(np.isfinite(v) for rnd in a[0] for r in rnd for v in r)


@pytest.mark.parametrize("wire,compute,sr", [("f32", "f32", False), ("bf16", "bf16", False), ("bf16", "bf16", True), ("fp8_e4m3", "bf16", True)])
@pytest.mark.parametrize("streamed", [False, True])
def test_one_pass_rounds_equal_sequential_rounds_bitwise(wire, compute, sr, streamed):
    b = _b()
    cfg, P, tok, lab = _case()
    one = _run(b, cfg, P, tok, lab, True, wire, compute, streamed, sr=sr, fusion=-1)
    seq = _run(b, cfg, P, tok, lab, False, wire, compute, streamed, sr=sr, fusion=-1)
    _same(one, seq)


@pytest.mark.parametrize("streamed,interval", [(False, 1), (True, 1), (True, 3)])
def test_one_pass_rounds_with_the_perturbation_in_the_weight_loader(streamed, interval):
    b = _b()
    cfg, P, tok, lab = _case(d_ffn=128)
    one = _run(b, cfg, P, tok, lab, True, "bf16", "bf16", streamed, fusion=1, interval=interval)
    seq = _run(b, cfg, P, tok, lab, False, "bf16", "bf16", streamed, fusion=1, interval=interval)
    _same(one, seq)


@pytest.mark.parametrize("sweeps,interval", [(2, 1), (4, 1), (1, 4)])
def test_one_pass_rounds_streamed_with_per_group_scratch_and_write_back_interval(sweeps, interval):
    b = _b()
    cfg, P, tok, lab = _case()
    one = _run(b, cfg, P, tok, lab, True, "bf16", "bf16", True, fusion=-1, sweeps=sweeps, interval=interval)
    seq = _run(b, cfg, P, tok, lab, False, "bf16", "bf16", True, fusion=-1, sweeps=sweeps, interval=interval)
    res = _run(b, cfg, P, tok, lab, True, "bf16", "bf16", False, fusion=-1)
    _same(one, seq)
    _same(one, res)


def test_one_pass_round_uploads_each_block_once():
    b = _b()
    cfg, P, tok, lab = _case(n_layers=7)
    ctx = b.Zo2Context(cfg, P, arena_bytes=96 << 20)
    ctx.step(tok, lab, 5, 1e-3, 1e-4)
    bucket = ctx.offs[16] * 4
    ctx.set_resident_budget(ctx.plan()["bytes_used"] - 3 * bucket)
    r = ctx.step_multi(tok, lab, [1, 2, 3, 4], 1e-3, 1e-4)
    st = ctx.step_stats()
    assert not ctx.plan()["resident"] and len(r) == 4
    assert st["bytes_up"] == 7 * bucket and st["bytes_down"] == 7 * bucket      # the pending update of step 5 went back
    r = ctx.step_multi(tok, lab, [11, 12], 1e-3, 1e-4)
    st = ctx.step_stats()
    assert st["bytes_up"] == 7 * bucket and st["bytes_down"] == 7 * bucket
    assert [s for s, _ in ctx.pending_list()] == [11, 12]
    ctx.close()


@pytest.mark.parametrize("tied", [True, False])
def test_fp32_one_pass_rounds_match_oracle(tied):
    b = _b()
    cfg, P, tok, lab = _case(n_layers=3, tied=tied)
    oz = zo_step.Zo2Blockwise(opt_model.OptShape(**cfg), copy.deepcopy(P))
    ctx = b.Zo2Context(cfg, P, arena_bytes=256 << 20)
    q = 3
    for j in range(3):
        seeds = [500 + 10 * j + i for i in range(q)]
        ro = [oz.step(tok, lab, seeds[0], 1e-3, 1e-4)] + [oz.step_extra(tok, lab, s, 1e-3, 1e-4) for s in seeds[1:]]
        rg = ctx.step_multi(tok, lab, seeds, 1e-3, 1e-4)
        for a, g in zip(ro, rg):
            assert abs(float(g[0]) - float(a[0])) <= 1e-5 * abs(float(a[0]))
            assert abs(float(g[1]) - float(a[1])) <= 1e-5 * abs(float(a[1]))
            assert abs(float(g[2]) - float(a[2])) <= 1e-5 * abs(float(a[0])) / 1e-3
    oz.flush(); ctx.flush(); ctx.sync_to_host()
    Pg = ctx.parameters()
    for n in oz.P:
        assert np.abs(Pg[n] - oz.P[n]).max() <= 1e-6, n
    ctx.close()


def test_step_multi_rejects_bad_arguments_and_one_direction_is_a_step():
    b = _b()
    cfg, P, tok, lab = _case(n_layers=2)
    ctx = b.Zo2Context(cfg, P, arena_bytes=64 << 20)
    ref = b.Zo2Context(cfg, P, arena_bytes=64 << 20)
    with pytest.raises(b.Zo2Error):
        ctx.step_multi(tok, lab, [], 1e-3, 1e-4)
    with pytest.raises(b.Zo2Error):
        ctx.step_multi(tok, lab, list(range(17)), 1e-3, 1e-4)
    with pytest.raises(b.Zo2Error):
        ctx.step_multi(tok, lab, [1, 2], 0.0, 1e-4)
    for j in range(3):
        a = ctx.step_multi(tok, lab, [70 + j], 1e-3, 1e-4)[0]
        r = ref.step(tok, lab, 70 + j, 1e-3, 1e-4)
        assert tuple(map(float, a)) == tuple(map(float, r))
    ctx.close(); ref.close()
