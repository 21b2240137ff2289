"""GPU tests of whole steps in which the block projections perturb in their weight loader (steps of few tokens):
against the oracle's Alg. 2, against the sweep-kernel path, streamed against resident, and with the other features
of the step (several directions per update, evaluation in between, stochastic rounding of the stored update)."""
import copy

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import codec, opt_model, zo_step

pytestmark = pytest.mark.gpu


def _b():
    from paper_2503_12668_amd import binding
    return binding


def _tiny(n_layers=4, tied=True):
    cfg = si.tiny_config(n_layers=n_layers, d_model=64, n_heads=4, d_ffn=128, vocab=211, max_pos=40, tied=tied)
    P = si.make_weights(cfg, seed=11, std=0.08, ln_jitter=True)
    tok = si.make_tokens(cfg["vocab"], 3, 23, seed=12)
    lab = si.next_token_labels(tok)
    lab[1, 4] = -100
    return cfg, P, tok, lab


@pytest.mark.parametrize("dt", ["bf16", "f16"])
@pytest.mark.parametrize("tied", [True, False])
def test_fused_loader_steps_track_oracle_and_the_sweep_path(dt, tied):
    b = _b()
    cfg, P, tok, lab = _tiny(tied=tied)
    Po = {n: codec.round_to(a, dt) for n, a in P.items()}
    oz = zo_step.Zo2Blockwise(opt_model.OptShape(**cfg), copy.deepcopy(Po), store=dt, compute=dt)
    fused = b.Zo2Context(cfg, P, wire=dt, compute=dt, arena_bytes=64 << 20)
    fused.set_loader_fusion(1)          # 69 tokens: above the default's 64
    plain = b.Zo2Context(cfg, P, wire=dt, compute=dt, arena_bytes=64 << 20)
    plain.set_loader_fusion(-1)
    for j in range(4):
        a = oz.step(tok, lab, 42 + j, 1e-3, 1e-2)
        f = fused.step(tok, lab, 42 + j, 1e-3, 1e-2)
        p = plain.step(tok, lab, 42 + j, 1e-3, 1e-2)
        for k in (0, 1):
            assert abs(float(f[k]) - float(a[k])) <= 2e-2 * abs(float(a[k])), (j, k)
            # same W+- bit for bit and the same products, added in another order, then rounded to 16 bits per layer
            assert abs(float(f[k]) - float(p[k])) <= (2e-3 if j == 0 else 2e-2) * abs(float(p[k])), (j, k)
    assert fused.plan()["loader_fusion"] and not plain.plan()["loader_fusion"]
    ev_f, ev_p = fused.eval(tok, lab), plain.eval(tok, lab)
    assert abs(float(ev_f) - float(ev_p)) <= 2e-2 * abs(float(ev_p))
    fused.close(); plain.close()


def test_first_step_of_both_paths_is_the_same_update_free_forward():
    """Without a pending update both paths start from identical parameters: the losses differ only by the summation
    order inside the projections (float32) and its effect on 16-bit roundings downstream."""
    b = _b()
    cfg, P, tok, lab = _tiny(n_layers=2)
    res = []
    for mode in (1, -1):
        ctx = b.Zo2Context(cfg, P, wire="bf16", compute="bf16", arena_bytes=64 << 20)
        ctx.set_loader_fusion(mode)
        res.append(ctx.step(tok, lab, 7, 1e-3, 0.0))
        ctx.close()
    assert abs(float(res[0][0]) - float(res[1][0])) <= 1e-3 * abs(float(res[1][0]))
    assert abs(float(res[0][1]) - float(res[1][1])) <= 1e-3 * abs(float(res[1][1]))


@pytest.mark.parametrize("sr", [False, True])
def test_fused_loader_streamed_equals_resident_bitwise(sr):
    b = _b()
    cfg, P, tok, lab = _tiny(n_layers=6)
    runs = {}
    for name in ("resident", "streamed"):
        ctx = b.Zo2Context(cfg, P, wire="bf16", compute="bf16", arena_bytes=64 << 20)
        ctx.set_loader_fusion(1)
        ctx.set_wire_rounding(sr)
        r = [ctx.step(tok, lab, 5, 1e-3, 1e-3)]
        if name == "streamed":
            ctx.set_resident_budget(ctx.plan()["bytes_used"] - 3 * ctx.offs[16] * 2)        # 3 slots for 6 blocks
            ctx.debug_set_slot_poison(True)
        r.append(ctx.step(tok, lab, 6, 1e-3, 1e-3))
        r.append(ctx.step_extra(tok, lab, 7, 1e-3, 5e-4))
        r.append(ctx.step(tok, lab, 8, 1e-3, 1e-3))
        ev = ctx.eval(tok, lab)
        r.append(ctx.step(tok, lab, 9, 1e-3, 1e-3))
        pl = ctx.plan()
        assert pl["loader_fusion"] and pl["resident"] == (name == "resident"), pl
        ctx.flush(); ctx.sync_to_host()
        runs[name] = ([tuple(map(float, x)) for x in r] + [float(ev)], ctx.parameters())
        ctx.close()
    assert runs["streamed"][0] == runs["resident"][0]
    for n in runs["resident"][1]:
        assert np.array_equal(runs["streamed"][1][n], runs["resident"][1][n]), n
    assert all(np.all(np.isfinite(x)) for x in runs["resident"][0])


def test_zero_lr_leaves_parameters_in_the_fused_path():
    b = _b()
    cfg, P, tok, lab = _tiny(n_layers=2)
    ctx = b.Zo2Context(cfg, P, wire="bf16", compute="bf16", arena_bytes=64 << 20)
    ctx.set_loader_fusion(1)
    r1 = ctx.step(tok, lab, 5, 1e-3, 0.0)
    r2 = ctx.step(tok, lab, 5, -1e-3, 0.0)
    assert ctx.plan()["loader_fusion"]
    ctx.flush(); ctx.sync_to_host()
    Pg = ctx.parameters()
    for n in P:
        assert np.array_equal(Pg[n], codec.round_to(P[n], "bf16")), n
    assert float(r1[0]) == float(r2[1]) and float(r1[1]) == float(r2[0]) and float(r1[2]) == float(r2[2])
    ctx.close()


@pytest.mark.timeout(600)
def test_fused_loader_one_block_at_opt1p3b_width_matches_oracle():
    """OPT-1.3B width (d 2048, 32 heads, FFN 8192), one block, batch 1 x 128: two steps (the second with a pending
    update) against the oracle's Alg. 2; bf16 bar.  Vocabulary cut to 4096 entries."""
    b = _b()
    cfg = si.opt_config("opt-1.3b", n_layers=1)
    cfg["vocab"] = 4096
    P = si.make_weights(cfg, seed=1)
    tok = si.make_tokens(cfg["vocab"], 1, 128, seed=2, dist="zipf")
    lab = si.next_token_labels(tok)
    Po = {n: codec.round_to(a, "bf16") for n, a in P.items()}
    oz = zo_step.Zo2Blockwise(opt_model.OptShape(**cfg), Po, store="bf16", compute="bf16")
    ctx = b.Zo2Context(cfg, P, wire="bf16", compute="bf16", arena_bytes=2 << 30)
    ctx.set_loader_fusion(1)
    for j in range(2):
        a = oz.step(tok, lab, 42 + j, 1e-3, 1e-4)
        g = ctx.step(tok, lab, 42 + j, 1e-3, 1e-4)
        print(j, a, g, flush=True)
        assert abs(float(g[0]) - float(a[0])) <= 2e-2 * abs(float(a[0]))
        assert abs(float(g[1]) - float(a[1])) <= 2e-2 * abs(float(a[1]))
    assert ctx.plan()["loader_fusion"]
    ctx.close()


def test_default_takes_the_loader_path_up_to_64_tokens_per_stream():
    b = _b()
    cfg, P, tok, lab = _tiny(n_layers=2)
    ctx = b.Zo2Context(cfg, P, wire="bf16", compute="bf16", arena_bytes=64 << 20)
    for batch, seq, want in ((2, 32, True), (4, 16, True), (3, 23, False), (5, 13, False)):
        t = si.make_tokens(cfg["vocab"], batch, seq, seed=3)
        ctx.step(t, si.next_token_labels(t), 9, 1e-3, 0.0)
        assert ctx.plan()["loader_fusion"] == want, (batch, seq)
    ctx.close()
