"""GPU parity of the single-forward evaluation (zo2_eval) and of the deferred update carried as data
(zo2_get_pending / zo2_set_pending) against the oracle, through the C ABI."""
import copy

import numpy as np
import pytest

import synth_inputs as si
from oracle import codec, opt_model, zo_step

pytestmark = pytest.mark.gpu


def _b():
    from paper_2503_12668_amd import binding
    return binding


def _setup(n_layers=3, tied=True):
    cfg = si.tiny_config(n_layers=n_layers, d_model=64, n_heads=4, d_ffn=136, vocab=211, max_pos=40, tied=tied)
    P = si.make_weights(cfg, seed=11, std=0.08, ln_jitter=True)
    tok = si.make_tokens(cfg["vocab"], 3, 23, seed=12)
    lab = si.next_token_labels(tok)
    lab[1, 4] = -100
    tok2 = si.make_tokens(cfg["vocab"], 3, 23, seed=77)
    lab2 = si.next_token_labels(tok2)
    return cfg, P, tok, lab, tok2, lab2


@pytest.mark.parametrize("tied", [True, False])
def test_eval_matches_oracle_and_training_goes_on(tied):
    b = _b()
    cfg, P, tok, lab, tok2, lab2 = _setup(tied=tied)
    oz = zo_step.Zo2Blockwise(opt_model.OptShape(**cfg), copy.deepcopy(P))
    ctx = b.Zo2Context(cfg, P, arena_bytes=256 << 20)
    # before any step: the loss of the initial parameters
    e_o, e_g = oz.eval_loss(tok2, lab2), ctx.eval(tok2, lab2)
    assert abs(float(e_g) - float(e_o)) <= 1e-5 * abs(float(e_o))
    for j in range(3):
        a, g = oz.step(tok, lab, 42 + j, 1e-3, 1e-4), ctx.step(tok, lab, 42 + j, 1e-3, 1e-4)
        assert abs(float(g[0]) - float(a[0])) <= 1e-5 * abs(float(a[0]))
    assert ctx.pending()[0] and ctx.pending()[1] == 44
    # the evaluation applies the pending update on the way
    e_o, e_g = oz.eval_loss(tok2, lab2), ctx.eval(tok2, lab2)
    print("eval", e_o, e_g)
    assert abs(float(e_g) - float(e_o)) <= 1e-5 * abs(float(e_o))
    assert ctx.pending() == (False, 0, np.float32(0))
    ctx.sync_to_host()
    Pg = ctx.parameters()
    for n in oz.P:
        assert np.abs(Pg[n] - oz.P[n]).max() <= 1e-6, n
    # a second evaluation (nothing pending) gives the same number, and training continues as the oracle's
    assert float(ctx.eval(tok2, lab2)) == float(e_g)
    for j in range(3, 5):
        a, g = oz.step(tok, lab, 42 + j, 1e-3, 1e-4), ctx.step(tok, lab, 42 + j, 1e-3, 1e-4)
        assert abs(float(g[0]) - float(a[0])) <= 1e-5 * abs(float(a[0]))
        assert abs(float(g[1]) - float(a[1])) <= 1e-5 * abs(float(a[1]))
    ctx.close()


@pytest.mark.parametrize("streamed", [False, True])
def test_eval_between_steps_changes_nothing(streamed):
    """Evaluating in the middle of training (resident or streamed) leaves losses and parameters bit-identical."""
    b = _b()
    cfg, P, tok, lab, tok2, lab2 = _setup(n_layers=7)
    runs = []
    for with_eval in (False, True):
        ctx = b.Zo2Context(cfg, P, arena_bytes=64 << 20)
        r = [ctx.step(tok, lab, 5, 1e-3, 1e-3)]
        if streamed:
            ctx.set_resident_budget(ctx.plan()["bytes_used"] - 3 * ctx.offs[16] * 4)
        r.append(ctx.step(tok, lab, 6, 1e-3, 1e-3))
        if with_eval:
            ev = ctx.eval(tok2, lab2)
            st = ctx.step_stats()
            if streamed:      # a pending update was applied: every block came up and went back once
                assert not ctx.plan()["resident"]
                assert st["bytes_up"] == 7 * ctx.offs[16] * 4 and st["bytes_down"] == 7 * ctx.offs[16] * 4
            ev2 = ctx.eval(tok2, lab2)
            assert float(ev) == float(ev2)
            if streamed:      # nothing pending any more: blocks are only read
                st = ctx.step_stats()
                assert st["bytes_up"] == 7 * ctx.offs[16] * 4 and st["bytes_down"] == 0
        r += [ctx.step(tok, lab, 7 + j, 1e-3, 1e-3) for j in range(2)]
        ctx.flush(); ctx.sync_to_host()
        runs.append((r, ctx.parameters(), ev if with_eval else None))
        ctx.close()
    assert [tuple(map(float, x)) for x in runs[0][0]] == [tuple(map(float, x)) for x in runs[1][0]]
    for n in runs[0][1]:
        assert np.array_equal(runs[0][1][n], runs[1][1][n]), n


def test_eval_streamed_equals_resident_bitwise():
    b = _b()
    cfg, P, tok, lab, tok2, lab2 = _setup(n_layers=7)
    vals = []
    for streamed in (False, True):
        ctx = b.Zo2Context(cfg, P, arena_bytes=64 << 20)
        ctx.step(tok, lab, 5, 1e-3, 1e-3)
        if streamed:
            ctx.set_resident_budget(ctx.plan()["bytes_used"] - 4 * ctx.offs[16] * 4)
        ctx.step(tok, lab, 6, 1e-3, 1e-3)
        vals.append(float(ctx.eval(tok2, lab2)))
        ctx.close()
    assert vals[0] == vals[1]


@pytest.mark.parametrize("wire,compute", [("bf16", "bf16"), ("f16", "f16")])
def test_eval_low_precision_tracks_oracle(wire, compute):
    b = _b()
    cfg, P, tok, lab, tok2, lab2 = _setup()
    Po = {n: codec.round_to(a, wire) for n, a in copy.deepcopy(P).items()}
    oz = zo_step.Zo2Blockwise(opt_model.OptShape(**cfg), Po, store=wire, compute=compute)
    ctx = b.Zo2Context(cfg, P, wire=wire, compute=compute, arena_bytes=256 << 20)
    for j in range(2):
        oz.step(tok, lab, 42 + j, 1e-3, 5e-3); ctx.step(tok, lab, 42 + j, 1e-3, 5e-3)
    e_o, e_g = oz.eval_loss(tok2, lab2), ctx.eval(tok2, lab2)
    assert abs(float(e_g) - float(e_o)) <= 2e-2 * abs(float(e_o))
    ctx.close()


def test_checkpoint_resume_is_bit_identical():
    """Parameters in the host buffers plus (seed, eta * g) of the deferred update are the whole state (Sec. 5.4):
    a fresh context given both continues exactly where the first one stood."""
    b = _b()
    cfg, P, tok, lab, _, _ = _setup()
    ctx_a = b.Zo2Context(cfg, P, arena_bytes=64 << 20)
    ra = [ctx_a.step(tok, lab, 42 + j, 1e-3, 1e-3 * (j + 1)) for j in range(5)]
    ctx_a.flush(); ctx_a.sync_to_host()
    Pa = ctx_a.parameters()
    ctx_a.close()

    ctx_b = b.Zo2Context(cfg, P, arena_bytes=64 << 20)
    rb = [ctx_b.step(tok, lab, 42 + j, 1e-3, 1e-3 * (j + 1)) for j in range(3)]
    ctx_b.sync_to_host()                      # does not flush: the update of step 3 is still pending
    saved = copy.deepcopy(ctx_b.parameters())
    has, seed, step = ctx_b.pending()
    assert has and seed == 44 and float(step) == float(np.float32(np.float32(3e-3) * rb[2][2]))
    ctx_b.close()

    ctx_c = b.Zo2Context(cfg, saved, arena_bytes=64 << 20)
    assert ctx_c.pending()[0] is False
    ctx_c.set_pending(has, seed, step)
    rc = [ctx_c.step(tok, lab, 42 + j, 1e-3, 1e-3 * (j + 1)) for j in range(3, 5)]
    ctx_c.flush(); ctx_c.sync_to_host()
    Pc = ctx_c.parameters()
    ctx_c.close()
    assert [tuple(map(float, x)) for x in ra] == [tuple(map(float, x)) for x in rb + rc]
    for n in Pa:
        assert np.array_equal(Pa[n], Pc[n]), n
    # dropping the saved update instead changes the result
    ctx_d = b.Zo2Context(cfg, saved, arena_bytes=64 << 20)
    rd = ctx_d.step(tok, lab, 45, 1e-3, 4e-3)
    assert float(rd[0]) != float(ra[3][0])
    with pytest.raises(b.Zo2Error):
        ctx_d.set_pending(True, 1, float("nan"))
    ctx_d.close()


def test_ablation_switches_change_time_not_results():
    """Table 4's reverse ablation as switches: no stream overlap (zo2_set_stream_overlap(0)) and no deferred update
    (zo2_flush after every step) leave every loss and parameter bit-identical."""
    b = _b()
    cfg, P, tok, lab, _, _ = _setup(n_layers=7)
    runs = []
    for mode in ("full", "serial", "flush_each_step"):
        ctx = b.Zo2Context(cfg, P, arena_bytes=64 << 20)
        r = [ctx.step(tok, lab, 5, 1e-3, 1e-3)]
        ctx.set_resident_budget(ctx.plan()["bytes_used"] - 4 * ctx.offs[16] * 4)      # 3 slots for 7 blocks
        if mode == "serial":
            ctx.set_stream_overlap(False)
        for j in range(1, 4):
            if mode == "flush_each_step":
                ctx.flush()
            r.append(ctx.step(tok, lab, 5 + j, 1e-3, 1e-3))
        assert not ctx.plan()["resident"]
        ctx.flush(); ctx.sync_to_host()
        runs.append((r, ctx.parameters()))
        ctx.close()
    for other in runs[1:]:
        assert [tuple(map(float, x)) for x in runs[0][0]] == [tuple(map(float, x)) for x in other[0]]
        for n in runs[0][1]:
            assert np.array_equal(runs[0][1][n], other[1][n]), n
