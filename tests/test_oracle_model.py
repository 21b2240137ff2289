"""Pins for the oracle's loss L(theta; B) (run without a GPU)."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import opt_model

from hf_reference import build_hf_opt


def _shape(cfg):
    return opt_model.OptShape(**cfg)


@pytest.mark.parametrize("tied", [True, False])
def test_logits_match_independent_opt(tied):
    """Layout conventions (q scaling, position offset, pre-LN order, ReLU FFN, weight
    tying, [out, in] matrices) against the transformers library's OPT module."""
    cfg = si.tiny_config(n_layers=2, d_model=48, n_heads=4, d_ffn=80, vocab=131, max_pos=20, tied=tied)
    P = si.make_weights(cfg, seed=5, std=0.2, ln_jitter=True)
    tok = si.make_tokens(cfg["vocab"], 3, 17, seed=6)
    ours = opt_model.logits(_shape(cfg), P, tok).numpy()
    with torch.no_grad():
        ref = build_hf_opt(cfg, P)(input_ids=torch.from_numpy(tok.astype(np.int64))).logits.numpy()
    assert ours.shape == ref.shape == (3, 17, 131)
    # the library's eager attention evaluates its softmax in float32 even for a float64
    # module, so agreement stops near 1e-7; a convention mistake would show at O(1)
    assert np.abs(ours - ref).max() < 3e-6 * max(1.0, np.abs(ref).max())
    assert np.abs(ours[:, 0] - ref[:, 0]).max() < 1e-12      # position 0: softmax over one key


def test_loss_matches_torch_cross_entropy_with_ignored_labels():
    cfg = si.tiny_config()
    P = si.make_weights(cfg, seed=1, std=0.3, ln_jitter=True)
    tok = si.make_tokens(cfg["vocab"], 2, 9, seed=3)
    lab = si.next_token_labels(tok)
    lab[0, 3] = -100
    s = _shape(cfg)
    lg = opt_model.logits(s, P, tok)
    ref = torch.nn.functional.cross_entropy(lg.reshape(-1, cfg["vocab"]),
                                            torch.from_numpy(lab.astype(np.int64)).reshape(-1),
                                            ignore_index=-100)
    assert abs(opt_model.loss(s, P, tok, lab) - float(ref)) < 1e-12


def test_causality():
    """Changing token t leaves the logits at positions < t unchanged."""
    cfg = si.tiny_config()
    P = si.make_weights(cfg, seed=1, std=0.3, ln_jitter=True)
    tok = si.make_tokens(cfg["vocab"], 1, 12, seed=3)
    s = _shape(cfg)
    a = opt_model.logits(s, P, tok).numpy()
    tok2 = tok.copy()
    tok2[0, 7] = (tok2[0, 7] + 1) % cfg["vocab"]
    b = opt_model.logits(s, P, tok2).numpy()
    assert np.array_equal(a[0, :7], b[0, :7])
    assert not np.allclose(a[0, 7:], b[0, 7:])


def test_loss_at_small_init_is_log_vocab():
    """With N(0, 0.02) weights the logits are nearly uniform: loss ~ ln(vocab)."""
    cfg = si.tiny_config(n_layers=2, d_model=64, n_heads=4, d_ffn=128, vocab=5003, max_pos=40)
    P = si.make_weights(cfg, seed=1)
    tok = si.make_tokens(cfg["vocab"], 2, 32, seed=2)
    l = opt_model.loss(_shape(cfg), P, tok, si.next_token_labels(tok))
    assert abs(l - math.log(5003)) < 0.05


def test_opt_family_parameter_counts():
    """Table 1's shapes with a tied LM head reproduce the nominal model sizes."""
    nominal = {"opt-125m": 125e6, "opt-1.3b": 1.3e9, "opt-2.7b": 2.7e9, "opt-6.7b": 6.7e9,
               "opt-13b": 13e9, "opt-30b": 30e9, "opt-66b": 66e9, "opt-175b": 175e9}
    for name, n in nominal.items():
        cnt = opt_model.n_params(_shape(si.opt_config(name)))
        assert abs(cnt - n) / n < 0.03, (name, cnt)


def test_tensor_table_matches_generator():
    cfg = si.tiny_config(tied=False)
    names = [(n, shp) for n, _, shp in opt_model.tensor_table(_shape(cfg))]
    assert names == si.tensor_names_and_shapes(cfg)
    ids = [tid for _, tid, _ in opt_model.tensor_table(_shape(cfg))]
    assert ids == list(range(len(ids)))
