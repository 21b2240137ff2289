"""An independently written OPT decoder (the `transformers` library's, randomly
initialised from a config, nothing downloaded) loaded with given weights; float64
on the CPU.  Used only to pin the oracle's model conventions and, through
autograd, its projected gradient."""
import numpy as np
import torch


def build_hf_opt(cfg, P):
    from transformers import OPTConfig, OPTForCausalLM
    hc = OPTConfig(vocab_size=cfg["vocab"], hidden_size=cfg["d_model"], num_hidden_layers=cfg["n_layers"],
                   ffn_dim=cfg["d_ffn"], num_attention_heads=cfg["n_heads"],
                   max_position_embeddings=cfg["max_pos"], do_layer_norm_before=True,
                   word_embed_proj_dim=cfg["d_model"], activation_function="relu", dropout=0.0,
                   attention_dropout=0.0, layerdrop=0.0, tie_word_embeddings=bool(cfg["tied"]),
                   enable_bias=True, layer_norm_elementwise_affine=True,
                   pad_token_id=None)      # no padding row: every embedding row gets its gradient
    hc._attn_implementation = "eager"
    m = OPTForCausalLM(hc).to(torch.float64).eval()
    sd = {}
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    sd["model.decoder.embed_tokens.weight"] = t(P["tok_emb"])
    sd["model.decoder.embed_positions.weight"] = t(P["pos_emb"])
    hfname = {"ln1": "self_attn_layer_norm", "q": "self_attn.q_proj", "k": "self_attn.k_proj",
              "v": "self_attn.v_proj", "o": "self_attn.out_proj", "ln2": "final_layer_norm",
              "fc1": "fc1", "fc2": "fc2"}
    for l in range(cfg["n_layers"]):
        for k, hn in hfname.items():
            sd[f"model.decoder.layers.{l}.{hn}.weight"] = t(P[f"blocks.{l}.{k}.w"])
            sd[f"model.decoder.layers.{l}.{hn}.bias"] = t(P[f"blocks.{l}.{k}.b"])
    sd["model.decoder.final_layer_norm.weight"] = t(P["final_ln.w"])
    sd["model.decoder.final_layer_norm.bias"] = t(P["final_ln.b"])
    sd["lm_head.weight"] = t(P["tok_emb"] if cfg["tied"] else P["lm_head.w"])
    missing, unexpected = m.load_state_dict(sd, strict=False)
    assert not unexpected, unexpected
    assert all("lm_head" in k for k in missing), missing
    return m


def hf_param_grads(cfg, P, tokens, labels):
    """Loss and dL/dtheta (name -> float64 array) by autograd through the HF module."""
    m = build_hf_opt(cfg, P)
    ids = torch.from_numpy(np.asarray(tokens, dtype=np.int64))
    lab = torch.from_numpy(np.asarray(labels, dtype=np.int64))
    logits = m(input_ids=ids).logits
    loss = torch.nn.functional.cross_entropy(logits.reshape(-1, logits.shape[-1]), lab.reshape(-1),
                                             ignore_index=-100)
    loss.backward()
    sd = dict(m.named_parameters())
    g = {}
    hfname = {"ln1": "self_attn_layer_norm", "q": "self_attn.q_proj", "k": "self_attn.k_proj",
              "v": "self_attn.v_proj", "o": "self_attn.out_proj", "ln2": "final_layer_norm",
              "fc1": "fc1", "fc2": "fc2"}
    g["tok_emb"] = sd["model.decoder.embed_tokens.weight"].grad.numpy()
    g["pos_emb"] = sd["model.decoder.embed_positions.weight"].grad.numpy()
    for l in range(cfg["n_layers"]):
        for k, hn in hfname.items():
            g[f"blocks.{l}.{k}.w"] = sd[f"model.decoder.layers.{l}.{hn}.weight"].grad.numpy()
            g[f"blocks.{l}.{k}.b"] = sd[f"model.decoder.layers.{l}.{hn}.bias"].grad.numpy()
    g["final_ln.w"] = sd["model.decoder.final_layer_norm.weight"].grad.numpy()
    g["final_ln.b"] = sd["model.decoder.final_layer_norm.bias"].grad.numpy()
    if not cfg["tied"]:
        g["lm_head.w"] = sd["lm_head.weight"].grad.numpy()
    return float(loss.detach()), g
