"""Oracle (test infrastructure): the loss L(theta; B) of an OPT-shaped decoder.

The paper's model is "an embedding layer, N transformer blocks and an LM head"
(Sec. 4.2), instantiated on the OPT family (Table 1).  OPT-shaped means:
learned token + position embeddings (position table offset by 2), pre-LayerNorm
blocks with multi-head causal self-attention and a ReLU FFN, a final LayerNorm
and an LM head tied to the token embedding unless stated otherwise.

Everything is evaluated in float64 from the given parameter values; no blocking,
no fusion.  torch CPU is used only as the matmul / softmax library.
"""
import math
from dataclasses import dataclass

import numpy as np
import torch

BLOCK_TENSORS = ("ln1.w", "ln1.b", "q.w", "q.b", "k.w", "k.b", "v.w", "v.b",
                 "o.w", "o.b", "ln2.w", "ln2.b", "fc1.w", "fc1.b", "fc2.w", "fc2.b")


@dataclass(frozen=True)
class OptShape:
    n_layers: int
    d_model: int
    n_heads: int
    d_ffn: int
    vocab: int
    max_pos: int
    pos_offset: int = 2
    tied: bool = True
    ln_eps: float = 1e-5


def _block_shape(s, t):
    d, f = s.d_model, s.d_ffn
    return {"ln1.w": (d,), "ln1.b": (d,), "q.w": (d, d), "q.b": (d,), "k.w": (d, d), "k.b": (d,),
            "v.w": (d, d), "v.b": (d,), "o.w": (d, d), "o.b": (d,), "ln2.w": (d,), "ln2.b": (d,),
            "fc1.w": (f, d), "fc1.b": (f,), "fc2.w": (d, f), "fc2.b": (d,)}[t]


def tensor_table(s):
    """Every parameter tensor in the fixed order that also numbers them for the
    random stream: (name, tensor_id, shape).  Module order follows Alg. 2:
    Embedding, W_1..W_N, LM head."""
    out = [("tok_emb", 0, (s.vocab, s.d_model)),
           ("pos_emb", 1, (s.max_pos + s.pos_offset, s.d_model))]
    tid = 2
    for l in range(s.n_layers):
        for t in BLOCK_TENSORS:
            out.append((f"blocks.{l}.{t}", tid, _block_shape(s, t)))
            tid += 1
    out.append(("final_ln.w", tid, (s.d_model,)))
    out.append(("final_ln.b", tid + 1, (s.d_model,)))
    if not s.tied:
        out.append(("lm_head.w", tid + 2, (s.vocab, s.d_model)))
    return out


def modules(s):
    """The tensor names grouped into the modules Alg. 2 walks over."""
    mods = [["tok_emb", "pos_emb"]]
    for l in range(s.n_layers):
        mods.append([f"blocks.{l}.{t}" for t in BLOCK_TENSORS])
    head = ["final_ln.w", "final_ln.b"] + ([] if s.tied else ["lm_head.w"])
    mods.append(head)
    return mods


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float64)


def layer_norm(x, w, b, eps):
    """(x - mean) / sqrt(var + eps) * w + b over the last axis, biased variance."""
    mu = x.mean(dim=-1, keepdim=True)
    var = ((x - mu) ** 2).mean(dim=-1, keepdim=True)      # biased variance
    return (x - mu) / torch.sqrt(var + eps) * w + b


def linear(x, w, b=None):
    """y = x w^T + b for a weight stored [out_features, in_features]."""
    y = x @ w.T
    return y if b is None else y + b


def causal_attention(q, k, v, n_heads):
    """softmax_{j <= i}(q_i . k_j) v_j per head; q, k, v [B, S, d] with head h in columns h d_h .. (h+1) d_h - 1;
    q already carries the 1 / sqrt(d_h) factor."""
    B, S, d = q.shape
    dh = d // n_heads
    q = q.view(B, S, n_heads, dh).transpose(1, 2)
    k = k.view(B, S, n_heads, dh).transpose(1, 2)
    v = v.view(B, S, n_heads, dh).transpose(1, 2)
    sc = q @ k.transpose(-1, -2)                           # [B, H, S, S]
    future = torch.triu(torch.ones(S, S, dtype=torch.bool), diagonal=1)
    sc = sc.masked_fill(future, float("-inf"))
    p = torch.softmax(sc, dim=-1)
    return (p @ v).transpose(1, 2).reshape(B, S, d)


def embed(s, P, tokens):
    """h0[b, t] = tok_emb[id] + pos_emb[t + pos_offset]."""
    ids = torch.from_numpy(np.asarray(tokens, dtype=np.int64))
    B, S = ids.shape
    pos = torch.arange(S) + s.pos_offset
    return _t(P["tok_emb"])[ids] + _t(P["pos_emb"])[pos][None, :, :]


def block_forward(s, P, l, h):
    """One pre-LN decoder block on h [B, S, d]."""
    g = lambda t: _t(P[f"blocks.{l}.{t}"])
    dh = s.d_model // s.n_heads
    x = layer_norm(h, g("ln1.w"), g("ln1.b"), s.ln_eps)
    q = linear(x, g("q.w"), g("q.b")) * dh ** -0.5
    k = linear(x, g("k.w"), g("k.b"))
    v = linear(x, g("v.w"), g("v.b"))
    ctx = causal_attention(q, k, v, s.n_heads)
    h = h + linear(ctx, g("o.w"), g("o.b"))
    x = layer_norm(h, g("ln2.w"), g("ln2.b"), s.ln_eps)
    y = torch.relu(linear(x, g("fc1.w"), g("fc1.b")))
    return h + linear(y, g("fc2.w"), g("fc2.b"))


def head_logits(s, P, h):
    x = layer_norm(h, _t(P["final_ln.w"]), _t(P["final_ln.b"]), s.ln_eps)
    return linear(x, _t(P["tok_emb"] if s.tied else P["lm_head.w"]))


def row_cross_entropy(logits, labels):
    """Per position: logsumexp(logits) - logits[label]; 0 where the label is -100.  logits [rows, vocab]."""
    lab = torch.from_numpy(np.asarray(labels, dtype=np.int64)).reshape(-1)
    keep = lab != -100
    lse = torch.logsumexp(logits, dim=-1)
    picked = logits.gather(1, lab.clamp(min=0)[:, None])[:, 0]
    return torch.where(keep, lse - picked, torch.zeros_like(lse))


def cross_entropy(logits, labels):
    """Mean over positions whose label is not -100 of logsumexp(logits) - logits[label]."""
    lab = torch.from_numpy(np.asarray(labels, dtype=np.int64)).reshape(-1)
    rows = row_cross_entropy(logits.reshape(-1, logits.shape[-1]), lab)
    return float(rows.sum() / int((lab != -100).sum()))


def logits(s, P, tokens):
    h = embed(s, P, tokens)
    for l in range(s.n_layers):
        h = block_forward(s, P, l, h)
    return head_logits(s, P, h)


def loss(s, P, tokens, labels):
    """L(theta; B) as a python float (float64)."""
    return cross_entropy(logits(s, P, tokens), labels)


def n_params(s):
    return sum(int(np.prod(shape)) for _, _, shape in tensor_table(s))
