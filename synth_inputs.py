"""Seeded synthetic inputs: decoder weights, token batches, labels.

Serves both the CPU oracle's tests and the HIP library's tests / bench so that
the two sides see identical inputs.  Holds no arithmetic of the method itself:
only shapes, names and random draws (numpy's own generators).

The paper measures on SST-2 text with released OPT checkpoints; neither is
available offline, and throughput does not depend on the values, so weights are
N(0, 0.02) draws and token ids are uniform or Zipf(1.1)-distributed over the
vocabulary (a stand-in for the skew of natural text).
"""
import numpy as np

BLOCK_TENSORS = ("ln1.w", "ln1.b", "q.w", "q.b", "k.w", "k.b", "v.w", "v.b",
                 "o.w", "o.b", "ln2.w", "ln2.b", "fc1.w", "fc1.b", "fc2.w", "fc2.b")

# name: (layers, d_model, heads, d_ffn); vocab 50272, max_pos 2048, pos_offset 2 (OPT family, Table 1)
OPT_FAMILY = {
    "opt-125m": (12, 768, 12, 3072),
    "opt-1.3b": (24, 2048, 32, 8192),
    "opt-2.7b": (32, 2560, 32, 10240),
    "opt-6.7b": (32, 4096, 32, 16384),
    "opt-13b": (40, 5120, 40, 20480),
    "opt-30b": (48, 7168, 56, 28672),
    "opt-66b": (64, 9216, 72, 36864),
    "opt-175b": (96, 12288, 96, 49152),
}


def opt_config(name, n_layers=None):
    L, d, h, f = OPT_FAMILY[name]
    return dict(n_layers=L if n_layers is None else n_layers, d_model=d, n_heads=h, d_ffn=f,
                vocab=50272, max_pos=2048, pos_offset=2, tied=True, ln_eps=1e-5)


def tiny_config(n_layers=2, d_model=32, n_heads=4, d_ffn=64, vocab=97, max_pos=24, tied=True):
    return dict(n_layers=n_layers, d_model=d_model, n_heads=n_heads, d_ffn=d_ffn, vocab=vocab,
                max_pos=max_pos, pos_offset=2, tied=tied, ln_eps=1e-5)


def block_tensor_shape(cfg, t):
    d, f = cfg["d_model"], cfg["d_ffn"]
    if t in ("q.w", "k.w", "v.w", "o.w"):
        return (d, d)
    if t == "fc1.w":
        return (f, d)
    if t == "fc2.w":
        return (d, f)
    if t == "fc1.b":
        return (f,)
    return (d,)


def tensor_names_and_shapes(cfg):
    out = [("tok_emb", (cfg["vocab"], cfg["d_model"])),
           ("pos_emb", (cfg["max_pos"] + cfg["pos_offset"], cfg["d_model"]))]
    for l in range(cfg["n_layers"]):
        for t in BLOCK_TENSORS:
            out.append((f"blocks.{l}.{t}", block_tensor_shape(cfg, t)))
    out.append(("final_ln.w", (cfg["d_model"],)))
    out.append(("final_ln.b", (cfg["d_model"],)))
    if not cfg["tied"]:
        out.append(("lm_head.w", (cfg["vocab"], cfg["d_model"])))
    return out


def make_weights(cfg, seed=1, std=0.02, ln_jitter=False):
    """name -> float32 array.  Matrices, embeddings and biases ~ N(0, std);
    LayerNorm gain 1 and bias 0 (with ln_jitter: 1 + N(0, std) and N(0, std),
    which makes a swapped or dropped LayerNorm parameter visible in tests)."""
    rng = np.random.Generator(np.random.Philox(seed))
    P = {}
    for name, shp in tensor_names_and_shapes(cfg):
        is_ln = ".ln" in name or name.startswith("final_ln")
        if is_ln and not ln_jitter:
            P[name] = np.ones(shp, np.float32) if name.endswith(".w") else np.zeros(shp, np.float32)
        else:
            a = rng.standard_normal(shp, dtype=np.float32) * np.float32(std)
            if is_ln and name.endswith(".w"):
                a = a + np.float32(1.0)
            P[name] = a.astype(np.float32)
    return P


def make_tokens(vocab, batch, seq, seed=2, dist="uniform", zipf_a=1.1):
    """int32 token ids [batch, seq].  "zipf": P(id = r-1) proportional to r^-a, r = 1..vocab."""
    rng = np.random.Generator(np.random.Philox(seed))
    if dist == "uniform":
        return rng.integers(0, vocab, size=(batch, seq), dtype=np.int64).astype(np.int32)
    if dist == "zipf":
        w = np.arange(1, vocab + 1, dtype=np.float64) ** (-zipf_a)
        cdf = np.cumsum(w) / w.sum()
        u = rng.random((batch, seq))
        return np.minimum(np.searchsorted(cdf, u, side="left"), vocab - 1).astype(np.int32)
    raise ValueError(dist)


def next_token_labels(tokens):
    """labels[b, t] = tokens[b, t+1]; the last position has no target (-100)."""
    lab = np.full_like(tokens, -100)
    lab[:, :-1] = tokens[:, 1:]
    return lab
