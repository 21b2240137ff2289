"""Oracle (test infrastructure): the zeroth-order SGD step.

Three forms of the same step, all on float32 parameters:

  step_in_place   the in-place form of Eq. 1-3: the parameters themselves are moved to
                 theta + eps z, then to theta - eps z, then back (three in-place moves
                 by eps z times +1, -2, +1, each with a separately rounded multiply and
                 add, z regenerated from the step seed for every move), and only then
                 updated.  It is what the exact-restore form below is pinned against.
  step_whole     Alg. 1 with the restore made exact: theta is never overwritten
                 by a perturbation; W+ = theta + eps z and W- = theta - eps z are
                 formed as copies (Eq. 2), then theta <- theta - eta g z (Eq. 3).
  Zo2Blockwise   Alg. 2 + Sec. 5.4: the model is walked module by module
                 (Embedding, W_1..W_N, LM head); each module first applies the
                 update left pending by the previous iteration (its g, its seed,
                 its learning rate), then is perturbed both ways and run on the
                 two activation streams.  The last g stays pending until flush().
  step_whole_multi / Zo2Blockwise.step_extra
                 the same estimator averaged over q directions (Sec. 3 notes that the
                 framework carries over to other ZO estimators; this is the q-sample
                 form of Eq. 1-2): g_i from direction z_i, i = 0..q-1, all at the same
                 parameters and batch, then theta <- theta - sum_i eta_i g_i z_i
                 (eta_i = eta / q for the average), applied in the order i = 0, 1, ...

Arithmetic shared by the last two ("canonical"): one fused multiply-add per
element, a*b+c evaluated exactly and rounded once to float32; then, if the
parameters are held in a low-bit transfer format (Sec. 5.5), rounded to it.
  theta' = store(fma(-c, z_prev, theta)),   c = float32(eta_prev * g_prev)
  W+-    = compute(fma(+-eps, z, theta'))
  l+-    = float32(L(W+-; B)),  g = float32(float32(l+ - l-) / float32(2 eps))
"""
import numpy as np

from . import codec, opt_model, philox


def _fma32(a, b, c):
    """float32(a*b + c) for float32 inputs.  The product of two float32 values is
    exact in float64; the float64 sum rounds once more before the final rounding
    to float32 (a double rounding that differs from a true fused multiply-add
    only when the float64 sum lands exactly on a float32 midpoint)."""
    return (np.float64(a) * np.asarray(b, dtype=np.float64) + np.asarray(c, dtype=np.float64)).astype(np.float32)


def _store(x, fmt, scale=1.0, r16=None):
    """Round float32 x to the parameter storage format (value returned as float32): to nearest, or -
    given 16 random bits per element - stochastically.  With a per-tensor scale s (8-bit formats,
    Sec. 5.5) the stored code is that of float32(x * s) and the value read back is float32(code / s):
    the scaled value is formed in float32, the working precision of the update, for both roundings.
    For a power-of-two s both operations are exact."""
    if fmt == "f32":
        return np.asarray(x, dtype=np.float32)
    xs = np.asarray(x, dtype=np.float32)
    if scale != 1.0:
        xs = (xs * np.float32(scale)).astype(np.float32)
    q = codec.round_to(xs, fmt) if r16 is None else codec.round_stochastic(xs, fmt, r16)
    if scale != 1.0:
        return (q.astype(np.float32) / np.float32(scale)).astype(np.float32)
    return q


def z_of(shape_cfg, seed, names=None):
    """z for the named tensors (default: all) at step seed `seed`."""
    out = {}
    for name, tid, shp in opt_model.tensor_table(shape_cfg):
        if names is None or name in names:
            out[name] = philox.gaussian(seed, tid, 0, int(np.prod(shp))).reshape(shp)
    return out


def projected_gradient(lp, lm, eps):
    """Eq. 2 in float32: g = (l+ - l-) / (2 eps)."""
    lp = np.float32(lp)
    lm = np.float32(lm)
    return np.float32(np.float32(lp - lm) / np.float32(np.float32(2.0) * np.float32(eps)))


# --------------------------------------------------------------------------- Eq. 1-3, in place
def step_in_place(cfg, P, tokens, labels, seed, eps, lr):
    """The estimator of Eq. 1-2 evaluated by moving the parameters themselves, then the update of
    Eq. 3: theta visits theta + eps z and theta - eps z through in-place moves by k eps z, k = +1, -2,
    +1 (the last one brings it back up to rounding), the loss being taken after the first two.  Every
    move is a float32 multiply followed by a float32 add, and z is drawn afresh from the step seed for
    each of them and for the update.  P (name -> float32 array) is modified in place.
    Returns (l+, l-, g)."""
    eps32 = np.float32(eps)
    losses = []
    for k in (1.0, -2.0, 1.0):
        z = z_of(cfg, seed)
        move = np.float32(np.float32(k) * eps32)
        for name in P:
            P[name] = (P[name] + (move * z[name]).astype(np.float32)).astype(np.float32)
        if len(losses) < 2:
            losses.append(np.float32(opt_model.loss(cfg, P, tokens, labels)))
    lp, lm = losses
    g = projected_gradient(lp, lm, eps)
    z = z_of(cfg, seed)
    step = np.float32(np.float32(lr) * g)
    for name in P:
        P[name] = (P[name] - (step * z[name]).astype(np.float32)).astype(np.float32)
    return lp, lm, g


# --------------------------------------------------------------------------- Alg. 1, exact restore
def step_whole(cfg, P, tokens, labels, seed, eps, lr, store="f32", compute="f32", scales=None):
    """Whole-model step with canonical arithmetic.  P modified in place."""
    scales = scales or {}
    z = z_of(cfg, seed)
    eps32 = np.float32(eps)
    Wp = {n: _store(_fma32(eps32, z[n], P[n]), compute) for n in P}
    lp = np.float32(opt_model.loss(cfg, Wp, tokens, labels))
    del Wp
    Wm = {n: _store(_fma32(-eps32, z[n], P[n]), compute) for n in P}
    lm = np.float32(opt_model.loss(cfg, Wm, tokens, labels))
    del Wm
    g = projected_gradient(lp, lm, eps)
    c = np.float32(np.float32(lr) * g)
    for n in P:
        P[n] = _store(_fma32(-c, z[n], P[n]), store, scales.get(n, 1.0))
    return lp, lm, g


def step_whole_multi(cfg, P, tokens, labels, seeds, eps, lrs, store="f32", compute="f32", scales=None):
    """q directions at the same parameters (Eq. 2 once per seed), then the q updates of Eq. 3 one after the
    other in the order of `seeds`, each with canonical arithmetic.  lrs[i] belongs to seeds[i].  P modified in
    place.  Returns a list of (l+, l-, g)."""
    scales = scales or {}
    eps32 = np.float32(eps)
    out = []
    for seed in seeds:
        z = z_of(cfg, seed)
        Wp = {n: _store(_fma32(eps32, z[n], P[n]), compute) for n in P}
        lp = np.float32(opt_model.loss(cfg, Wp, tokens, labels))
        del Wp
        Wm = {n: _store(_fma32(-eps32, z[n], P[n]), compute) for n in P}
        lm = np.float32(opt_model.loss(cfg, Wm, tokens, labels))
        del Wm
        out.append((lp, lm, projected_gradient(lp, lm, eps)))
    for (lp, lm, g), seed, lr in zip(out, seeds, lrs):
        z = z_of(cfg, seed)
        c = np.float32(np.float32(lr) * g)
        for n in P:
            P[n] = _store(_fma32(-c, z[n], P[n]), store, scales.get(n, 1.0))
    return out


# --------------------------------------------------------------------------- Alg. 2 + deferred update
class Zo2Blockwise:
    """Alg. 2 with the update of iteration j-1 applied when each module is
    visited in iteration j (Sec. 5.4).  `pending` = (g, seed, lr) of the last
    iteration, or None."""

    def __init__(self, cfg, P, store="f32", compute="f32", scales=None, rounding="nearest"):
        self.cfg = cfg
        self.P = P
        self.store = store
        self.compute = compute
        self.scales = scales or {}
        self.rounding = rounding            # of the stored theta': "nearest" (the paper's cast) or "stochastic"
        self.pending = None
        self.extra = []
        self.ids = {name: tid for name, tid, _ in opt_model.tensor_table(cfg)}

    def _z(self, name, seed):
        a = self.P[name]
        return philox.gaussian(seed, self.ids[name], 0, a.size).reshape(a.shape)

    def _update_module(self, names):
        if self.pending is None:
            return
        for g, seed, lr in [self.pending] + self.extra:
            c = np.float32(np.float32(lr) * np.float32(g))
            for n in names:
                r16 = None
                if self.rounding == "stochastic" and self.store != "f32":
                    r16 = philox.rounding_bits(seed, self.ids[n], 0, self.P[n].size).reshape(self.P[n].shape)
                self.P[n] = _store(_fma32(-c, self._z(n, seed), self.P[n]), self.store, self.scales.get(n, 1.0), r16)

    def _perturbed_pair(self, names, seed, eps):
        """(W+, W-) of a module: z drawn once, used with both signs (Eq. 2)."""
        Wp, Wm = {}, {}
        for n in names:
            z = self._z(n, seed)
            Wp[n] = _store(_fma32(np.float32(eps), z, self.P[n]), self.compute)
            Wm[n] = _store(_fma32(-np.float32(eps), z, self.P[n]), self.compute)
        return Wp, Wm

    def _walk(self, tokens, labels, seed, eps, update):
        """One pass of Alg. 2 over the modules; `update`: apply what is pending to each module first."""
        cfg = self.cfg
        mods = opt_model.modules(cfg)
        # Embedding
        if update:
            self._update_module(mods[0])
        W = self._perturbed_pair(mods[0], seed, eps)
        emb_W = W
        acts = [opt_model.embed(cfg, W[k], tokens) for k in (0, 1)]
        # transformer blocks
        for l in range(cfg.n_layers):
            names = mods[1 + l]
            if update:
                self._update_module(names)
            W = self._perturbed_pair(names, seed, eps)
            acts = [opt_model.block_forward(cfg, W[k], l, acts[k]) for k in (0, 1)]
        # LM head (its tied weight was already updated with the embedding module)
        names = mods[-1]
        if update:
            self._update_module(names)
        W = self._perturbed_pair(names, seed, eps)
        losses = []
        for k in (0, 1):
            Wk = dict(W[k])
            if cfg.tied:
                Wk["tok_emb"] = emb_W[k]["tok_emb"]
            lg = opt_model.head_logits(cfg, Wk, acts[k])
            losses.append(np.float32(opt_model.cross_entropy(lg, labels)))
        return losses[0], losses[1], projected_gradient(losses[0], losses[1], eps)

    def step(self, tokens, labels, seed, eps, lr):
        lp, lm, g = self._walk(tokens, labels, seed, eps, update=True)
        self.pending = (g, seed, lr)
        self.extra = []
        return lp, lm, g

    def step_extra(self, tokens, labels, seed, eps, lr):
        """A further direction at the parameters the last step() left (its own update and the extras so far
        stay pending, nothing is applied): its (g, seed, lr) joins them."""
        if self.pending is None:
            raise ValueError("step_extra needs a step() before it")
        lp, lm, g = self._walk(tokens, labels, seed, eps, update=False)
        self.extra.append((g, seed, lr))
        return lp, lm, g

    def flush(self):
        """Apply the update still pending after the last iteration."""
        for names in opt_model.modules(self.cfg):
            self._update_module(names)
        self.pending = None
        self.extra = []

    def eval_loss(self, tokens, labels):
        """L(theta; B) with one unperturbed forward (the single-forward evaluation regime of the paper's
        Limitation section).  The deferred update (Sec. 5.4) belongs to theta already, so it is applied
        first; the forward then sees the parameters in the compute format, as the dual forward does."""
        self.flush()
        W = {n: _store(a, self.compute) for n, a in self.P.items()}
        return np.float32(opt_model.loss(self.cfg, W, tokens, labels))
