"""CPU only: what the kernels' placement of the RMSNorm rounding point costs against the checker, measured
without any kernel.

The checker rounds the normalised, gained activation, h = bf16(x s g) with s = rsqrt(mean x^2 + eps), and
multiplies h by the weights as given.  The fused bf16 path of the library cannot know s when it writes the
operand (s needs the whole row, the writer owns 64 columns of it), so it writes bf16(x g) and applies s to
the fp32 result of the projection: (bf16(x g) W) s.  Both are equal in exact arithmetic; in bf16 they
are two different roundings of the same operand.  This file re-states the checker's block forward with
that one rounding point moved (float64 everywhere else, nothing shared with the library) and compares:

  same    the re-statement with the checker's own rounding point: must reproduce the checker exactly
  late    operand bf16(x g), row factor after the contraction (what the fused path computes)
  fold    operand bf16(x), gain folded into re-rounded weights bf16(W g) (an earlier design; dropped because
          it is never better than `late` and worse with non-trivial gains)
  shadow  the checker itself with a 1e-7 relative perturbation in front of its rounding points: the noise
          floor the GPU parity tests use
  off     the checker without operand rounding: the size of bf16 operand rounding itself

Result (2 layers at the LlamaGen-XL width, printed by the test): `late` differs from the checker by about
1.25 x `off` in rms and about twice the shadow floor at the maximum - the size of one independent set of
operand roundings.  That is nearly all of the difference between the library and the checker seen on the
GPU at the same shape, and it is why the bf16 bound of the parity tests is max(3e-2, 2 x floor) and not
the floor itself."""
import dataclasses

import numpy as np

from oracle import vvs_oracle as vo
from paper_2511_13587_amd import synth

F64 = np.float64


class MovedRounding(vo.Oracle):
    """The checker's block forward (Section 2, "Visual AR Generation Model": same steps, same order) with the
    rounding point of the three kinds of RMSNorm placed according to `variant`."""

    def __init__(self, cfg, weights, variant):
        super().__init__(cfg, weights)
        self.variant, self._folded = variant, {}

    def norm_then_project(self, x, gname, mats):
        rb, w = self.rb, self.w
        s = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + self.eps)
        g = w[gname]
        out = []
        for name, cols in mats:
            W = w[name] if cols is None else w[name][:, cols[0]:cols[1]]
            if self.variant == "late":
                out.append((rb(x * g) @ W) * s)
            elif self.variant == "fold":
                if (name, gname) not in self._folded:
                    self._folded[(name, gname)] = rb(W * g[:, None])
                out.append((rb(x) @ self._folded[(name, gname)]) * s)
            else:
                out.append(rb(x * s * g) @ W)
        return out

    def forward_block(self, row, x_in, img_index, mask, logits_for=None):
        rb, w = self.rb, self.w
        x = np.asarray(x_in, dtype=F64).copy()
        T = x.shape[0]
        mask = np.asarray(mask).astype(bool)
        pos = [self._grid_pos(int(i)) for i in img_index]
        gr = np.array([p[0] for p in pos], dtype=F64)[:, None, None]
        gc = np.array([p[1] for p in pos], dtype=F64)[:, None, None]
        new_kv = []
        for l in range(self.L):
            q, k, v = self.norm_then_project(x, f"l{l}.g1", [(f"l{l}.wq", None), (f"l{l}.wk", None), (f"l{l}.wv", None)])
            q = rb(self._rope_block(q.reshape(T, self.H, self.dh), gr, gc))
            k = rb(self._rope_block(k.reshape(T, self.H, self.dh), gr, gc))
            v = rb(v.reshape(T, self.H, self.dh))
            new_kv.append((k, v))
            keys = np.concatenate([self.kc[row][l], k], axis=0)
            vals = np.concatenate([self.vc[row][l], v], axis=0)
            S = keys.shape[0] - T
            vis = np.concatenate([np.ones((T, S), dtype=bool), mask], axis=1)
            o = np.empty((T, self.H, self.dh))
            for hd in range(self.H):
                sc = np.where(vis, q[:, hd, :] @ keys[:, hd, :].T / np.sqrt(self.dh), -np.inf)
                o[:, hd, :] = vo.softmax(sc) @ vals[:, hd, :]
            x = x + rb(o.reshape(T, self.d)) @ w[f"l{l}.wo"]
            gate, up = self.norm_then_project(x, f"l{l}.g2", [(f"l{l}.wg", None), (f"l{l}.wu", None)])
            x = x + rb(vo.silu(gate) * up) @ w[f"l{l}.wd"]
        self.block_features = self._feature(x)
        sel = np.arange(T) if logits_for is None else np.asarray(logits_for)
        logits = np.full((T, self.hi - self.lo), np.nan)
        logits[sel] = self.norm_then_project(x[sel], "gf", [("wout", (self.lo, self.hi))])[0]
        return logits, new_kv


def test_cost_of_the_late_row_factor():
    shape = synth.XL_TREE.replace(n_layers=2, n_prompts=1, prefix_len=16)
    w = synth.make_weights(shape, gain_jitter=0.1)
    cfg = dataclasses.asdict(shape)
    pc, pu = synth.make_prefix(shape)
    forced = synth.make_forced_tokens(shape, 12)
    parent = synth.tree_parents(shape.tree_widths, shape.n_nodes)
    q, toks = synth.make_draft(shape, parent, 0)
    u = synth.make_uniforms(shape, shape.n_nodes, 0)

    def logits_of(o):
        o.prefill(pc, pu, forced, np.array([0.5]))
        o.pending[:] = 7
        o.verify(parent, toks, q, u)
        return o.raw_logits.copy()

    base = logits_of(vo.Oracle(cfg, w))
    shadow = vo.Oracle(cfg, w)
    rb0, rng = shadow.rb, np.random.default_rng(1)
    shadow.rb = lambda x: rb0(np.asarray(x, dtype=F64) * (1.0 + 1e-7 * rng.standard_normal(np.shape(x))))
    off = vo.Oracle(cfg, w)
    off.rb = vo._ident
    runs = {"shadow": logits_of(shadow), "off": logits_of(off)}
    for variant in ("same", "late", "fold"):
        runs[variant] = logits_of(MovedRounding(cfg, w, variant))
    err = {k: (float(np.abs(v - base).max()), float(np.sqrt(np.mean((v - base) ** 2)))) for k, v in runs.items()}
    print(f"logit rms {np.sqrt(np.mean(base ** 2)):.3f}; difference from the checker (max-abs, rms): " +
          ", ".join(f"{k} {m:.4f} / {r:.5f}" for k, (m, r) in err.items()))
    assert err["same"][0] == 0.0                                  # the re-statement is the checker
    # one independent set of operand roundings: about the size of operand rounding itself ...
    assert 0.9 * err["off"][1] < err["late"][1] < 1.6 * err["off"][1]
    # ... above the floor of a same-rounding-points evaluation, and within the bound the GPU tests use
    assert err["shadow"][0] < err["late"][0] <= max(3e-2, 3.0 * err["shadow"][0])
    assert err["late"][1] <= max(8e-3, 3.0 * err["shadow"][1])
    # the dropped design: never better
    assert err["fold"][1] >= err["late"][1]
