"""Shared helpers of the GPU parity tests: build the HIP context and the CPU checker on the same
seeded inputs and compare their outputs with the tolerances of the parity contract.

Tolerances (max-abs): fp32 model: logits 1e-4, probabilities 1e-3.  bf16 model: raw logits 3e-2, or
three times the checker's OWN logit change under a 1e-7 relative perturbation in front of its rounding
points if that is larger (measured by the test on the same inputs: `Pair(shadow=True)`).  A bf16
model is chaotic at the level of a bf16 ulp - such a perturbation grows to rounding noise within one
layer and then adds up over the layers - so two correct evaluations cannot agree better than that
floor (1e-2 .. 5e-2 at the widths and depths tested).  The factor 3: the perturbed checker still
rounds at the same points as the checker, whereas the kernels round some operands at other points
(bf16(x) before the RMSNorm factor instead of after it, attention weights before normalisation), which
makes their rounding noise independent of the checker's from the first layer on (a factor sqrt 2 in
rms), and the maximum over ~1e6 logits of two such differences spreads by another ~1.5.  The CFG mix l_u + s (l_c - l_u) multiplies the error of each row by |s| and
|s - 1|, hence the mixed-logit bound is (|s| + |s - 1|) times the raw one.  Decisions
(accept length, path, next token) must be identical whenever every draw the checker consulted was
farther than GUARD from its threshold; the final inverse-CDF draw is compared in interval form."""
import dataclasses
import math

import numpy as np
import torch

from oracle import vvs_oracle as vo
from paper_2511_13587_amd import binding as vb
from paper_2511_13587_amd import synth

GUARD = 1e-3


def logit_tol(shape, noise_floor=None):
    if shape.dtype == synth.DTYPE_FP32:
        return 1e-4
    if shape.n_layers > 12:
        assert noise_floor is not None, "deep bf16 shapes need the checker's measured noise floor"
    return max(3e-2, 3.0 * (noise_floor or 0.0))


def mixed_tol(shape, noise_floor=None):
    s = shape.cfg_scale
    return logit_tol(shape, noise_floor) * (abs(s) + abs(s - 1.0))


def perturbed_rounding(oracle, eps=1e-7, seed=1):
    """Makes the checker multiply every value by (1 + eps * N(0,1)) in front of its bf16 rounding points
    (the size of an fp32-vs-float64 summation difference).  Returns the checker."""
    base, rng = oracle.rb, np.random.default_rng(seed)
    oracle.rb = lambda x: base(np.asarray(x, dtype=np.float64) * (1.0 + eps * rng.standard_normal(np.shape(x))))
    return oracle


class Pair:
    """The HIP context and the checker, fed with identical inputs."""

    def __init__(self, shape, weights=None, gain_jitter=0.0, std=0.02, with_oracle=True, shadow=False, feature_pre_norm=0):
        self.shape = shape
        self.w = weights if weights is not None else synth.make_weights(shape, std=std, gain_jitter=gain_jitter)
        self.cfg = vb.make_config(shape, feature_pre_norm=feature_pre_norm)
        ocfg = dict(dataclasses.asdict(shape), feature_slots=self.cfg.feature_slots, feature_pre_norm=feature_pre_norm)
        self.ctx = vb.Context(self.cfg)
        self.ctx.load_weights_from_host(self.w, synth.weight_names(shape))
        self.oracle = vo.Oracle(ocfg, self.w) if with_oracle else None
        # a second checker with perturbed rounding measures the noise floor of this shape on these inputs
        self.shadow = perturbed_rounding(vo.Oracle(ocfg, self.w)) if shadow else None
        self.floor = 0.0
        self.dev = self.ctx.device
        B = shape.n_prompts
        self.accept_len = torch.zeros(B, dtype=torch.int32, device=self.dev)
        self.path = torch.zeros((B, vb.VVS_MAX_T), dtype=torch.int32, device=self.dev)
        self.next_token = torch.zeros(B, dtype=torch.int32, device=self.dev)
        self.nbr = None

    def set_neighbors(self, nbr):
        self.nbr = torch.from_numpy(np.ascontiguousarray(nbr, dtype=np.int32)).to(self.dev)
        self.ctx.vvs_set_neighbors(self.nbr)
        if self.oracle is not None:
            self.oracle.set_neighbors(nbr)
        if self.shadow is not None:
            self.shadow.set_neighbors(nbr)

    def dev_prefix(self, pc, pu):
        if self.shape.prefix_kind == synth.PREFIX_CLASS:
            return torch.from_numpy(pc).to(self.dev), (None if pu is None else torch.from_numpy(pu).to(self.dev))
        return vb.to_device(pc, self.shape.dtype), vb.to_device(pu, self.shape.dtype)

    def prefill(self, n_forced=0, u=None, run_oracle=True, robust_u=False):
        """robust_u: choose each prompt's uniform in the middle of the CDF interval of the checker's most
        probable first token, so that low-precision logit noise cannot change the first token."""
        shape = self.shape
        pc, pu = synth.make_prefix(shape)
        forced = synth.make_forced_tokens(shape, n_forced) if n_forced else None
        if u is None:
            u = np.random.default_rng(shape.seed + 5).random(shape.n_prompts, dtype=np.float32)
        if robust_u:
            self.oracle.prefill(pc, pu, forced, u)
            u = np.zeros(shape.n_prompts, dtype=np.float32)
            for b in range(shape.n_prompts):
                p = self.oracle.prefill_probs[b]
                top = int(np.argmax(p))
                u[b] = np.float32(p[:top].sum() + 0.5 * p[top])
        dpc, dpu = self.dev_prefix(pc, pu)
        dforced = None if forced is None else torch.from_numpy(forced).to(self.dev)
        du = torch.from_numpy(np.asarray(u, dtype=np.float32)).to(self.dev)
        first = torch.zeros(shape.n_prompts, dtype=torch.int32, device=self.dev)
        self.ctx.vvs_prefill(dpc, dpu, dforced, du, first)
        torch.cuda.synchronize()
        ofirst = None
        if run_oracle and self.oracle is not None:
            ofirst = self.oracle.prefill(pc, pu, forced, u)
            if self.shadow is not None:
                self.shadow.prefill(pc, pu, forced, u)
                self.floor = max(self.floor, float(np.abs(self.shadow.prefill_logits - self.oracle.prefill_logits).max()))
        return first.cpu().numpy(), ofirst, u

    def verify(self, parent, tokens, q, u, mode=0, run_oracle=True, mask=None, n_post=0):
        N = 0 if tokens is None else tokens.shape[1]
        dtok = None if N == 0 else torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(self.dev)
        dq = None if N == 0 else torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).to(self.dev)
        du = torch.from_numpy(np.ascontiguousarray(u, dtype=np.float32)).to(self.dev)
        if n_post:
            self.ctx.vvs_verify_post(N, n_post, parent, mask, dtok, dq, du, mode, self.accept_len, self.path, self.next_token)
        else:
            self.ctx.vvs_verify(N, parent, mask, dtok, dq, du, mode, self.accept_len, self.path, self.next_token)
        torch.cuda.synchronize()
        out = (self.accept_len.cpu().numpy().copy(), self.path.cpu().numpy().copy(), self.next_token.cpu().numpy().copy())
        oout = None
        if run_oracle and self.oracle is not None:
            oparent = np.arange(N) if parent is None else parent
            otok = np.zeros((self.shape.n_prompts, 0), dtype=np.int64) if N == 0 else tokens
            oq = np.zeros((self.shape.n_prompts, 1, self.shape.v_eff)) if N == 0 else q
            same_state = self.shadow is not None and all(
                self.shadow.kv_len(b) == self.oracle.kv_len(b) for b in range(self.shape.n_prompts))
            if same_state:
                self.shadow.pending[:] = self.oracle.pending
            oout = self.oracle.verify(oparent, otok, oq, u, mode, n_post=n_post)
            if same_state:
                self.shadow.verify(oparent, otok, oq, u, mode, n_post=n_post)
                self.floor = max(self.floor, float(np.abs(self.shadow.raw_logits - self.oracle.raw_logits).max()))
        return out, oout

    def commit(self, run_oracle=True):
        self.ctx.vvs_kv_commit()
        torch.cuda.synchronize()
        if run_oracle and self.oracle is not None:
            self.oracle.kv_commit()
            if self.shadow is not None and self.shadow.last is not None:
                self.shadow.kv_commit()

    def gpu_logits(self):
        raw, mixed, probs = self.ctx.vvs_debug_logits()
        torch.cuda.synchronize()
        return raw.cpu().numpy(), mixed.cpu().numpy(), probs.cpu().numpy()

    def close(self):
        self.ctx.close()


def check_logits(pair, label=""):
    """GPU raw / mixed logits and probabilities of the last verify against the checker's."""
    shape, o = pair.shape, pair.oracle
    raw, mixed, probs = pair.gpu_logits()
    e_raw = np.abs(raw - o.raw_logits).max()
    e_mix = np.abs(mixed - o.mixed_logits).max()
    e_p = np.abs(probs - o.probs).max()
    assert np.isfinite(raw).all() and np.isfinite(probs).all(), label
    assert e_raw <= logit_tol(shape, pair.floor), f"{label}: raw logits differ by {e_raw} (checker noise floor {pair.floor})"
    assert e_mix <= mixed_tol(shape, pair.floor), f"{label}: mixed logits differ by {e_mix}"
    if shape.dtype == synth.DTYPE_FP32:
        assert e_p <= 1e-3, f"{label}: probabilities differ by {e_p}"
    assert np.abs(probs.sum(-1) - 1).max() < 1e-4
    return e_raw, e_mix, e_p


def decisions_match(out, oout, traces, lo, guard=GUARD):
    """Compares (accept_len, path, next_token) per prompt.  Returns (n_exact, n_guarded): prompts
    whose outcome had to be (and was) identical / prompts where a consulted draw was inside the guard
    band, which only need a valid outcome (for the final draw: a token whose CDF interval lies within
    the guard of the uniform).  Raises AssertionError on a real mismatch."""
    a_g, path_g, next_g = out
    a_o, paths_o, next_o = oout
    exact = guarded = 0
    for b in range(len(a_o)):
        tr = traces[b]
        if tr is None:                               # finished prompt
            assert a_g[b] == 0 and next_g[b] == -1
            exact += 1
            continue
        robust = tr["accept_margin"] > guard and tr["relax_margin"] > 1e-6
        if not robust:
            guarded += 1
            assert 0 <= a_g[b] < len(path_g[b]) and path_g[b][0] == 0
            continue
        assert a_g[b] == a_o[b], f"prompt {b}: accept_len {a_g[b]} vs {a_o[b]} (margin {tr['accept_margin']})"
        assert list(path_g[b][:a_g[b] + 1]) == list(paths_o[b]), f"prompt {b}: path"
        assert (path_g[b][a_g[b] + 1:] == -1).all()
        # final draw, interval form
        cdf, u = tr["term_cdf"], tr["term_u"]
        lo_id = int(next_o[b])
        t = int(next_g[b])
        off = lo                                     # ids are full-vocabulary ids; the CDF is indexed inside the slice
        tl = t - off
        assert 0 <= tl < len(cdf), f"prompt {b}: token {t} outside the slice"
        c_lo = cdf[tl - 1] if tl > 0 else 0.0
        assert c_lo - guard <= u <= cdf[tl] + guard, f"prompt {b}: token {t} not within {guard} of u in the CDF"
        ol = lo_id - off
        o_lo = cdf[ol - 1] if ol > 0 else 0.0
        if o_lo + guard < u < cdf[ol] - guard:
            assert t == lo_id, f"prompt {b}: next token {t} vs {lo_id}"
            exact += 1
        else:
            guarded += 1
    return exact, guarded
