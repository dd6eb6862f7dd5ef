"""Shared helpers of the GPU parity tests: build the HIP context and the CPU checker on the same
seeded inputs and compare their outputs with the tolerances of the parity contract.

fp32 model: logits 1e-4, probabilities 1e-3 (max-abs), decisions identical outside a guard of 1e-3.

bf16 model, raw logits: max-abs <= max(3e-2, f x floor) and rms <= max(8e-3, f x rms floor) with f = 2 when
the library runs its separate normalisation kernels (they round where the checker does) and f = 3 when it
runs the fused layer, whose RMSNorm operand is rounded at another point (bf16(x g) with the row factor
applied after the projection): tests/test_rounding_points.py measures on the CPU alone, without any kernel,
that this placement by itself differs from the checker by 2.0 .. 2.6 x the floor.  The
floor is the checker's OWN logit change under a 1e-7 relative perturbation in front of its rounding
points, measured by the test on the same inputs (`Pair(shadow=True)`): a bf16 model is chaotic at the
level of a bf16 ulp - such a perturbation (the size of an fp32-vs-float64 summation difference) grows
to rounding noise within a layer and then adds up over the layers - so two correct evaluations cannot
agree better than that floor.  3e-2 is the contract's figure; it is the bound for shallow models.
The CFG mix l_u + s (l_c - l_u) multiplies the error of each row by |s| and |s - 1|, hence the
mixed-logit bound is (|s| + |s - 1|) times the raw one.
bf16 probabilities: a logit error eps moves every probability by at most a factor exp(+-2 eps), so
they are compared (a) with the float64 softmax of the kernel's own mixed logits, to 2e-6 (this is the
kernel's softmax, independent of the model's noise), and (b) with the checker's, to (exp(2 eps) - 1) p
for the measured eps; the measured max-abs difference is reported (with s = 7.5 it is above the
contract's 1e-3 whenever the mixed-logit error exceeds about 2e-3: DESIGN, numerics contract).
K / V cache: layer 0 within 2 bf16 ulps of the checker (4 for the fused layer; ulp of the element, or of the
tensor's rms for smaller elements), deeper layers within that + 3 x the shadow's own K / V change.
Decisions (accept length, path, next token) must be identical whenever every draw the checker
consulted was farther than the guard from its threshold; the final inverse-CDF draw is compared in
interval form; inside the guard the outcome must still be one the checker reaches with the consulted
uniforms moved by at most the guard."""
import dataclasses
import math

import numpy as np
import torch

from oracle import vvs_oracle as vo
from paper_2511_13587_amd import binding as vb
from paper_2511_13587_amd import synth

GUARD = 1e-3


FLOOR_FACTOR = 2.0          # separate normalisation kernels: the checker's rounding points
FLOOR_FACTOR_FUSED = 3.0    # fused layer: the norm operand is rounded at another point (see above)


def logit_tol(shape, noise_floor=None, fused=True):
    if shape.dtype == synth.DTYPE_FP32:
        return 1e-4
    if shape.n_layers > 12:
        assert noise_floor is not None, "deep bf16 shapes need the checker's measured noise floor"
    return max(3e-2, (FLOOR_FACTOR_FUSED if fused else FLOOR_FACTOR) * (noise_floor or 0.0))


def logit_rms_tol(shape, rms_floor=None, fused=True):
    if shape.dtype == synth.DTYPE_FP32:
        return 1e-5
    return max(8e-3, (FLOOR_FACTOR_FUSED if fused else FLOOR_FACTOR) * (rms_floor or 0.0))


def rms(a):
    a = np.asarray(a, dtype=np.float64)
    return float(np.sqrt(np.mean(a * a)))


def bf16_ulp(a):
    """Spacing of bf16 values at the magnitude of each element (8 significant bits)."""
    a = np.abs(np.asarray(a, dtype=np.float64))
    return 2.0 ** (np.floor(np.log2(np.maximum(a, 2.0 ** -120))) - 7)


def mixed_tol(shape, noise_floor=None, fused=True):
    s = shape.cfg_scale
    return logit_tol(shape, noise_floor, fused) * (abs(s) + abs(s - 1.0))


def perturbed_rounding(oracle, eps=1e-7, seed=1):
    """Makes the checker multiply every value by (1 + eps * N(0,1)) in front of its bf16 rounding points
    (the size of an fp32-vs-float64 summation difference).  Returns the checker."""
    base, rng = oracle.rb, np.random.default_rng(seed)
    oracle.rb = lambda x: base(np.asarray(x, dtype=np.float64) * (1.0 + eps * rng.standard_normal(np.shape(x))))
    return oracle


class Pair:
    """The HIP context and the checker, fed with identical inputs.  `sample`: the prompts the checker
    computes (default: all); the GPU always runs the whole batch.  Checker-side arrays (logits, traces,
    caches) are indexed by position in `sample`."""

    def __init__(self, shape, weights=None, gain_jitter=0.0, std=0.02, with_oracle=True, shadow=False, feature_pre_norm=0,
                 sample=None, norm_mode=0):
        self.shape = shape
        self.w = weights if weights is not None else synth.make_weights(shape, std=std, gain_jitter=gain_jitter)
        self.cfg = vb.make_config(shape, feature_pre_norm=feature_pre_norm, norm_mode=norm_mode)
        self.sample = list(range(shape.n_prompts)) if sample is None else list(sample)
        oshape = shape.replace(n_prompts=len(self.sample))
        ocfg = dict(dataclasses.asdict(oshape), feature_slots=self.cfg.feature_slots, feature_pre_norm=feature_pre_norm)
        self.ctx = vb.Context(self.cfg)
        self.ctx.load_weights_from_host(self.w, synth.weight_names(shape))
        self.oracle = vo.Oracle(ocfg, self.w) if with_oracle else None
        # a second checker with perturbed rounding measures the noise floor of this shape on these inputs
        self.shadow = perturbed_rounding(vo.Oracle(ocfg, self.w)) if shadow else None
        self.floor = 0.0          # max-abs raw-logit difference between the checker and its shadow so far
        self.floor_rms = 0.0      # the same in rms, of the last call
        self.dev = self.ctx.device
        # does any forward of this context (a verify over 1 + n_nodes tokens, a prefill chunk) take the fused layer?
        chunk = 32 if shape.d_head > 64 else 64
        self.fused = shape.dtype == synth.DTYPE_BF16 and (self.ctx.vvs_plan_is_fused(shape.n_nodes + 1) or self.ctx.vvs_plan_is_fused(chunk))
        B = shape.n_prompts
        self.accept_len = torch.zeros(B, dtype=torch.int32, device=self.dev)
        self.path = torch.zeros((B, vb.VVS_MAX_T), dtype=torch.int32, device=self.dev)
        self.next_token = torch.zeros(B, dtype=torch.int32, device=self.dev)
        self.nbr = None
        self.nbr_host = None
        self.last_call = None

    # rows of the GPU batch that belong to the sampled prompts, in the checker's order
    def rows(self):
        return [2 * b + i for b in self.sample for i in (0, 1)]

    def set_neighbors(self, nbr):
        self.nbr_host = np.asarray(nbr)
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

    def _note_floor(self, a, b):
        d = np.asarray(a) - np.asarray(b)
        self.floor = max(self.floor, float(np.abs(d).max()))
        self.floor_rms = rms(d)

    def prefill(self, n_forced=0, u=None, run_oracle=True, robust_u=False):
        """robust_u: choose each sampled prompt's uniform in the middle of the CDF interval of the checker's
        most probable first token, so that low-precision logit noise cannot change the first token."""
        shape, sm = self.shape, self.sample
        pc, pu = synth.make_prefix(shape)
        forced = synth.make_forced_tokens(shape, n_forced) if n_forced else None
        if u is None:
            u = np.random.default_rng(shape.seed + 5).random(shape.n_prompts, dtype=np.float32)
        u = np.array(u, dtype=np.float32)
        opu = pu if (pu is None or shape.prefix_kind == synth.PREFIX_DENSE) else pu[sm]
        oforced = None if forced is None else forced[sm]
        if robust_u:
            self.oracle.prefill(pc[sm], opu, oforced, u[sm])
            for i, b in enumerate(sm):
                p = self.oracle.prefill_probs[i]
                top = int(np.argmax(p))
                u[b] = np.float32(p[:top].sum() + 0.5 * p[top])
        dpc, dpu = self.dev_prefix(pc, pu)
        dforced = None if forced is None else torch.from_numpy(forced).to(self.dev)
        du = torch.from_numpy(u).to(self.dev)
        first = torch.zeros(shape.n_prompts, dtype=torch.int32, device=self.dev)
        self.ctx.vvs_prefill(dpc, dpu, dforced, du, first)
        torch.cuda.synchronize()
        ofirst = None
        if run_oracle and self.oracle is not None:
            ofirst = self.oracle.prefill(pc[sm], opu, oforced, u[sm])
            if self.shadow is not None:
                self.shadow.prefill(pc[sm], opu, oforced, u[sm])
                self._note_floor(self.shadow.prefill_logits, self.oracle.prefill_logits)
        return first.cpu().numpy(), ofirst, u

    def verify(self, parent, tokens, q, u, mode=0, run_oracle=True, mask=None, n_post=0):
        N = 0 if tokens is None else tokens.shape[1]
        sm = self.sample
        dtok = None if N == 0 else torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(self.dev)
        dq = None if N == 0 else torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).to(self.dev)
        du = torch.from_numpy(np.ascontiguousarray(u, dtype=np.float32)).to(self.dev)
        if n_post:
            self.ctx.vvs_verify_post(N, n_post, parent, mask, dtok, dq, du, mode, self.accept_len, self.path, self.next_token)
        else:
            self.ctx.vvs_verify(N, parent, mask, dtok, dq, du, mode, self.accept_len, self.path, self.next_token)
        torch.cuda.synchronize()
        out = (self.accept_len.cpu().numpy().copy(), self.path.cpu().numpy().copy(), self.next_token.cpu().numpy().copy())
        self.last_call = dict(parent=np.arange(N) if parent is None else np.asarray(parent), tokens=tokens, q=q, u=np.asarray(u),
                              mode=mode, n_post=n_post)
        oout = None
        if run_oracle and self.oracle is not None:
            ns = len(sm)
            oparent = np.arange(N) if parent is None else parent
            otok = np.zeros((ns, 0), dtype=np.int64) if N == 0 else tokens[sm]
            oq = np.zeros((ns, 1, self.shape.v_eff)) if N == 0 else q[sm]
            ou = np.asarray(u)[sm]
            same_state = self.shadow is not None and all(self.shadow.kv_len(b) == self.oracle.kv_len(b) for b in range(ns))
            if same_state:
                self.shadow.pending[:] = self.oracle.pending
            oout = self.oracle.verify(oparent, otok, oq, ou, mode, n_post=n_post)
            if same_state:
                self.shadow.verify(oparent, otok, oq, ou, mode, n_post=n_post)
                self._note_floor(self.shadow.raw_logits, self.oracle.raw_logits)
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


def check_logits(pair, label="", sharp=None):
    """GPU raw / mixed logits and probabilities of the last verify against the checker's (for the sampled
    prompts).  Returns a dict of the measured errors.  sharp: optional extra bound on the raw-logit error
    as a multiple of the checker's noise floor."""
    shape, o = pair.shape, pair.oracle
    raw, mixed, probs = pair.gpu_logits()
    assert np.isfinite(raw).all() and np.isfinite(probs).all(), label
    assert np.abs(probs.sum(-1) - 1).max() < 1e-4
    # (a) the kernel's own mix and softmax, checked on its own logits for every prompt of the batch
    s = shape.cfg_scale
    lc, lu = raw[0::2].astype(np.float64), raw[1::2].astype(np.float64)
    e_selfmix = float(np.abs(mixed - (lu + s * (lc - lu))).max())
    e_selfsm = float(np.abs(probs - vo.softmax(mixed.astype(np.float64))).max())
    assert e_selfmix <= 2e-5 * max(1.0, float(np.abs(mixed).max())), f"{label}: CFG mix of the kernel's own logits off by {e_selfmix}"
    assert e_selfsm <= 2e-6, f"{label}: softmax of the kernel's own mixed logits off by {e_selfsm}"
    # (b) against the checker
    rows, sm = pair.rows(), pair.sample
    d_raw = raw[rows] - o.raw_logits
    e_raw, r_raw = float(np.abs(d_raw).max()), rms(d_raw)
    e_mix = float(np.abs(mixed[sm] - o.mixed_logits).max())
    dp = np.abs(probs[sm] - o.probs)
    e_p = float(dp.max())
    tol, rtol = logit_tol(shape, pair.floor, pair.fused), logit_rms_tol(shape, pair.floor_rms, pair.fused)
    assert e_raw <= tol, f"{label}: raw logits differ by {e_raw} (bound {tol}, checker noise floor {pair.floor})"
    assert r_raw <= rtol, f"{label}: raw logits differ by {r_raw} rms (bound {rtol}, checker rms floor {pair.floor_rms})"
    assert e_mix <= mixed_tol(shape, pair.floor, pair.fused), f"{label}: mixed logits differ by {e_mix}"
    if sharp is not None:
        assert e_raw <= max(sharp * pair.floor, 2e-3), f"{label}: raw logits differ by {e_raw}, floor {pair.floor}"
    if shape.dtype == synth.DTYPE_FP32:
        assert e_p <= 1e-3, f"{label}: probabilities differ by {e_p}"
    else:
        # a logit error eps changes every probability by at most a factor exp(+-2 eps)
        bound = math.expm1(2.0 * e_mix) * np.maximum(probs[sm], o.probs) + 1e-7
        assert (dp <= bound).all(), f"{label}: probabilities differ by more than the mixed-logit error {e_mix} allows ({e_p})"
    return dict(raw=e_raw, raw_rms=r_raw, mixed=e_mix, prob=e_p, floor=pair.floor, floor_rms=pair.floor_rms)


def check_kv(pair, layer, n_slots, label="", prompts=None):
    """Cached K and V of the sampled prompts' rows, slots 0 .. n_slots - 1 of `layer`, against the checker.
    fp32: 1e-4.  bf16: layer 0 within n bf16 ulps, deeper layers within n ulps + 3 x the largest K / V
    difference between the checker and its shadow at that layer; n = 2 when the separate normalisation kernels
    run (same operand, same rounding point: one ulp for the summation order, one of margin) and n = 4 for the
    fused layer (its norm output is rounded at another point: two roundings of std 0.29 ulp each on every one of
    the d operands move an element by up to ~2 ulps at the maximum over 1e5 .. 1e6 elements, in front of the
    element's own rounding).  The ulp is that of the element, or of the
    rms of the compared tensor for elements below it: an element is a sum of ~d terms, so what differs in
    front of its own rounding (another rounding of the norm's output, another summation order) is
    proportional to the size of the terms, not to how far they happen to cancel."""
    o, sh = pair.oracle, pair.shadow
    worst = 0.0
    for b in (pair.sample if prompts is None else prompts):
        i = pair.sample.index(b)                      # the checker's index of GPU prompt b
        for j in (0, 1):
            k, v = pair.ctx.vvs_debug_kv(layer, 2 * b + j, n_slots)
            for name, g, want, shw in (("K", k, o.kc[2 * i + j][layer], sh.kc[2 * i + j][layer] if sh else None),
                                       ("V", v, o.vc[2 * i + j][layer], sh.vc[2 * i + j][layer] if sh else None)):
                want = want[:n_slots].reshape(n_slots, -1)
                got = g.cpu().numpy().astype(np.float64)
                err = np.abs(got - want)
                if pair.shape.dtype == synth.DTYPE_FP32:
                    assert err.max() < 1e-4, f"{label}: {name} of prompt {b} row {j} layer {layer} differs by {err.max()}"
                    continue
                extra = 0.0
                if layer > 0:
                    assert shw is not None and shw.shape[0] >= n_slots, "deeper layers need the shadow checker"
                    extra = 3.0 * float(np.abs(shw[:n_slots].reshape(n_slots, -1) - want).max())
                mag = np.maximum(np.maximum(np.abs(want), np.abs(got)), rms(want))
                tol = (4.0 if pair.fused else 2.0) * bf16_ulp(mag) + extra
                bad = err > tol
                assert not bad.any(), (f"{label}: {name} of prompt {b} row {j} layer {layer}: {int(bad.sum())} of {bad.size} elements off, "
                                       f"worst {err.max():.3e} (allowed {tol[np.unravel_index(np.argmax(err - tol), err.shape)]:.3e})")
                worst = max(worst, float((err / bf16_ulp(mag)).max()))
    return worst


def _valid_outcome(a, path, nxt, parent, lo, hi):
    """Structure every outcome must have: a parent chain from the root, -1 behind it, a token of the slice."""
    assert 0 <= a < len(path) and path[0] == 0
    for i in range(1, a + 1):
        assert 1 <= path[i] <= len(parent) and parent[path[i] - 1] == path[i - 1], f"path {list(path[:a + 1])} is not a parent chain"
    assert (np.asarray(path[a + 1:]) == -1).all()
    assert lo <= nxt < hi, f"token {nxt} outside the slice"


def _final_draw_ok(tr, t_local, guard):
    """Interval form of the final inverse-CDF draw.  Returns (valid, must_equal_checker)."""
    cdf, u = tr["term_cdf"], tr["term_u"]
    if not (0 <= t_local < len(cdf)):
        return False, False
    c_lo = cdf[t_local - 1] if t_local > 0 else 0.0
    return bool(c_lo - guard <= u <= cdf[t_local] + guard), False


def decisions_match(out, oout, traces, lo, guard=GUARD, redecide=None, parent=None, hi=None, prompts=None):
    """Compares (accept_len, path, next_token) per prompt (prompts: the GPU prompt of every checker entry).
    Returns (n_exact, n_guarded): prompts whose outcome had to be (and was) identical / prompts where a
    consulted draw was inside the guard band.  A guarded outcome must still be well-formed, and - when
    `redecide(i, u)` is given (the checker's decision for entry i with other uniforms) - be the outcome the
    checker reaches with the consulted accept draws moved by at most the guard (all up, all down, or one
    node at a time), its final token inside the guard of that outcome's CDF interval.
    Raises AssertionError on a real mismatch."""
    a_g, path_g, next_g = out
    a_o, paths_o, next_o = oout
    exact = guarded = 0
    for i in range(len(a_o)):
        b = i if prompts is None else prompts[i]
        tr = traces[i]
        if tr is None:                               # finished prompt
            assert a_g[b] == 0 and next_g[b] == -1
            exact += 1
            continue
        a, path, t = int(a_g[b]), path_g[b], int(next_g[b])
        if parent is not None:
            _valid_outcome(a, path, t, parent, lo, hi if hi is not None else lo + len(tr["term_cdf"]))
        robust = tr["accept_margin"] > guard and tr["relax_margin"] > 1e-6
        if not robust:
            guarded += 1
            assert 0 <= a < len(path) and path[0] == 0
            if redecide is not None:
                u0 = redecide.u(i)
                T = u0.shape[0]
                shifts = [np.zeros(T), np.full(T, guard), np.full(T, -guard)]
                for j in range(1, T):
                    for sgn in (1.0, -1.0):
                        e = np.zeros(T)
                        e[j] = sgn * guard
                        shifts.append(e)
                ok = False
                for sh in shifts:
                    u = u0.copy()
                    u[:, 0] = np.clip(u[:, 0] + sh, 0.0, 1.0 - 1e-12)
                    a2, path2, nxt2, tr2 = redecide(i, u)
                    if a2 == a and list(path2) == list(path[:a + 1]) and _final_draw_ok(tr2, t - lo, guard)[0]:
                        ok = True
                        break
                assert ok, f"prompt {b}: outcome (a={a}, path={list(path[:a + 1])}, next={t}) is not reachable within the guard"
            continue
        assert a == a_o[i], f"prompt {b}: accept_len {a} vs {a_o[i]} (margin {tr['accept_margin']})"
        assert list(path[:a + 1]) == list(paths_o[i]), f"prompt {b}: path"
        assert (path[a + 1:] == -1).all()
        # final draw, interval form (ids are full-vocabulary ids; the CDF is indexed inside the slice)
        cdf, u = tr["term_cdf"], tr["term_u"]
        lo_id = int(next_o[i])
        assert _final_draw_ok(tr, t - lo, guard)[0], f"prompt {b}: token {t} not within {guard} of u in the CDF"
        ol = lo_id - lo
        o_lo = cdf[ol - 1] if ol > 0 else 0.0
        if o_lo + guard < u < cdf[ol] - guard:
            assert t == lo_id, f"prompt {b}: next token {t} vs {lo_id}"
            exact += 1
        else:
            guarded += 1
    return exact, guarded


class Redecide:
    """The checker's acceptance procedure on given distributions, for decisions_match: entry i is decided
    again with other uniforms.  p [n, T, V] target distributions, q [n, T, V] draft, tokens [n, N] full ids."""

    def __init__(self, p, q, tokens, parent, u, caps, mode, nbr, shape, n_post=0):
        self.p, self.q, self.tokens, self.parent, self.uu = p, q, tokens, np.asarray(parent), np.asarray(u, dtype=np.float64)
        self.caps, self.mode, self.nbr, self.shape, self.n_post = caps, mode, nbr, shape, n_post

    def u(self, i):
        return self.uu[i].copy()

    def __call__(self, i, u):
        sh, tr = self.shape, {}
        a, path, nxt = vo.decide(np.asarray(self.p[i], dtype=np.float64), np.asarray(self.q[i], dtype=np.float64),
                                 np.asarray(self.tokens[i]) - sh.logit_lo, self.parent, u, self.caps[i], self.mode, self.nbr,
                                 sh.relax_k, sh.relax_delta, sh.logit_lo, trace=tr, n_forced=self.n_post)
        return a, path, sh.logit_lo + nxt, tr


def check_decisions_on_gpu_probs(pair, out, guard=GUARD):
    """End-to-end check of the acceptance stage inside a full verify call, for EVERY prompt of the batch: the
    checker's acceptance procedure, run in float64 on the probabilities the kernel itself produced, must
    give the kernel's outcome (identical outside the guard, reachable inside it).  Independent of the
    model's logit noise, so it holds for bf16 models at any depth.  Call it before the commit (the
    end-of-image cap is taken from the context's state).  Returns (n_exact, n_guarded)."""
    shape, lc = pair.shape, pair.last_call
    _, _, probs = pair.gpu_logits()
    B = shape.n_prompts
    N = len(lc["parent"])
    if N == 0:
        return 0, 0
    n_emitted = pair.ctx.vvs_read_state()[1]
    caps = [int(shape.grid - n_emitted[b] - 1) for b in range(B)]
    rd = Redecide(probs, lc["q"], lc["tokens"], lc["parent"], lc["u"], caps, lc["mode"], pair.nbr_host, shape, lc["n_post"])
    a_o, paths_o, next_o, traces = [], [], [], []
    for b in range(B):
        if n_emitted[b] >= shape.grid:               # finished prompt
            a_o.append(0); paths_o.append([0]); next_o.append(-1); traces.append(None)
            continue
        a, path, nxt, tr = rd(b, rd.u(b))
        a_o.append(a); paths_o.append(path); next_o.append(nxt); traces.append(tr)
    return decisions_match(out, (np.array(a_o), paths_o, np.array(next_o)), traces, shape.logit_lo, guard, redecide=rd,
                           parent=lc["parent"], hi=shape.logit_hi)
