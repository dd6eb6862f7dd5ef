"""CPU checker ("oracle") for the target-model verification pass of speculative decoding for
visual autoregressive models.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, float64 NumPy statement of what the verify
pass computes, written from the paper's problem statement; it shares no code with the HIP library
and must never be imported by the product path (only by tests, the smoke check and the benchmark's
CPU-baseline leg).

What it follows
---------------
* Autoregressive factorisation (Section 2, "Visual AR Generation Model"): token s+l is predicted
  from tokens 1..s+l-1.  `forward_one` is literally that: one token, its visible keys/values, one
  logit row.  `forward_block` is the same computation for several tokens at once under an
  ancestor mask (tree verification, Section 3 "Verification Redundancy"); the test-suite equates the
  two.
* Speculative decoding (Section 2, "Speculative Decoding"): a drafted token x is accepted with
  probability min(1, target(x)/draft(x)); at the first rejection a replacement is drawn from the
  normalised positive part of (target - draft); if every candidate is accepted one more token is
  drawn from the last target distribution.  NOTE the paper writes p for the draft and q for the
  target; this file uses p = target, q = draft (the convention of the work it cites), and takes the
  residual as max(0, target - draft): the only sign for which the procedure is lossless, which the
  tests verify by enumeration.
* Relaxed acceptance (Section 2, last sentence; the printed formula reuses one index for two
  things): the acceptance numerator adds the target mass of the drafted token's latent nearest
  neighbours, taken in ascending distance while the added mass stays within a budget delta.
* KV cache upkeep (Section 4.1): the keys/values of accepted tokens join the cache so that the next
  call is conditioned exactly as plain AR decoding would be.
* Post verification (Section 4.1): tokens that were accepted without verification in the previous
  step are put in front of the new candidates and go through the same target pass; they are not
  tested again (they are already part of the output) - the pass only gives them their keys/values,
  which restores exact AR conditioning for everything behind them.  Here they are the first n_post
  nodes of the tree, a chain below the root, accepted unconditionally.
* Token-level feature cache (Section 4.3; Algorithm 2, "UpdateCache"): the target's hidden state
  in front of the output head ("feature") of every token that joins the sequence is kept in a ring
  of the most recent few (the supplementary material uses 5) per row.

Readings where the paper is silent (architecture, CFG, RoPE, tree rule) are listed in the project's
design notes; each is marked "reading:" below.

Parity status: the relaxed rule's *residual* (what is resampled after a relaxed rejection) is a
reading that no statement of the paper fixes -> "parity unpinned" beyond the invariants tested
(delta=0 equals strict, monotonicity, total-variation bound, closed form for delta>=1).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------------------------
# number formats
# ----------------------------------------------------------------------------------------------
def round_bf16(x):
    """Round float64/float32 values to the nearest bf16 (ties to even), returned as float64.
    reading: in a bf16 model every tensor-contraction operand is a bf16 value; sums are wider."""
    f = np.asarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    keep = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return keep.view(np.float32).astype(F64)


def _ident(x):
    return np.asarray(x, dtype=F64)


class _W64:
    """Read-only view of the weight dict that hands out float64 copies (made once per tensor)."""

    def __init__(self, weights):
        self._w, self._c = weights, {}

    def __getitem__(self, name):
        if name not in self._c:
            self._c[name] = np.asarray(self._w[name], dtype=F64)
        return self._c[name]


# ----------------------------------------------------------------------------------------------
# model pieces  (reading: pre-norm decoder block, RMSNorm, multi-head attention with as many KV
# heads as query heads, SwiGLU MLP, 2D RoPE, no biases, untied input/output embeddings)
# ----------------------------------------------------------------------------------------------
def rmsnorm(x, g, eps):
    x = np.asarray(x, dtype=F64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g


def silu(x):
    return x / (1.0 + np.exp(-x))


def rope_angles(d_head, base):
    """theta_i = base^(-2 i / (d_head/2)), i = 0 .. d_head/4 - 1 (one set per half of the head)."""
    half = d_head // 2
    i = np.arange(half // 2, dtype=F64)
    return base ** (-2.0 * i / half)


def rope_2d(v, grid_row, grid_col, base):
    """reading: 2D rotary embedding.  v [..., d_head].  The first half of the head dims is rotated
    by the token's grid row, the second half by its grid column; inside a half, adjacent pairs
    (2i, 2i+1) rotate by angle pos * theta_i.  A prefix token is passed with row = col = 0, which is
    the identity."""
    v = np.asarray(v, dtype=F64)
    d_head = v.shape[-1]
    half = d_head // 2
    th = rope_angles(d_head, base)
    out = np.empty_like(v)
    for h, pos in ((0, grid_row), (1, grid_col)):
        seg = v[..., h * half:(h + 1) * half]
        a = seg[..., 0::2]
        b = seg[..., 1::2]
        c, s = np.cos(pos * th), np.sin(pos * th)
        o = np.empty_like(seg)
        o[..., 0::2] = a * c - b * s
        o[..., 1::2] = a * s + b * c
        out[..., h * half:(h + 1) * half] = o
    return out


def softmax(z):
    z = np.asarray(z, dtype=F64)
    m = np.max(z, axis=-1, keepdims=True)
    e = np.exp(z - m)
    return e / np.sum(e, axis=-1, keepdims=True)


class Oracle:
    """State: per row r (row 2b = conditional, 2b+1 = unconditional) and per layer the cached keys
    and values (float64 arrays [S, H, d_head], already bf16 values for a bf16 model); per prompt the
    number of emitted image tokens and the pending token (emitted, its K/V not yet cached)."""

    def __init__(self, cfg: dict, weights: dict):
        c = dict(cfg)
        self.L, self.d, self.H, self.F = c["n_layers"], c["d_model"], c["n_heads"], c["d_ff"]
        self.dh = self.d // self.H
        self.V, self.lo, self.hi = c["vocab"], c["logit_lo"], c["logit_hi"]
        self.gh, self.gw, self.P = c["grid_h"], c["grid_w"], c["prefix_len"]
        self.G = self.gh * self.gw
        self.prefix_kind = c["prefix_kind"]
        self.n_classes = c.get("n_classes", 1000)
        self.B = c["n_prompts"]
        self.R = 2 * self.B
        self.scale = float(c["cfg_scale"])
        self.eps = float(c["rms_eps"])
        self.base = float(c["rope_base"])
        self.relax_k = int(c.get("relax_k", 0))
        self.relax_delta = float(c.get("relax_delta", 0.0))
        self.rb = round_bf16 if c["dtype"] == 1 else _ident
        self.ring_slots = int(c.get("feature_slots", 5))
        self.feature_pre_norm = bool(c.get("feature_pre_norm", 0))   # reading: feature = input of the output head (after the final norm) unless switched
        self.w = _W64(weights)                # float32 arrays [in, out], read as float64
        self.nbr = None
        self.reset()

    # -- state ---------------------------------------------------------------------------------
    def reset(self):
        self.kc = [[np.zeros((0, self.H, self.dh)) for _ in range(self.L)] for _ in range(self.R)]
        self.vc = [[np.zeros((0, self.H, self.dh)) for _ in range(self.L)] for _ in range(self.R)]
        self.n_emitted = np.zeros(self.B, dtype=np.int64)
        self.pending = -np.ones(self.B, dtype=np.int64)
        self.last = None
        self.ring = [[] for _ in range(self.R)]      # per row: the most recent features, oldest first

    def set_neighbors(self, nbr):
        self.nbr = np.asarray(nbr)

    def kv_len(self, b):
        return self.kc[2 * b][0].shape[0]

    # -- forward -------------------------------------------------------------------------------
    def _grid_pos(self, img_index):
        """image token index -> (grid row, grid col); prefix tokens (index < 0) -> (0, 0)."""
        if img_index < 0:
            return 0, 0
        return img_index // self.gw, img_index % self.gw

    def _qkv(self, l, h):
        w = self.w
        q = h @ w[f"l{l}.wq"]
        k = h @ w[f"l{l}.wk"]
        v = h @ w[f"l{l}.wv"]
        return q, k, v

    def forward_one(self, x_in, img_index, visible_k, visible_v, want_logits=True):
        """The definition: ONE token with input embedding x_in [d] at image index img_index (-1 for
        a prefix token).  visible_k / visible_v: per layer, arrays [n_vis, H, d_head] of the keys /
        values of every earlier token this one may look at.  Returns (logits over the allowed slice
        or None, per-layer (k, v) of this token [H, d_head])."""
        rb, w = self.rb, self.w
        x = np.asarray(x_in, dtype=F64).copy()
        gr, gc = self._grid_pos(img_index)
        new_kv = []
        for l in range(self.L):
            h = rb(rmsnorm(x, w[f"l{l}.g1"], self.eps))
            q, k, v = self._qkv(l, h)
            q = rb(rope_2d(q.reshape(self.H, self.dh), gr, gc, self.base))
            k = rb(rope_2d(k.reshape(self.H, self.dh), gr, gc, self.base))
            v = rb(v.reshape(self.H, self.dh))
            new_kv.append((k, v))
            keys = np.concatenate([visible_k[l], k[None]], axis=0)     # [n, H, dh]
            vals = np.concatenate([visible_v[l], v[None]], axis=0)
            o = np.empty((self.H, self.dh))
            for hd in range(self.H):
                s = keys[:, hd, :] @ q[hd] / np.sqrt(self.dh)
                o[hd] = softmax(s) @ vals[:, hd, :]
            x = x + rb(o.reshape(self.d)) @ w[f"l{l}.wo"]
            h2 = rb(rmsnorm(x, w[f"l{l}.g2"], self.eps))
            act = rb(silu(h2 @ w[f"l{l}.wg"]) * (h2 @ w[f"l{l}.wu"]))
            x = x + act @ w[f"l{l}.wd"]
        logits = None
        self.one_feature = self._feature(x)
        if want_logits:
            hf = rb(rmsnorm(x, w["gf"], self.eps))
            logits = hf @ w["wout"][:, self.lo:self.hi]
        return logits, new_kv

    def _feature(self, x):
        """Feature of a token = its hidden state in front of the output head, in the model's storage
        format.  reading: after the final norm (exactly what the head multiplies); the switch
        feature_pre_norm keeps the residual stream itself instead."""
        if self.feature_pre_norm:
            return self.rb(np.asarray(x, dtype=F64))
        return self.rb(rmsnorm(x, self.w["gf"], self.eps))

    def forward_block(self, row, x_in, img_index, mask, logits_for=None):
        """The same computation for T tokens of one row at once.  x_in [T, d]; img_index [T];
        mask [T, T] (1 = token i may look at token j of this block; must contain the diagonal);
        every cached position of the row is visible to all of them.  Returns (logits [T, V_eff] with
        only the rows in logits_for filled (default all), list per layer of (k, v) [T, H, d_head])."""
        rb, w = self.rb, self.w
        x = np.asarray(x_in, dtype=F64).copy()
        T = x.shape[0]
        mask = np.asarray(mask).astype(bool)
        pos = [self._grid_pos(int(i)) for i in img_index]
        gr = np.array([p[0] for p in pos], dtype=F64)[:, None, None]
        gc = np.array([p[1] for p in pos], dtype=F64)[:, None, None]
        new_kv = []
        for l in range(self.L):
            h = rb(rmsnorm(x, w[f"l{l}.g1"], self.eps))
            q, k, v = self._qkv(l, h)
            q = rb(self._rope_block(q.reshape(T, self.H, self.dh), gr, gc))
            k = rb(self._rope_block(k.reshape(T, self.H, self.dh), gr, gc))
            v = rb(v.reshape(T, self.H, self.dh))
            new_kv.append((k, v))
            ck, cv = self.kc[row][l], self.vc[row][l]
            S = ck.shape[0]
            keys = np.concatenate([ck, k], axis=0)
            vals = np.concatenate([cv, v], axis=0)
            vis = np.concatenate([np.ones((T, S), dtype=bool), mask], axis=1)   # [T, S+T]
            o = np.empty((T, self.H, self.dh))
            for hd in range(self.H):
                s = q[:, hd, :] @ keys[:, hd, :].T / np.sqrt(self.dh)
                s = np.where(vis, s, -np.inf)
                o[:, hd, :] = softmax(s) @ vals[:, hd, :]
            x = x + rb(o.reshape(T, self.d)) @ w[f"l{l}.wo"]
            h2 = rb(rmsnorm(x, w[f"l{l}.g2"], self.eps))
            act = rb(silu(h2 @ w[f"l{l}.wg"]) * (h2 @ w[f"l{l}.wu"]))
            x = x + act @ w[f"l{l}.wd"]
        self.block_features = self._feature(x)                      # [T, d]
        sel = np.arange(T) if logits_for is None else np.asarray(logits_for)
        logits = np.full((T, self.hi - self.lo), np.nan)
        hf = rb(rmsnorm(x[sel], w["gf"], self.eps))
        logits[sel] = hf @ w["wout"][:, self.lo:self.hi]
        return logits, new_kv

    def _rope_block(self, v, gr, gc):
        """rope_2d with a different position per token: v [T, H, dh]; gr, gc [T, 1, 1]."""
        half = self.dh // 2
        th = rope_angles(self.dh, self.base)
        out = np.empty_like(v)
        for hseg, pos in ((0, gr), (1, gc)):
            seg = v[..., hseg * half:(hseg + 1) * half]
            a, b = seg[..., 0::2], seg[..., 1::2]
            c, s = np.cos(pos * th), np.sin(pos * th)
            o = np.empty_like(seg)
            o[..., 0::2] = a * c - b * s
            o[..., 1::2] = a * s + b * c
            out[..., hseg * half:(hseg + 1) * half] = o
        return out

    # -- embeddings ----------------------------------------------------------------------------
    def embed_tokens(self, tokens):
        return self.w["embed"][np.asarray(tokens, dtype=np.int64)]

    def prefix_embeddings(self, prefix_cond, prefix_uncond, b):
        """(cond [P, d], uncond [P, d]) input vectors of prompt b.  reading: class prefix = rows of
        a class table whose last row is the null class; dense prefix = vectors fed as they are, the
        unconditional row uses one shared null prefix."""
        if self.prefix_kind == 0:
            tab = self.w["prefix_embed"]
            ids = np.asarray(prefix_cond[b], dtype=np.int64)
            unc = (np.full_like(ids, self.n_classes) if prefix_uncond is None
                   else np.asarray(prefix_uncond[b], dtype=np.int64))
            return tab[ids], tab[unc]
        return np.asarray(prefix_cond[b], dtype=F64), np.asarray(prefix_uncond, dtype=F64)

    # -- CFG + softmax -------------------------------------------------------------------------
    def mix(self, logit_c, logit_u):
        """reading: classifier-free guidance in logit space, l_u + s (l_c - l_u), softmax at
        temperature 1 (Section 5: "temperature 1.0") over the allowed id slice only."""
        lc, lu = np.asarray(logit_c, dtype=F64), np.asarray(logit_u, dtype=F64)
        mixed = lu + self.scale * (lc - lu)
        return mixed, softmax(mixed)

    # -- entry points --------------------------------------------------------------------------
    def prefill(self, prefix_cond, prefix_uncond, forced_tokens, uniforms):
        """Run the prefix (and optionally teacher-forced image tokens, int [B, n_forced]) through
        the model with a causal mask, cache their K/V, and sample the next image token of every
        prompt from the CFG-mixed distribution at the last position with uniforms[b]."""
        self.reset()
        n_forced = 0 if forced_tokens is None else np.asarray(forced_tokens).shape[1]
        assert n_forced <= self.G - 1
        first = np.zeros(self.B, dtype=np.int64)
        self.prefill_logits = np.zeros((self.R, self.hi - self.lo))
        self.prefill_probs = np.zeros((self.B, self.hi - self.lo))
        for b in range(self.B):
            pc, pu = self.prefix_embeddings(prefix_cond, prefix_uncond, b)
            rows_logits = []
            for row, pre in ((2 * b, pc), (2 * b + 1, pu)):
                x_in = pre
                idx = [-1] * self.P
                if n_forced:
                    x_in = np.concatenate([pre, self.embed_tokens(forced_tokens[b])], axis=0)
                    idx = idx + list(range(n_forced))
                T = x_in.shape[0]
                logits, new_kv = self.forward_block(row, x_in, idx, np.tril(np.ones((T, T))), logits_for=[T - 1])
                for l, (k, v) in enumerate(new_kv):
                    self.kc[row][l] = np.concatenate([self.kc[row][l], k], axis=0)
                    self.vc[row][l] = np.concatenate([self.vc[row][l], v], axis=0)
                rows_logits.append(logits[T - 1])
                self.prefill_logits[row] = logits[T - 1]
                # reading: the cache starts with the feature of the last prefilled position (the one the
                # first token is sampled from)
                self._push_features(row, self.block_features[T - 1:T])
            _, p = self.mix(rows_logits[0], rows_logits[1])
            self.prefill_probs[b] = p
            first[b] = self.lo + inverse_cdf(p, float(uniforms[b]))
            self.pending[b] = first[b]
            self.n_emitted[b] = n_forced + 1
        return first

    def verify(self, parent, draft_tokens, draft_probs, uniforms, mode=0, n_post=0):
        """One verification pass.  parent int [N] (None = chain over draft_tokens.shape[1] nodes);
        draft_tokens int [B, N] (full-vocabulary ids); draft_probs [B, T, V_eff]; uniforms
        [B, T, 2]; mode 0 strict, 1 relaxed.  Returns accept_len [B], path (list of node-id lists),
        next_token [B].  Keeps the per-node K/V, features and the outcome for kv_commit().
        n_post > 0 (Section 4.1, post verification): nodes 1..n_post are the tokens accepted without
        verification in the previous step, a chain below the root; every other node descends from
        node n_post.  They are accepted without a test (their draft rows and uniforms are not read)
        and count in accept_len."""
        draft_tokens = np.asarray(draft_tokens, dtype=np.int64).reshape(self.B, -1)
        N = draft_tokens.shape[1]
        parent = np.arange(N) if parent is None else np.asarray(parent, dtype=np.int64)
        assert 0 <= n_post <= N
        assert all(int(parent[i - 1]) == i - 1 for i in range(1, n_post + 1)), "post-verified tokens form a chain below the root"
        assert all(int(parent[j - 1]) >= n_post for j in range(n_post + 1, N + 1)), "candidates descend from the last post-verified token"
        T = N + 1
        depth = np.zeros(T, dtype=np.int64)
        mask = np.zeros((T, T), dtype=np.uint8)
        for j in range(T):
            i = j
            while True:
                mask[j, i] = 1
                if i == 0:
                    break
                i = int(parent[i - 1])
            if j:
                depth[j] = depth[parent[j - 1]] + 1
        accept_len = np.zeros(self.B, dtype=np.int64)
        next_token = -np.ones(self.B, dtype=np.int64)
        paths, node_kv, node_feat = [], [], []
        self.traces = [None] * self.B
        self.mixed_logits = np.zeros((self.B, T, self.hi - self.lo))
        self.raw_logits = np.zeros((self.R, T, self.hi - self.lo))
        self.probs = np.zeros_like(self.mixed_logits)
        for b in range(self.B):
            toks = np.concatenate([[self.pending[b]], draft_tokens[b]])
            x_in = self.embed_tokens(np.maximum(toks, 0))
            idx = self.n_emitted[b] - 1 + depth
            kv_rows, feat_rows = [], []
            for row in (2 * b, 2 * b + 1):
                logits, new_kv = self.forward_block(row, x_in, idx, mask)
                self.raw_logits[row] = logits
                kv_rows.append(new_kv)
                feat_rows.append(self.block_features)
            node_kv.append(kv_rows)
            node_feat.append(feat_rows)
            mixed, p = self.mix(self.raw_logits[2 * b], self.raw_logits[2 * b + 1])
            self.mixed_logits[b], self.probs[b] = mixed, p
            if self.n_emitted[b] >= self.G:          # image finished: nothing to verify
                paths.append([0])
                continue
            cap = self.G - self.n_emitted[b] - 1
            tr = {}
            a, path, nxt = decide(p, np.asarray(draft_probs[b], dtype=F64), draft_tokens[b] - self.lo, parent,
                                  np.asarray(uniforms[b], dtype=F64), cap, mode,
                                  self.nbr, self.relax_k, self.relax_delta, self.lo, trace=tr, n_forced=n_post)
            self.traces[b] = tr
            accept_len[b], next_token[b] = a, self.lo + nxt
            paths.append(path)
        self.last = dict(paths=paths, node_kv=node_kv, node_feat=node_feat, tokens=draft_tokens, accept_len=accept_len,
                         next_token=next_token)
        return accept_len, paths, next_token

    def kv_commit(self):
        """Section 4.1: keep the K/V of the pending token and of the accepted path, in order; the
        resampled / bonus token becomes the new pending token."""
        assert self.last is not None, "kv_commit without a preceding verify"
        for b in range(self.B):
            if self.last["next_token"][b] < 0:
                continue
            path = self.last["paths"][b]
            for i, row in enumerate((2 * b, 2 * b + 1)):
                for l, (k, v) in enumerate(self.last["node_kv"][b][i]):
                    self.kc[row][l] = np.concatenate([self.kc[row][l], k[path]], axis=0)
                    self.vc[row][l] = np.concatenate([self.vc[row][l], v[path]], axis=0)
                self._push_features(row, self.last["node_feat"][b][i][path])
            self.n_emitted[b] += len(path)
            self.pending[b] = self.last["next_token"][b]
        self.last = None

    def _push_features(self, row, feats):
        """Section 4.3 / Algorithm 2 "UpdateCache": the features of the tokens that just joined the
        cache are appended in sequence order; only the most recent ring_slots stay."""
        self.ring[row] = (self.ring[row] + [np.array(f, dtype=F64) for f in feats])[-self.ring_slots:] if self.ring_slots else []

    def features(self, row):
        """The cached features of a row, oldest first: array [n <= ring_slots, d]."""
        return np.stack(self.ring[row]) if self.ring[row] else np.zeros((0, self.d))

    def emitted_tokens(self, b):
        """Tokens that the last verify emitted for prompt b: accepted draft tokens, then the
        resampled / bonus token."""
        path = self.last["paths"][b]
        return [int(self.last["tokens"][b][j - 1]) for j in path[1:]] + [int(self.last["next_token"][b])]


# ----------------------------------------------------------------------------------------------
# the acceptance procedure
# ----------------------------------------------------------------------------------------------
def inverse_cdf(p, u):
    """reading: sample by inverse CDF in ascending id: first id whose running sum exceeds u * total;
    if rounding pushes past the end, the last id with non-zero mass."""
    p = np.asarray(p, dtype=F64)
    c = np.cumsum(p)
    hit = np.nonzero(c > u * c[-1])[0]
    if hit.size:
        return int(hit[0])
    return int(np.nonzero(p > 0)[0][-1])


def relaxed_target(P, x, nbr_row, k, delta, trace=None):
    """Relaxed rule: walk the neighbour list of x in ascending distance, absorbing target mass while
    the absorbed total stays <= delta (stop at the first neighbour that would exceed it).  Returns
    (numerator, modified target: absorbed mass moved onto x)."""
    Pt = P.copy()
    absorbed = 0.0
    for n in nbr_row[:k]:
        n = int(n)
        if n < 0 or n >= P.shape[0]:       # neighbour outside the allowed slice: no target mass
            continue
        if trace is not None:
            trace["relax_margin"] = min(trace["relax_margin"], abs(absorbed + P[n] - delta))
        if absorbed + P[n] > delta:
            break
        absorbed += P[n]
        Pt[n] = 0.0
    Pt[x] = P[x] + absorbed
    return Pt[x], Pt


def decide(p_rows, q_rows, tok_local, parent, u, cap, mode=0, nbr=None, relax_k=0, relax_delta=0.0, lo=0, trace=None, n_forced=0):
    """Acceptance walk for one prompt.

    p_rows [T, V] target distributions at the root (0) and at every draft node; q_rows [T, V]:
    q_rows[j] = draft distribution the children of node j were drawn from; tok_local [N] drafted
    token of node j = tok_local[j-1] (ids inside the slice); parent [N]; u [T, 2]; cap = how many
    draft tokens may still be accepted before the image is full.

    At the current node the children are tried in ascending node id (reading: recursive rejection
    over siblings drawn without replacement: after a rejection the target becomes the normalised
    positive part of target - draft, the rejected token leaves the draft distribution, which is
    renormalised).  A chain is the one-child case and is exactly the procedure of Section 2.
    Uniform u[c, 0] decides node c; u[j, 1] draws the final token when the walk ends at node j.
    Nodes 1..n_forced (post verification, Section 4.1) are accepted without a test: no uniform is
    consumed and the target is left as it is.  The end-of-image cap still holds for them.
    Returns (accept_len, path node ids starting with 0, next token id inside the slice).
    `trace` (a dict, optional) only records how close each decision was to flipping - the distance of
    every consulted uniform to its threshold, of every budget test to delta, and the CDF of the final
    draw - for tests that compare against lower-precision arithmetic; it changes nothing."""
    if trace is not None:
        trace.update(accept_margin=np.inf, relax_margin=np.inf)
    T = p_rows.shape[0]
    children = [[] for _ in range(T)]
    for j in range(1, T):
        children[int(parent[j - 1])].append(j)
    cur, a, path = 0, 0, [0]
    while True:
        P = np.asarray(p_rows[cur], dtype=F64).copy()
        accepted = None
        if a < cap and children[cur] and children[cur][0] <= n_forced:
            accepted = children[cur][0]
        elif a < cap and children[cur]:
            Q = np.asarray(q_rows[cur], dtype=F64).copy()
            for c in children[cur]:
                x = int(tok_local[c - 1])
                if mode == 1 and relax_k > 0:
                    num, Pt = relaxed_target(P, x, nbr[lo + x] - lo, relax_k, relax_delta, trace)
                else:
                    num, Pt = P[x], P
                if trace is not None:
                    thr = min(1.0, num / Q[x]) if Q[x] > 0 else (1.0 if num > 0 else 0.0)
                    trace["accept_margin"] = min(trace["accept_margin"], abs(u[c, 0] - thr))
                if u[c, 0] * Q[x] < num:            # u < min(1, num / Q[x]); 0/0 rejects
                    accepted = c
                    break
                R = np.maximum(0.0, Pt - Q)
                Z = R.sum()
                P = R / Z if Z > 0 else Pt
                Q[x] = 0.0
                Zq = Q.sum()
                if Zq <= 0:
                    break
                Q = Q / Zq
        if accepted is not None:
            cur = accepted
            a += 1
            path.append(cur)
            continue
        if trace is not None:
            trace.update(term_node=cur, term_u=float(u[cur, 1]), term_cdf=np.cumsum(P) / np.sum(P))
        return a, path, inverse_cdf(P, u[cur, 1])
