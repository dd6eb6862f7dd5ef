"""CPU checker ("oracle") for the draft side of feature-level speculative decoding: the drafter M_D
that turns cached target features and the latest tokens into a tree of candidate tokens with the
distribution each group of siblings was taken from.

TEST INFRASTRUCTURE ONLY: float64 NumPy, one token at a time; shares no code with the HIP library
(it builds on the other checker file, oracle/vvs_oracle.py) and is never imported by the product path.

What it follows
---------------
* Section 3, "Stale Feature Reusability", and Algorithm 2 ("f_t <- Retrieve(C, a)", "C_t <- M_D(f_t, a)"):
  the drafter is conditioned on the last n cached target features together with the n latest
  tokens of the sequence; when the previous step was accepted without verification the features are
  older than the tokens they are paired with (stale) - the pairing is by recency, not by position.
* Section 4.1: under verification skipping the inputs are the stale features and the embeddings of the
  selected token sequence.
* Section 2, "Speculative Decoding": the drafter's output for a node is a distribution over the next
  token; it is the draft distribution the acceptance rule divides by.

The paper takes the drafter itself from the feature-level drafting work it cites and prints nothing of
its inside.  Readings (each is marked "reading:" below):
* a drafter input vector is W_fc applied to the concatenation [token embedding ; feature] (token
  half first), W_fc of shape [2 d, d], no bias;
* the drafter body is ONE decoder block of the target's kind (same attention, rotary embedding, MLP,
  norms) followed by a final norm with its own gain; it uses the target's token embedding table and
  output head;
* the feature the drafter hands to its own next level is the same kind of vector the target caches:
  the input of the output head (after the drafter's final norm), or the residual stream in front of
  it when the context says so;
* the drafter keeps no state between calls: its attention context is the n (feature, token) pairs of
  this call plus the ancestors of the node inside the candidate tree;
* a pair sits at the image position of its token; a tree node at the root's position plus its depth;
* conditional and unconditional rows are mixed exactly as for the target (logit space, same scale),
  softmax at temperature 1 over the allowed id slice;
* the candidate tree has a fixed shape per call; the c-th child (in node-id order) of a node carries
  the token with the c-th largest mixed logit at that node, ties to the lower id (greedy top-k
  expansion).  Optionally the children's tokens are given by the caller and only the distributions
  are computed.

Parity status: all of the above is a reading of a cited method, not of a formula the paper prints, so
the function is "parity unpinned" against the paper; the tests pin it to the already pinned target
checker (a drafter whose input map passes the token embedding through is a one-layer target model)
and to brute-force definitions of the tree rule.
"""
from __future__ import annotations

import numpy as np

from oracle import vvs_oracle as vo

F64 = np.float64


class Drafter:
    def __init__(self, cfg: dict, weights: dict):
        """cfg: the target's config dict (n_layers is ignored: the drafter has one block); weights:
        embed, prefix_embed (unused), l0.*, gf, wout as for a one-layer model, plus fc [2 d, d]."""
        c = dict(cfg)
        c["n_layers"] = 1
        c["feature_slots"] = 0
        self.m = vo.Oracle(c, weights)
        self.fc = np.asarray(weights["fc"], dtype=F64)
        assert self.fc.shape == (2 * self.m.d, self.m.d)

    def input_vector(self, token, feature):
        """reading: W_fc [embedding of the token ; feature]."""
        z = np.concatenate([self.m.w["embed"][int(token)], np.asarray(feature, dtype=F64)])
        return self.m.rb(z) @ self.fc

    def draft(self, parent, recent_tokens, features, root_index, given_tokens=None):
        """One drafting call.

        parent int [N]: shape of the candidate tree (parent[j-1] = parent of node j, root 0 = the
        latest token of the sequence); recent_tokens int [B, k]: the k latest tokens of every prompt,
        oldest first (full-vocabulary ids; the last one is the root); features: per ROW (2b = cond,
        2b+1 = uncond) an array [k, d], the k most recent cached target features, oldest first;
        root_index int [B]: image index of the root token; given_tokens int [B, N] or None.
        Returns (tokens int [B, N] full-vocabulary ids, q float [B, N+1, V_eff]: q[b, j] = distribution
        of the children of node j, zero rows for leaves).  self.mixed [B, N+1, V_eff] keeps the mixed
        logits of the expanded nodes (NaN rows for leaves)."""
        m = self.m
        parent = np.asarray(parent, dtype=np.int64)
        N = len(parent)
        T = N + 1
        recent_tokens = np.asarray(recent_tokens, dtype=np.int64)
        B, k = recent_tokens.shape
        children = [[] for _ in range(T)]
        depth = np.zeros(T, dtype=np.int64)
        for j in range(1, T):
            children[int(parent[j - 1])].append(j)
            depth[j] = depth[int(parent[j - 1])] + 1
        V = m.hi - m.lo
        tokens = np.zeros((B, N), dtype=np.int64)
        q = np.zeros((B, T, V))
        self.mixed = np.full((B, T, V), np.nan)
        for b in range(B):
            first = max(0, int(root_index[b]) - (k - 1))       # image index of the oldest pair
            rows = (2 * b, 2 * b + 1)
            ctx_k = {r: [np.zeros((0, m.H, m.dh))] for r in rows}     # one layer
            ctx_v = {r: [np.zeros((0, m.H, m.dh))] for r in rows}
            node_kv, node_feat, node_logits = {}, {}, {}
            # the k (feature, token) pairs, one token at a time; the last one is the root
            for i in range(k):
                for r in rows:
                    x_in = self.input_vector(recent_tokens[b, i], features[r][i])
                    logits, kv = m.forward_one(x_in, first + i, ctx_k[r], ctx_v[r], want_logits=(i == k - 1))
                    if i < k - 1:
                        ctx_k[r] = [np.concatenate([ctx_k[r][0], kv[0][0][None]], axis=0)]
                        ctx_v[r] = [np.concatenate([ctx_v[r][0], kv[0][1][None]], axis=0)]
                    else:
                        node_kv[(r, 0)], node_feat[(r, 0)], node_logits[(r, 0)] = kv[0], m.one_feature.copy(), logits
            for j in range(T):                                   # parents come before their children
                if not children[j]:
                    continue
                if j > 0:
                    anc = []
                    a = int(parent[j - 1])
                    while True:
                        anc.append(a)
                        if a == 0:
                            break
                        a = int(parent[a - 1])
                    anc = anc[::-1]                              # root first
                    for r in rows:
                        x_in = self.input_vector(tokens[b, j - 1], node_feat[(r, int(parent[j - 1]))])
                        vis_k = [np.concatenate([ctx_k[r][0]] + [node_kv[(r, a)][0][None] for a in anc], axis=0)]
                        vis_v = [np.concatenate([ctx_v[r][0]] + [node_kv[(r, a)][1][None] for a in anc], axis=0)]
                        logits, kv = m.forward_one(x_in, first + (k - 1) + int(depth[j]), vis_k, vis_v)
                        node_kv[(r, j)], node_feat[(r, j)], node_logits[(r, j)] = kv[0], m.one_feature.copy(), logits
                mixed, p = m.mix(node_logits[(rows[0], j)], node_logits[(rows[1], j)])
                self.mixed[b, j], q[b, j] = mixed, p
                if given_tokens is not None:
                    for c in children[j]:
                        tokens[b, c - 1] = int(given_tokens[b][c - 1])
                else:
                    left = mixed.copy()
                    for c in children[j]:                        # greedy: the largest logit not yet taken, lower id on ties
                        best = int(np.argmax(left))
                        tokens[b, c - 1] = m.lo + best
                        left[best] = -np.inf
        return tokens, q
