"""CPU checker ("oracle") for the verification-free step of VVS: which candidate path is kept without
asking the target model, how far it is truncated, and when a step may skip verification.

TEST INFRASTRUCTURE ONLY: plain Python / float64 NumPy written from the paper; shares no code with
the HIP library and is never imported by the product path.

What it follows
---------------
* Candidate paths: the candidate tree of a step is the set P of its root-to-leaf token paths
  (Section 4.2; the root - the last emitted token - is not part of a path).
* Unverified token selection (Section 4.2): one path is drawn uniformly from P, and only its first
  gamma = min(L_s, floor(mean path length of P)) tokens are kept (Eq. 1).
* Uniform-interval schedule (Section 4.4, first policy): with interval i, after i - 1 verified steps
  the i-th step skips verification.
* Dynamic schedule (Section 4.4, Eq. 2 and Algorithm 1): the step skips verification when the last
  step was verified and the weighted average similarity of the candidate paths reaches a
  threshold; the paths are down-sampled with stride 2 before the similarity is computed.
* No two consecutive verification-free steps (Section 4.1, last paragraph; Algorithm 1, first test).

Readings (the paper does not spell these out):
* S^(l) of Eq. 2 = mean cosine similarity, over all unordered pairs of (down-sampled) paths that both
  have a token at position l, of the latent codebook embeddings of their tokens at that position.
  Positions that fewer than two paths reach carry no evidence: they are left out and the weights
  alpha^l are renormalised over the positions that remain; if no position remains (fewer than two
  paths) the similarity is 1 (a single candidate agrees with itself).  An all-zero embedding has
  cosine 0 with everything.
* Downsample(C, stride 2) keeps every second path, starting with the first, paths ordered by the
  node id of their leaf.
* The uniform draw of a path: index floor(u * |P|) for a uniform u in [0, 1), paths in the same order.
"""
from __future__ import annotations

import math

import numpy as np


def tree_paths(parent):
    """parent int [N], parent[j-1] = parent of node j (root 0).  Returns the root-to-leaf paths as lists
    of node ids (root excluded), ordered by leaf id.  A tree without nodes has no path."""
    N = len(parent)
    has_child = [False] * (N + 1)
    for j in range(1, N + 1):
        has_child[int(parent[j - 1])] = True
    paths = []
    for leaf in range(1, N + 1):
        if has_child[leaf]:
            continue
        p = [leaf]
        while int(parent[p[-1] - 1]) != 0:
            p.append(int(parent[p[-1] - 1]))
        paths.append(p[::-1])
    return paths


def truncation_length(paths, selected):
    """Eq. 1: gamma = min(L_s, floor(mean length of the paths))."""
    mean_len = sum(len(p) for p in paths) / len(paths)
    return min(len(paths[selected]), int(math.floor(mean_len)))


def select_unverified(parent, u):
    """Section 4.2: uniform draw of one candidate path with the uniform u in [0, 1), truncated by Eq. 1.
    Returns the node ids of the kept tokens (possibly empty when the tree is empty)."""
    paths = tree_paths(parent)
    if not paths:
        return []
    s = min(int(math.floor(float(u) * len(paths))), len(paths) - 1)
    return paths[s][:truncation_length(paths, s)]


def path_similarity(parent, tokens, embed, alpha, stride=2):
    """Eq. 2 for one prompt.  tokens int [N]: token id of node j = tokens[j-1]; embed float [V, dim]."""
    paths = tree_paths(parent)[::stride]
    E = np.asarray(embed, dtype=np.float64)
    L = max((len(p) for p in paths), default=0)
    num = den = 0.0
    for l in range(L):
        reach = [p[l] for p in paths if len(p) > l]
        if len(reach) < 2:
            continue
        total, pairs = 0.0, 0
        for i in range(len(reach)):
            for j in range(i + 1, len(reach)):
                a, b = E[int(tokens[reach[i] - 1])], E[int(tokens[reach[j] - 1])]
                na, nb = math.sqrt(float(a @ a)), math.sqrt(float(b @ b))
                total += float(a @ b) / (na * nb) if na > 0 and nb > 0 else 0.0
                pairs += 1
        num += alpha ** l * (total / pairs)
        den += alpha ** l
    return num / den if den > 0 else 1.0


def skip_uniform(step_index, interval):
    """Uniform-interval policy: steps are counted from 0; with interval i >= 2 the steps i-1, 2i-1, ...
    are verification-free (after i - 1 verified steps the i-th is skipped), which also keeps two
    skips apart."""
    return interval >= 2 and (step_index + 1) % interval == 0


def skip_dynamic(similarity, threshold, last_step_verified):
    """Algorithm 1: never right after a verification-free step; otherwise skip iff the similarity
    reaches the threshold."""
    return bool(last_step_verified) and similarity >= threshold
