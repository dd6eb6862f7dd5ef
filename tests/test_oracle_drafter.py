"""Pins for the CPU checker's drafter (oracle/vvs_drafter.py).  The paper prints nothing of the
drafter's inside (it cites the feature-level drafting method), so the pins are:

* a drafter whose input map passes the token embedding through unchanged is a one-layer model of the
  target's kind: its distributions must equal those of the (already pinned) target checker run as a
  block over the same tokens, positions and ancestor sets;
* a drafter whose input map passes the FEATURE through: the root is fed the cached feature, a node is
  fed the feature its parent produced; siblings that differ only in their token get the same
  distribution;
* the general input map is linear in [token embedding ; feature], token half first;
* the tree rule by brute force (full sort), distinct siblings, normalised rows, zero rows for leaves;
* the level-by-level block formulation (all context pairs and all expanded nodes recomputed under an
  ancestor mask each level) gives the same result as the one-token-at-a-time definition;
* guidance scale 1 ignores the unconditional row; positions follow the root's image index."""
import dataclasses

import numpy as np
import pytest

from oracle import vvs_drafter as vd
from oracle import vvs_oracle as vo
from paper_2511_13587_amd import synth

SMALL = synth.Shape("small", 1, 64, 4, 96, 128, 16, 112, 4, 5, 3, synth.PREFIX_DENSE, 2, 7, (2, 3, 2),
                    synth.DTYPE_FP32, 3.0, seed=91)


def setup(shape=SMALL, fc=None, std=0.15, **cfg_extra):
    tw = synth.make_weights(shape, std=std, gain_jitter=0.2)
    dw = synth.make_drafter_weights(shape, tw, std=std, gain_jitter=0.2)
    if fc is not None:
        dw["fc"] = fc
    cfg = dataclasses.asdict(shape)
    cfg.update(cfg_extra)
    return vd.Drafter(cfg, dw), dw, cfg


def inputs(shape, k, seed=0):
    rng = np.random.default_rng(seed)
    recent = rng.integers(shape.logit_lo, shape.logit_hi, (shape.n_prompts, k))
    feats = [rng.standard_normal((k, shape.d_model)) for _ in range(2 * shape.n_prompts)]
    root = rng.integers(k - 1, shape.grid - 8, shape.n_prompts)
    return recent, feats, root


def ancestors(parent, j):
    out = []
    while j != 0:
        j = int(parent[j - 1])
        out.append(j)
    return out[::-1]


def block_model(cfg, dw):
    c = dict(cfg)
    c["n_layers"] = 1
    return vo.Oracle(c, dw)


@pytest.mark.parametrize("k", [1, 3])
def test_token_only_input_map_is_a_one_layer_target_model(k):
    d = SMALL.d_model
    fc = np.concatenate([np.eye(d), np.zeros((d, d))]).astype(np.float32)
    dr, dw, cfg = setup(fc=fc)
    parent = synth.tree_parents(SMALL.tree_widths, SMALL.n_nodes, seed=2)
    recent, feats, root = inputs(SMALL, k)
    tokens, q = dr.draft(parent, recent, feats, root)
    m = block_model(cfg, dw)
    T = len(parent) + 1
    kids = [[c for c in range(1, T) if parent[c - 1] == j] for j in range(T)]
    depth = synth.node_depths(parent)
    for b in range(SMALL.n_prompts):
        for j in range(T):
            if not kids[j]:
                assert (q[b, j] == 0).all()
                continue
            path = ancestors(parent, j)[1:] + ([j] if j else [])          # tree nodes from below the root down to j
            seq = list(recent[b]) + [int(tokens[b, n - 1]) for n in path]
            idx = [root[b] - (k - 1) + i for i in range(k)] + [root[b] + depth[n] for n in path]
            n = len(seq)
            rows = []
            for row in (2 * b, 2 * b + 1):
                m.reset()
                logits, _ = m.forward_block(row, m.embed_tokens(seq), idx, np.tril(np.ones((n, n))), logits_for=[n - 1])
                rows.append(logits[n - 1])
            _, want = m.mix(rows[0], rows[1])
            assert np.allclose(q[b, j], want, atol=1e-12), (b, j)
            order = np.argsort(-np.log(want), kind="stable")[:len(kids[j])]
            assert [int(tokens[b, c - 1]) for c in kids[j]] == [SMALL.logit_lo + int(o) for o in order]


def test_feature_only_input_map_feeds_cached_and_produced_features():
    d = SMALL.d_model
    fc = np.concatenate([np.zeros((d, d)), np.eye(d)]).astype(np.float32)
    dr, dw, cfg = setup(fc=fc)
    parent = np.array([0, 0, 1, 1, 2], dtype=np.int32)       # two expanded children of the root, three grandchildren
    k = 2
    recent, feats, root = inputs(SMALL, k, seed=1)
    tokens, q = dr.draft(parent, recent, feats, root)
    m = block_model(cfg, dw)
    for b in range(SMALL.n_prompts):
        idx = [root[b] - 1, root[b], root[b] + 1]
        rows_root, rows_child = [], []
        for row in (2 * b, 2 * b + 1):
            m.reset()
            logits, _ = m.forward_block(row, feats[row], idx[:2], np.tril(np.ones((2, 2))), logits_for=[1])
            rows_root.append(logits[1])
            f_root = m.block_features[1]
            m.reset()
            x3 = np.concatenate([feats[row], f_root[None]], axis=0)
            logits, _ = m.forward_block(row, x3, idx, np.tril(np.ones((3, 3))), logits_for=[2])
            rows_child.append(logits[2])
        assert np.allclose(q[b, 0], m.mix(rows_root[0], rows_root[1])[1], atol=1e-12)
        want = m.mix(rows_child[0], rows_child[1])[1]
        assert np.allclose(q[b, 1], want, atol=1e-12) and np.allclose(q[b, 2], want, atol=1e-12)   # siblings differ only in their token
        assert tokens[b, 0] != tokens[b, 1]


def test_input_map_is_linear_in_token_half_then_feature_half():
    dr, dw, _ = setup()
    d = SMALL.d_model
    rng = np.random.default_rng(5)
    f = rng.standard_normal(d)
    tok = 37
    want = dw["embed"][tok].astype(np.float64) @ dw["fc"][:d].astype(np.float64) + f @ dw["fc"][d:].astype(np.float64)
    assert np.allclose(dr.input_vector(tok, f), want, atol=1e-12)


def levelwise(dr, cfg, dw, parent, recent, feats, root, tokens):
    """The block formulation: per level, ONE masked forward over the context pairs and every expanded
    node so far; inputs of tree nodes use the features the previous level's forward produced."""
    m = block_model(cfg, dw)
    B, k = recent.shape
    T = len(parent) + 1
    kids = [[c for c in range(1, T) if parent[c - 1] == j] for j in range(T)]
    depth = synth.node_depths(parent)
    internal = [j for j in range(1, T) if kids[j]]
    q = np.zeros((B, T, m.hi - m.lo))
    for b in range(B):
        first = max(0, root[b] - (k - 1))
        prev_feat, prev_slot = {}, {}
        for level in range(int(depth.max())):
            nodes = [j for j in internal if depth[j] <= level]
            slot = {0: k - 1}
            slot.update({j: k + i for i, j in enumerate(nodes)})
            n = k + len(nodes)
            mask = np.zeros((n, n))
            mask[:k, :k] = np.tril(np.ones((k, k)))
            for j in nodes:
                mask[slot[j], :k] = 1
                mask[slot[j], slot[j]] = 1
                for a in ancestors(parent, j)[1:]:
                    mask[slot[j], slot[a]] = 1
            idx = [first + i for i in range(k)] + [first + k - 1 + depth[j] for j in nodes]
            new_feat, logit_rows = {}, {}
            for row in (2 * b, 2 * b + 1):
                x_in = [dr.input_vector(recent[b, i], feats[row][i]) for i in range(k)]
                x_in += [dr.input_vector(tokens[b, j - 1], prev_feat[row][prev_slot[int(parent[j - 1])]]) for j in nodes]
                m.reset()
                logits, _ = m.forward_block(row, np.stack(x_in), idx, mask)
                new_feat[row], logit_rows[row] = m.block_features.copy(), logits
            for j in [0] + nodes:
                if depth[j] == level:
                    q[b, j] = m.mix(logit_rows[2 * b][slot[j]], logit_rows[2 * b + 1][slot[j]])[1]
            prev_feat, prev_slot = new_feat, slot
    return q


@pytest.mark.parametrize("dtype", [synth.DTYPE_FP32, synth.DTYPE_BF16])
def test_levelwise_block_formulation_equals_the_definition(dtype):
    shape = SMALL.replace(dtype=dtype)
    dr, dw, cfg = setup(shape)
    parent = synth.tree_parents(shape.tree_widths, shape.n_nodes, seed=4)
    recent, feats, root = inputs(shape, 3, seed=2)
    if dtype == synth.DTYPE_BF16:
        feats = [vo.round_bf16(f) for f in feats]
    tokens, q = dr.draft(parent, recent, feats, root)
    q2 = levelwise(dr, cfg, dw, parent, recent, feats, root, tokens)
    assert np.allclose(q, q2, atol=1e-12)
    assert np.allclose(q.sum(-1)[q.sum(-1) > 0], 1.0)


def test_tree_rule_by_full_sort_and_given_tokens():
    dr, dw, cfg = setup()
    parent = synth.tree_parents((3, 4, 2), 9, seed=7)
    recent, feats, root = inputs(SMALL, 2, seed=3)
    tokens, q = dr.draft(parent, recent, feats, root)
    T = len(parent) + 1
    for b in range(SMALL.n_prompts):
        for j in range(T):
            kids = [c for c in range(1, T) if parent[c - 1] == j]
            if not kids:
                assert np.isnan(dr.mixed[b, j]).all() and (q[b, j] == 0).all()
                continue
            order = np.argsort(-dr.mixed[b, j], kind="stable")
            got = [int(tokens[b, c - 1]) - SMALL.logit_lo for c in kids]
            assert got == [int(o) for o in order[:len(kids)]] and len(set(got)) == len(got)
            assert abs(q[b, j].sum() - 1) < 1e-12 and np.all(np.diff(q[b, j][order]) <= 0)
    assert tokens.min() >= SMALL.logit_lo and tokens.max() < SMALL.logit_hi
    # giving the drafter its own tokens back changes nothing; other tokens change only what lies below them
    t2, q2 = dr.draft(parent, recent, feats, root, given_tokens=tokens)
    assert np.array_equal(t2, tokens) and np.array_equal(q2, q)
    other = tokens.copy()
    other[:, 0] = SMALL.logit_lo + (other[:, 0] - SMALL.logit_lo + 1) % SMALL.v_eff
    t3, q3 = dr.draft(parent, recent, feats, root, given_tokens=other)
    assert np.array_equal(t3, other) and np.array_equal(q3[:, 0], q[:, 0])
    below = [j for j in range(1, T) if 1 in ancestors(parent, j) + [j] and q[0, j].any()]
    assert below and all(not np.allclose(q3[:, j], q[:, j]) for j in below)


def test_guidance_scale_one_ignores_the_unconditional_row_and_positions_matter():
    shape = SMALL.replace(cfg_scale=1.0)
    dr, dw, cfg = setup(shape)
    parent = np.array([0, 1], dtype=np.int32)
    recent, feats, root = inputs(shape, 2, seed=4)
    _, q = dr.draft(parent, recent, feats, root)
    feats2 = [f if r % 2 == 0 else f + 1.0 for r, f in enumerate(feats)]
    _, q2 = dr.draft(parent, recent, feats2, root)
    assert np.allclose(q, q2, atol=1e-12)
    _, q3 = dr.draft(parent, recent, feats, root + 1)
    assert not np.allclose(q, q3)
    # a root closer to the start of the image than the context is long: the pairs start at index 0
    _, q4 = dr.draft(parent, recent, feats, np.zeros(shape.n_prompts, dtype=np.int64))
    _, q5 = dr.draft(parent, recent, feats, np.ones(shape.n_prompts, dtype=np.int64))
    assert np.allclose(q4, q5, atol=1e-12)
