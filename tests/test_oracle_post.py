"""Pins for the CPU checker's post verification and feature cache (oracle/vvs_oracle.py):

* post verification (Section 4.1): putting the tokens that were accepted without verification in
  front of the new candidates and running ONE pass gives the same logits, the same decisions and
  the same cache as first making those tokens part of the context by an ordinary prefill and then
  verifying the candidates alone ("restores exact AR conditioning");
* the unverified tokens are never tested: whatever their draft rows and uniforms hold, they are on
  the accepted path; the end-of-image cap still holds;
* token-level feature cache (Section 4.3, Algorithm 2 "UpdateCache"): after every commit the ring of
  a row holds the features of the most recent cached tokens, oldest first - checked against a plain
  list kept by the test and against one-token-at-a-time forwards (the definition);
* a feature is the input of the output head: feature @ W_out reproduces the raw logits."""
import dataclasses

import numpy as np
import pytest

from oracle import vvs_oracle as vo
from paper_2511_13587_amd import synth

SMALL = synth.Shape("small", 2, 64, 4, 96, 128, 0, 128, 4, 5, 3, synth.PREFIX_DENSE, 2, 4, None,
                    synth.DTYPE_FP32, 3.0, draft_std=2.0, seed=77)


def build(shape, gain_jitter=0.2, std=0.08, **extra):
    w = synth.make_weights(shape, std=std, gain_jitter=gain_jitter)
    cfg = dataclasses.asdict(shape)
    cfg.update(extra)
    return vo.Oracle(cfg, w), w


def post_parents(n_post, tree_parent):
    """Tree of the candidates hung below a chain of n_post unverified tokens."""
    shifted = [p + n_post for p in tree_parent]
    return np.array(list(range(n_post)) + shifted, dtype=np.int32)


@pytest.mark.parametrize("n_post", [1, 3, 5])
@pytest.mark.parametrize("tree", [False, True])
def test_post_verification_equals_prefill_then_verify(n_post, tree):
    widths = (2, 3, 2) if tree else None
    shape = SMALL.replace(n_nodes=7 if tree else 4, tree_widths=widths)
    N = shape.n_nodes
    parent = synth.tree_parents(shape.tree_widths, N, seed=5)
    pc, pu = synth.make_prefix(shape)
    m = 6                                                    # image tokens s_0 .. s_m known so far
    seq = synth.make_forced_tokens(shape, m + 1)
    q, toks = synth.make_draft(shape, parent, 0)
    u = synth.make_uniforms(shape, N, 0)

    # A: s_0 .. s_{m-1} are context, s_m is the pending token, the candidates are verified alone
    oa, w = build(shape)
    oa.prefill(pc, pu, seq[:, :m], np.full(shape.n_prompts, 0.5))
    oa.pending[:] = seq[:, m]
    oa.verify(parent, toks, q, u)
    # a correlated draft so that candidates are accepted as well
    q2, toks2 = synth.make_draft(shape.replace(draft_noise_std=0.3), parent, 1, base_logits=oa.mixed_logits.astype(np.float32))
    a_a, paths_a, nxt_a = oa.verify(parent, toks2, q2, u)
    logits_a = oa.raw_logits.copy()
    oa.kv_commit()

    # B: only s_0 .. s_{m-n_post-1} are context; s_{m-n_post} is pending; s_{m-n_post+1} .. s_m arrive unverified
    ob, _ = build(shape)
    ob.prefill(pc, pu, seq[:, :m - n_post], np.full(shape.n_prompts, 0.5))
    ob.pending[:] = seq[:, m - n_post]
    parent_b = post_parents(n_post, parent)
    toks_b = np.concatenate([seq[:, m - n_post + 1:m + 1], toks2], axis=1)
    rng = np.random.default_rng(3)
    V = shape.v_eff
    q_b = np.concatenate([rng.random((shape.n_prompts, n_post, V)), q2], axis=1)       # rows 0..n_post-1 are never read
    u_b = np.concatenate([np.ones((shape.n_prompts, n_post, 2)) * 0.999999, u], axis=1)  # would reject everything if it were read
    a_b, paths_b, nxt_b = ob.verify(parent_b, toks_b, q_b, u_b, n_post=n_post)
    for b in range(shape.n_prompts):
        assert a_b[b] == a_a[b] + n_post
        assert paths_b[b] == list(range(n_post + 1)) + [j + n_post for j in paths_a[b][1:]]
        assert nxt_b[b] == nxt_a[b]
    assert np.max(np.abs(ob.raw_logits[:, n_post:] - logits_a)) < 1e-10
    assert max(a_a) > 0                                      # candidates behind the unverified tokens were accepted too
    ob.kv_commit()
    assert np.array_equal(ob.n_emitted, oa.n_emitted) and np.array_equal(ob.pending, oa.pending)
    for row in range(2 * shape.n_prompts):
        for l in range(shape.n_layers):
            assert ob.kc[row][l].shape == oa.kc[row][l].shape
            assert np.allclose(ob.kc[row][l], oa.kc[row][l], atol=1e-10)
            assert np.allclose(ob.vc[row][l], oa.vc[row][l], atol=1e-10)
        # both rings hold the features of the same most recent tokens (A's prefill cached only its last position)
        fa, fb = oa.features(row), ob.features(row)
        k = min(len(fa), len(fb))
        assert k >= 2 and np.allclose(fb[-k:], fa[-k:], atol=1e-9)


def test_unverified_tokens_are_not_tested_and_cap_holds():
    shape = SMALL.replace(n_nodes=6)
    o, _ = build(shape)
    pc, pu = synth.make_prefix(shape)
    G = shape.grid_h * shape.grid_w
    o.prefill(pc, pu, synth.make_forced_tokens(shape, G - 4), np.full(shape.n_prompts, 0.5))   # n_emitted = G - 3: room for 2 more accepted tokens
    parent = post_parents(3, [0, 1, 2])
    rng = np.random.default_rng(0)
    toks = rng.integers(0, shape.v_eff, (shape.n_prompts, 6))
    q = rng.random((shape.n_prompts, 7, shape.v_eff))
    q /= q.sum(-1, keepdims=True)
    u = np.full((shape.n_prompts, 7, 2), 0.999999)
    a, paths, nxt = o.verify(parent, toks, q, u, n_post=3)
    # 3 unverified tokens, but only G - n_emitted - 1 = 2 may still be accepted; the walk stops there
    assert list(a) == [2] * shape.n_prompts and all(p == [0, 1, 2] for p in paths)
    o.kv_commit()
    assert (o.n_emitted == G).all()


def test_chain_and_descent_are_required():
    shape = SMALL.replace(n_nodes=4)
    o, _ = build(shape)
    pc, pu = synth.make_prefix(shape)
    o.prefill(pc, pu, None, np.full(shape.n_prompts, 0.5))
    q, toks = synth.make_draft(shape, np.arange(4), 0)
    u = synth.make_uniforms(shape, 4, 0)
    with pytest.raises(AssertionError):
        o.verify(np.array([0, 0, 1, 2]), toks, q, u, n_post=2)      # node 2 does not hang below node 1
    with pytest.raises(AssertionError):
        o.verify(np.array([0, 1, 0, 2]), toks, q, u, n_post=2)      # node 3 bypasses the unverified tokens


@pytest.mark.parametrize("pre_norm", [0, 1])
def test_feature_ring_against_a_plain_list_and_single_token_forwards(pre_norm):
    shape = SMALL.replace(n_nodes=4)
    o, w = build(shape, feature_pre_norm=pre_norm)
    pc, pu = synth.make_prefix(shape)
    first = o.prefill(pc, pu, synth.make_forced_tokens(shape, 2), np.full(shape.n_prompts, 0.5))
    assert all(o.features(r).shape == (1, shape.d_model) for r in range(2 * shape.n_prompts))
    parent = np.arange(4)
    mine = [[o.features(r)[0]] for r in range(2 * shape.n_prompts)]          # the test's own list per row
    lens = []
    for it in range(4):
        q, toks = synth.make_draft(shape, parent, it)
        o.verify(parent, toks, q, synth.make_uniforms(shape, 4, it))
        q2, toks2 = synth.make_draft(shape.replace(draft_noise_std=0.3), parent, it, base_logits=o.mixed_logits.astype(np.float32))
        a, paths, nxt = o.verify(parent, toks2, q2, synth.make_uniforms(shape, 4, 50 + it))
        # definition: the feature of a path token = hidden state of a one-token forward over its context
        for b in range(shape.n_prompts):
            for row in (2 * b, 2 * b + 1):
                vis_k = [o.kc[row][l].copy() for l in range(shape.n_layers)]
                vis_v = [o.vc[row][l].copy() for l in range(shape.n_layers)]
                for i, node in enumerate(paths[b]):
                    tok = o.pending[b] if node == 0 else toks2[b, node - 1]
                    _, new_kv = o.forward_one(np.asarray(w["embed"][tok], dtype=np.float64), int(o.n_emitted[b] - 1 + i), vis_k, vis_v)
                    mine[row].append(o.one_feature.copy())
                    for l, (k, v) in enumerate(new_kv):
                        vis_k[l] = np.concatenate([vis_k[l], k[None]], axis=0)
                        vis_v[l] = np.concatenate([vis_v[l], v[None]], axis=0)
        lens.append(int(a.max()))
        o.kv_commit()
        for row in range(2 * shape.n_prompts):
            want = np.stack(mine[row][-5:])
            got = o.features(row)
            assert got.shape == want.shape and np.allclose(got, want, atol=1e-9), (it, row)
    assert max(lens) >= 2                                     # pushes of several tokens at once happened
    assert o.features(0).shape[0] == 5                        # and the ring wrapped


def test_feature_times_head_is_the_logit_row():
    shape = SMALL.replace(n_nodes=4, logit_lo=32, logit_hi=96)
    o, w = build(shape)
    pc, pu = synth.make_prefix(shape)
    o.prefill(pc, pu, None, np.full(shape.n_prompts, 0.5))
    q, toks = synth.make_draft(shape, np.arange(4), 0)
    a, paths, _ = o.verify(np.arange(4), toks, q, synth.make_uniforms(shape, 4, 0))
    raw = o.raw_logits.copy()
    o.kv_commit()
    wout = np.asarray(w["wout"], dtype=np.float64)[:, 32:96]
    for b in range(shape.n_prompts):
        for row in (2 * b, 2 * b + 1):
            f = o.features(row)[-len(paths[b]):]
            assert np.allclose(f @ wout, raw[row][paths[b]], atol=1e-10)


def test_ring_can_be_switched_off():
    shape = SMALL.replace(n_nodes=2)
    o, _ = build(shape, feature_slots=0)
    pc, pu = synth.make_prefix(shape)
    o.prefill(pc, pu, None, np.full(shape.n_prompts, 0.5))
    assert o.features(0).shape == (0, shape.d_model)
