"""GPU parity of post verification (vvs_verify_post; Section 4.1) and of the token-level feature cache
(vvs_read_features; Section 4.3, Algorithm 2 "UpdateCache") against the CPU checker, through the C ABI."""
import numpy as np
import pytest

from paper_2511_13587_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gc():
    from tests import gpu_common
    return gpu_common


def post_parents(n_post, tree_parent):
    return np.array(list(range(n_post)) + [int(p) + n_post for p in tree_parent], dtype=np.int32)


def ring_of(pair, row):
    return pair.oracle.features(row)


def check_features(pair, tol, label=""):
    feats, count = pair.ctx.vvs_read_features()
    worst = 0.0
    for row in range(2 * pair.shape.n_prompts):
        want = ring_of(pair, row)
        assert count[row // 2] == len(want), (label, row, count, len(want))
        got = feats[row, :len(want)]
        assert (feats[row, len(want):] == 0).all()
        worst = max(worst, float(np.abs(got - want).max()) if len(want) else 0.0)
    assert worst <= tol, f"{label}: features differ by {worst} (bound {tol})"
    return worst


@pytest.mark.parametrize("pre_norm", [0, 1])
def test_tiny_post_verification_whole_image_fp32(gc, pre_norm):
    """fp32 shape, whole image: every call carries 0-5 unverified tokens in front of a small tree; logits
    1e-4, decisions identical outside the guard band, state, cache and feature ring after every commit."""
    shape = synth.TINY.replace(n_nodes=9)
    pair = gc.Pair(shape, gain_jitter=0.1, feature_pre_norm=pre_norm)
    pair.prefill()
    check_features(pair, 1e-4, "after prefill")
    base_tree = np.array([0, 0, 1, 1])                           # 4 candidates: two children of the last unverified token, two grandchildren
    rng = np.random.default_rng(11)
    calls = same = 0
    posts = []
    while pair.oracle.n_emitted[0] < shape.grid and calls < 40:
        n_post = int(rng.integers(0, 6))
        parent = post_parents(n_post, base_tree)
        N = len(parent)
        sh = shape.replace(n_nodes=N)
        q, toks = synth.make_draft(sh, parent, calls)
        u = synth.make_uniforms(sh, N, calls)
        out, oout = pair.verify(parent, toks, q, u, n_post=n_post)
        gc.check_logits(pair, f"call {calls}")
        gc.decisions_match(out, oout, pair.oracle.traces, shape.logit_lo)
        if not ((out[0] == oout[0]).all() and (out[2] == oout[2]).all()):
            break                                                # a guarded draw went the other way: stop the lockstep
        for b in range(shape.n_prompts):                         # the unverified tokens are on the path unless the image ends first
            cap = shape.grid - pair.oracle.n_emitted[b] - 1
            if pair.oracle.traces[b] is not None:
                assert list(out[1][b][:min(n_post, cap) + 1]) == list(range(min(n_post, cap) + 1))
        same += 1
        posts.append(n_post)
        pair.commit()
        st = pair.ctx.vvs_read_state()
        assert st[0, 0] == pair.oracle.kv_len(0) and st[1, 0] == pair.oracle.n_emitted[0] and st[2, 0] == pair.oracle.pending[0]
        check_features(pair, 1e-4, f"call {calls}")
        calls += 1
    assert same == calls and calls >= 5 and max(posts) >= 4 and 0 in posts
    S = pair.oracle.kv_len(0)
    for layer in range(shape.n_layers):
        for row in range(shape.n_rows):
            k, v = pair.ctx.vvs_debug_kv(layer, row, S)
            assert np.abs(k.cpu().numpy() - pair.oracle.kc[row][layer].reshape(S, -1)).max() < 1e-4
            assert np.abs(v.cpu().numpy() - pair.oracle.vc[row][layer].reshape(S, -1)).max() < 1e-4
    pair.close()


def test_post_verification_argument_errors(gc):
    shape = synth.TINY.replace(n_nodes=6)
    pair = gc.Pair(shape, with_oracle=False)
    pair.prefill(run_oracle=False)
    q, toks = synth.make_draft(shape, np.arange(6), 0)
    u = synth.make_uniforms(shape, 6, 0)
    vb = gc.vb
    for parent, n_post in ((np.array([0, 0, 1, 2, 3, 4]), 2),      # node 2 is not below node 1
                           (np.array([0, 1, 0, 2, 3, 4]), 2),      # node 3 bypasses the unverified tokens
                           (np.arange(6), 7), (np.arange(6), -1)):
        with pytest.raises(vb.VvsError) as e:
            pair.verify(parent, toks, q, u, n_post=n_post, run_oracle=False)
        assert e.value.status == vb.VVS_EINVAL
    pair.verify(np.arange(6), toks, q, u, n_post=6, run_oracle=False)   # everything unverified: a chain of forced tokens
    assert (pair.accept_len.cpu().numpy() == 6).all()
    pair.close()


def test_xl_shape_post_verification_bf16(gc):
    """Config 3's shape with 2 layers (bf16, the 5-kernel path): 3 unverified tokens in front of the
    26-node tree (T = 30 query tokens per row).  Logits within the noise-floor bound; the committed
    path starts with the unverified tokens; features within the same kind of bound."""
    n_post = 3
    base = synth.XL_TREE.replace(n_layers=2)
    tree = synth.tree_parents(base.tree_widths, base.n_nodes)
    parent = post_parents(n_post, tree)
    N = len(parent)
    shape = base.replace(n_nodes=N, tree_widths=None)
    pair = gc.Pair(shape, shadow=True)
    first, ofirst, _ = pair.prefill(n_forced=45, robust_u=True)
    assert (first == ofirst).all()
    fl = float(np.abs(pair.shadow.features(0) - pair.oracle.features(0)).max())
    scale = float(np.abs(pair.oracle.features(0)).max())
    check_features(pair, max(3 * fl, 2.0 ** -7 * scale), "after prefill")
    q, toks = synth.make_draft(shape, parent, 0)
    u = synth.make_uniforms(shape, N, 0)
    out, oout = pair.verify(parent, toks, q, u, n_post=n_post, mask=synth.ancestor_mask(parent))
    e = gc.check_logits(pair, "xl post")
    print("xl post verification (raw, mixed, prob errors; floor):", e, pair.floor)
    for b in range(shape.n_prompts):
        assert out[0][b] >= n_post and list(out[1][b][:n_post + 1]) == list(range(n_post + 1))
    if (out[0] == oout[0]).all() and (out[2] == oout[2]).all() and all(list(out[1][b][:out[0][b] + 1]) == list(oout[1][b]) for b in range(shape.n_prompts)):
        pair.commit()
        st = pair.ctx.vvs_read_state()
        for b in range(shape.n_prompts):
            assert st[0, b] == pair.oracle.kv_len(b) and st[1, b] == pair.oracle.n_emitted[b]
        fl = max(float(np.abs(pair.shadow.features(r) - pair.oracle.features(r)).max()) for r in range(2 * shape.n_prompts))
        worst = check_features(pair, max(3 * fl, 2.0 ** -7 * scale), "after commit")
        print("xl post verification: feature error", worst, "checker noise floor", fl, "largest feature", scale)
    pair.close()


def test_xl_shape_feature_ring_bf16(gc):
    """Config 3's shape with 2 layers (bf16): a call whose 5 tokens are all unverified has a path that
    no logit noise can change, so both sides commit the same tokens and the feature rings (5 newest
    of 1 + 6 features, wrapped) must agree to the checker's own noise."""
    shape = synth.XL_TREE.replace(n_layers=2, n_nodes=5, tree_widths=None)
    pair = gc.Pair(shape, shadow=True)
    pair.prefill(n_forced=45, robust_u=True)
    parent = np.arange(5, dtype=np.int32)
    q, toks = synth.make_draft(shape, parent, 0)
    u = synth.make_uniforms(shape, 5, 0)
    out, oout = pair.verify(parent, toks, q, u, n_post=5)
    gc.check_logits(pair, "xl all-unverified chain")
    assert (out[0] == 5).all() and (oout[0] == 5).all()
    pair.commit()
    st = pair.ctx.vvs_read_state()
    for b in range(shape.n_prompts):
        assert st[0, b] == pair.oracle.kv_len(b) and st[1, b] == pair.oracle.n_emitted[b]
    fl = max(float(np.abs(pair.shadow.features(r) - pair.oracle.features(r)).max()) for r in range(2 * shape.n_prompts))
    scale = max(float(np.abs(pair.oracle.features(r)).max()) for r in range(2 * shape.n_prompts))
    worst = check_features(pair, max(3 * fl, 2.0 ** -7 * scale), "after commit")
    print("xl feature ring: error", worst, "checker noise floor", fl, "largest feature", scale)
    S = pair.oracle.kv_len(0)
    for layer in range(shape.n_layers):
        gc.check_kv(pair, layer, S, "xl feature ring")
    pair.close()
