"""Pins for the CPU checker's transformer forward, CFG mix, prefill / verify / commit bookkeeping
(oracle/vvs_oracle.py) against what the paper and the mathematics fix:

* autoregressive factorisation (Section 2): scoring K drafted tokens (chain or tree) in one pass
  gives the same logits as K one-token passes along each root-to-node path;
* restoring KV entries re-establishes exact AR conditioning (Section 4.1): verify + commit leaves
  the same cache as a fresh prefill over everything emitted so far;
* library special case: with rotation-free (prefix) positions the block forward equals a
  composition of PyTorch's own rms_norm / linear / scaled_dot_product_attention / silu;
* rotary embedding: textbook properties and hand values;
* bf16 rounding equals PyTorch's float->bfloat16 conversion."""
import dataclasses

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import vvs_oracle as vo
from paper_2511_13587_amd import synth

SMALL = synth.Shape("small", 2, 64, 4, 96, 128, 0, 128, 4, 5, 3, synth.PREFIX_DENSE, 2, 4, None,
                    synth.DTYPE_FP32, 3.0, draft_std=2.0, seed=77)
SMALL_SLICE = SMALL.replace(name="small_slice", logit_lo=32, logit_hi=96, prefix_kind=synth.PREFIX_CLASS,
                            prefix_len=1, n_classes=10)


def build(shape, gain_jitter=0.2, std=0.08):
    w = synth.make_weights(shape, std=std, gain_jitter=gain_jitter)
    return vo.Oracle(dataclasses.asdict(shape), w), w


def run_prefill(o, shape, n_forced=0, seed=0):
    pc, pu = synth.make_prefix(shape)
    forced = synth.make_forced_tokens(shape, n_forced) if n_forced else None
    u = np.random.default_rng(seed).random(shape.n_prompts)
    return o.prefill(pc, pu, forced, u), (pc, pu)


# ------------------------------------------------------------------------------------------------
def test_round_bf16_matches_torch():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4096) * 10.0 ** rng.integers(-6, 6, 4096),
                        [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -9, -1.0 - 2.0 ** -8, 0.0, 65504.0]])
    x = x.astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(vo.round_bf16(x), want)
    assert np.array_equal(synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x)).astype(np.float64), want)


def test_rope_properties():
    rng = np.random.default_rng(1)
    dh, base = 16, 10000.0
    q, k = rng.standard_normal(dh), rng.standard_normal(dh)
    assert np.array_equal(vo.rope_2d(q, 0, 0, base), q)                     # prefix: identity
    for r, c in ((3, 5), (0, 7), (11, 0)):
        assert abs(np.linalg.norm(vo.rope_2d(q, r, c, base)) - np.linalg.norm(q)) < 1e-12
    # the score depends on the row / column offsets only
    s1 = vo.rope_2d(q, 5, 7, base) @ vo.rope_2d(k, 2, 3, base)
    s2 = vo.rope_2d(q, 9, 4, base) @ vo.rope_2d(k, 6, 0, base)
    assert abs(s1 - s2) < 1e-12
    s3 = vo.rope_2d(q, 5, 7, base) @ vo.rope_2d(k, 2, 4, base)
    assert abs(s1 - s3) > 1e-6
    # the grid row only touches the first half of the head, the column only the second half
    v = vo.rope_2d(q, 4, 0, base)
    assert np.array_equal(v[dh // 2:], q[dh // 2:]) and not np.allclose(v[:dh // 2], q[:dh // 2])
    v = vo.rope_2d(q, 0, 4, base)
    assert np.array_equal(v[:dh // 2], q[:dh // 2]) and not np.allclose(v[dh // 2:], q[dh // 2:])


def test_rope_hand_values():
    # d_head = 8: two pairs per half, angles theta_0 = 1, theta_1 = 10000^(-2/4) = 0.01
    assert np.allclose(vo.rope_angles(8, 10000.0), [1.0, 0.01], atol=1e-15)
    v = np.array([1.0, 0.0, 0.0, 2.0, 1.0, 1.0, 3.0, 0.0])
    out = vo.rope_2d(v, 2, 5, 10000.0)
    want = np.array([np.cos(2.0), np.sin(2.0),                                  # (1,0) by 2 rad
                     -2.0 * np.sin(0.02), 2.0 * np.cos(0.02),                   # (0,2) by 0.02 rad
                     np.cos(5.0) - np.sin(5.0), np.sin(5.0) + np.cos(5.0),      # (1,1) by 5 rad
                     3.0 * np.cos(0.05), 3.0 * np.sin(0.05)])                   # (3,0) by 0.05 rad
    assert np.allclose(out, want, atol=1e-14)


def test_rmsnorm_silu_softmax_against_torch():
    rng = np.random.default_rng(2)
    x, g = rng.standard_normal((5, 32)), rng.standard_normal(32)
    tx, tg = torch.from_numpy(x), torch.from_numpy(g)
    assert np.allclose(vo.rmsnorm(x, g, 1e-5), F.rms_norm(tx, (32,), tg, 1e-5).numpy(), atol=1e-13)
    assert np.allclose(vo.silu(x), F.silu(tx).numpy(), atol=1e-14)
    assert np.allclose(vo.softmax(x * 30), torch.softmax(tx * 30, -1).numpy(), atol=1e-14)


def torch_prefix_forward(shape, w, prefix):
    """Rotation-free causal forward of a [P, d] prefix built from PyTorch library routines only."""
    t = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    x = torch.from_numpy(np.asarray(prefix, dtype=np.float64))
    P, d, H = x.shape[0], shape.d_model, shape.n_heads
    for l in range(shape.n_layers):
        h = F.rms_norm(x, (d,), t[f"l{l}.g1"], shape.rms_eps)
        q, k, v = (F.linear(h, t[f"l{l}.{n}"].T).view(P, H, d // H).transpose(0, 1) for n in ("wq", "wk", "wv"))
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(0, 1).reshape(P, d)
        x = x + F.linear(o, t[f"l{l}.wo"].T)
        h = F.rms_norm(x, (d,), t[f"l{l}.g2"], shape.rms_eps)
        x = x + F.linear(F.silu(F.linear(h, t[f"l{l}.wg"].T)) * F.linear(h, t[f"l{l}.wu"].T), t[f"l{l}.wd"].T)
    hf = F.rms_norm(x, (d,), t["gf"], shape.rms_eps)
    return F.linear(hf, t["wout"].T[shape.logit_lo:shape.logit_hi]).numpy()


def test_prefix_forward_equals_torch_library_composition():
    shape = SMALL.replace(prefix_len=7)
    o, w = build(shape)
    _, (pc, pu) = run_prefill(o, shape)
    for b in range(shape.n_prompts):
        want_c = torch_prefix_forward(shape, w, pc[b])[-1]
        want_u = torch_prefix_forward(shape, w, pu)[-1]
        assert np.allclose(o.prefill_logits[2 * b], want_c, atol=1e-10)
        assert np.allclose(o.prefill_logits[2 * b + 1], want_u, atol=1e-10)
    # rows are (conditional, unconditional) pairs: different prompts differ, null rows agree
    assert not np.allclose(o.prefill_logits[0], o.prefill_logits[2])
    assert np.allclose(o.prefill_logits[1], o.prefill_logits[3], atol=1e-12)


@pytest.mark.parametrize("dtype,tol", [(synth.DTYPE_FP32, 1e-10), (synth.DTYPE_BF16, 2e-2)])
@pytest.mark.parametrize("tree", [False, True])
def test_block_verify_equals_sequential_single_token_forwards(dtype, tol, tree):
    widths = (2, 3, 2) if tree else None
    shape = SMALL.replace(dtype=dtype, n_nodes=7 if tree else 4, tree_widths=widths)
    o, w = build(shape)
    run_prefill(o, shape, n_forced=6)
    parent = synth.tree_parents(shape.tree_widths, shape.n_nodes, seed=5)
    q, toks = synth.make_draft(shape, parent, 0)
    u = synth.make_uniforms(shape, shape.n_nodes, 0)
    pending = o.pending.copy()
    n_emitted = o.n_emitted.copy()
    o.verify(parent, toks, q, u)
    depth = synth.node_depths(parent)
    if tree:
        assert depth.max() == 3 and len(set(parent.tolist())) < len(parent)
    for b in range(shape.n_prompts):
        for row in (2 * b, 2 * b + 1):
            for j in range(shape.n_nodes + 1):
                # fresh chain over root -> j, one token at a time, starting from the cached K/V
                chain = [j]
                while chain[-1] != 0:
                    chain.append(int(parent[chain[-1] - 1]))
                chain.reverse()
                vis_k = [o.kc[row][l].copy() for l in range(shape.n_layers)]
                vis_v = [o.vc[row][l].copy() for l in range(shape.n_layers)]
                for node in chain:
                    tok = pending[b] if node == 0 else toks[b, node - 1]
                    x_in = np.asarray(w["embed"][tok], dtype=np.float64)
                    logits, new_kv = o.forward_one(x_in, int(n_emitted[b] - 1 + depth[node]), vis_k, vis_v)
                    for l, (k, v) in enumerate(new_kv):
                        vis_k[l] = np.concatenate([vis_k[l], k[None]], axis=0)
                        vis_v[l] = np.concatenate([vis_v[l], v[None]], axis=0)
                assert np.max(np.abs(logits - o.raw_logits[row, j])) < tol, (row, j)


def test_cfg_mix_and_slice():
    shape = SMALL_SLICE
    o, _ = build(shape)
    rng = np.random.default_rng(4)
    lc, lu = rng.standard_normal(shape.v_eff), rng.standard_normal(shape.v_eff)
    o.scale = 1.0
    assert np.allclose(o.mix(lc, lu)[1], vo.softmax(lc), atol=1e-15)
    o.scale = 0.0
    assert np.allclose(o.mix(lc, lu)[1], vo.softmax(lu), atol=1e-15)
    o.scale = 3.0
    m, p = o.mix(lc, lu)
    assert np.allclose(m, 3.0 * lc - 2.0 * lu, atol=1e-14) and abs(p.sum() - 1) < 1e-14
    # every emitted id lies inside the allowed slice
    o.scale = shape.cfg_scale
    first, _ = run_prefill(o, shape)
    assert ((first >= shape.logit_lo) & (first < shape.logit_hi)).all()
    parent = synth.tree_parents(None, shape.n_nodes)
    for it in range(6):
        q, toks = synth.make_draft(shape, parent, it)
        assert ((toks >= shape.logit_lo) & (toks < shape.logit_hi)).all()
        _, _, nxt = o.verify(parent, toks, q, synth.make_uniforms(shape, shape.n_nodes, it))
        assert ((nxt >= shape.logit_lo) & (nxt < shape.logit_hi)).all()
        o.kv_commit()


@pytest.mark.parametrize("tree", [False, True])
def test_commit_equals_fresh_prefill(tree):
    widths = (3, 3, 2) if tree else None
    shape = SMALL.replace(n_nodes=8 if tree else 4, tree_widths=widths)
    o, w = build(shape)
    first, (pc, pu) = run_prefill(o, shape)
    emitted = [[int(first[b])] for b in range(shape.n_prompts)]
    parent = synth.tree_parents(shape.tree_widths, shape.n_nodes, seed=9)
    for it in range(3):
        # "correlated" draft so that several tokens are accepted: q = target of a first dry pass
        q, toks = synth.make_draft(shape, parent, it)
        o.verify(parent, toks, q, synth.make_uniforms(shape, shape.n_nodes, it))
        q2, toks2 = synth.make_draft(shape.replace(draft_noise_std=0.3), parent, it,
                                     base_logits=o.mixed_logits.astype(np.float32))
        u = synth.make_uniforms(shape, shape.n_nodes, 100 + it)
        a, paths, nxt = o.verify(parent, toks2, q2, u)
        for b in range(shape.n_prompts):
            emitted[b] += o.emitted_tokens(b)
            assert len(o.emitted_tokens(b)) == a[b] + 1 >= 1
        o.kv_commit()
    assert max(len(e) for e in emitted) > 4          # something was accepted
    n = min(len(e) for e in emitted)
    # a fresh prefill over prefix + emitted tokens (all but the pending one) must rebuild the cache
    for b in range(shape.n_prompts):
        o2 = vo.Oracle(dataclasses.asdict(shape), w)
        forced = np.array([emitted[bb][:len(emitted[b]) - 1] if bb == b else
                           (emitted[b][:len(emitted[b]) - 1]) for bb in range(shape.n_prompts)])
        o2.prefill(np.stack([pc[b]] * shape.n_prompts), pu, forced, np.full(shape.n_prompts, 0.5))
        assert o2.n_emitted[0] == o.n_emitted[b] == len(emitted[b])
        for row_new, row_old in ((0, 2 * b), (1, 2 * b + 1)):
            for l in range(shape.n_layers):
                assert o2.kc[row_new][l].shape == o.kc[row_old][l].shape
                assert np.allclose(o2.kc[row_new][l], o.kc[row_old][l], atol=1e-10)
                assert np.allclose(o2.vc[row_new][l], o.vc[row_old][l], atol=1e-10)
    assert n >= 4


def test_whole_image_bookkeeping_and_tpf():
    """Tokens-per-forward bookkeeping (Section 5, metrics): with no draft each pass emits exactly
    one token (TPF = 1.00); with drafts every pass emits accept_len + 1 >= 1 tokens and the image
    ends after exactly G tokens."""
    shape = SMALL.replace(n_prompts=1)
    o, _ = build(shape)
    run_prefill(o, shape)
    passes = 0
    while o.n_emitted[0] < shape.grid:
        a, _, nxt = o.verify(np.zeros(0, dtype=int), np.zeros((1, 0), dtype=int),
                             np.zeros((1, 1, shape.v_eff)), np.array([[[0.5, 0.123]]]))
        assert a[0] == 0 and nxt[0] >= 0
        o.kv_commit()
        passes += 1
    assert passes == shape.grid - 1 and o.kv_len(0) == shape.prefix_len + shape.grid - 1
    a, _, nxt = o.verify(np.zeros(0, dtype=int), np.zeros((1, 0), dtype=int),
                         np.zeros((1, 1, shape.v_eff)), np.array([[[0.5, 0.5]]]))
    assert nxt[0] == -1                                   # finished prompts emit nothing
    o2, _ = build(shape)
    run_prefill(o2, shape)
    parent = synth.tree_parents(None, 4)
    total, passes = 1, 0
    while o2.n_emitted[0] < shape.grid:
        q, toks = synth.make_draft(shape, parent, passes)
        a, _, _ = o2.verify(parent, toks, q * 0 + 1.0 / shape.v_eff, np.zeros((1, 5, 2)))  # u = 0: accept all
        total += a[0] + 1
        o2.kv_commit()
        passes += 1
    assert total == shape.grid == o2.n_emitted[0] and passes < shape.grid - 1


def test_synthetic_tree_shapes():
    for shape, depth in ((synth.XL_TREE, 6), (synth.XL_STRESS, 7)):
        parent = synth.tree_parents(shape.tree_widths, shape.n_nodes)
        assert len(parent) == shape.n_nodes and all(parent[j] <= j for j in range(len(parent)))
        assert synth.node_depths(parent).max() == depth
        m = synth.ancestor_mask(parent)
        assert (np.diag(m) == 1).all() and (m[:, 0] == 1).all() and np.triu(m, 1).sum() == 0
        assert (m.sum(1) == synth.node_depths(parent) + 1).all()
    assert (synth.ancestor_mask(synth.tree_parents(None, 5)) == np.tril(np.ones((6, 6)))).all()


def test_bf16_rounding_noise_floor():
    """Why bf16 shapes are compared with a logit tolerance of a few 1e-2: a relative perturbation of
    1e-7 (fp32-vs-float64 summation order) in front of the bf16 rounding points is amplified to bf16
    rounding noise within a couple of layers, while the same perturbation leaves a model without
    operand rounding unchanged to ~1e-6."""
    shape = synth.Shape("noise", 2, 256, 4, 512, 512, 0, 512, 8, 8, 4, synth.PREFIX_DENSE, 1, 6, None,
                        synth.DTYPE_BF16, 7.5, seed=5)
    w = synth.make_weights(shape)
    outs = {}
    for dtype in (synth.DTYPE_BF16, synth.DTYPE_FP32):
        for eps in (0.0, 1e-7):
            o = vo.Oracle(dataclasses.asdict(shape.replace(dtype=dtype)), w)
            if eps:
                base, rng = o.rb, np.random.default_rng(1)
                o.rb = lambda x, base=base, rng=rng: base(np.asarray(x, dtype=np.float64) * (1 + eps * rng.standard_normal(np.shape(x))))
            run_prefill(o, shape, n_forced=10)
            parent = synth.tree_parents(None, shape.n_nodes)
            q, toks = synth.make_draft(shape, parent, 0)
            o.verify(parent, toks, q, synth.make_uniforms(shape, shape.n_nodes, 0))
            outs[(dtype, eps)] = o.raw_logits.copy()
    noise_bf16 = np.abs(outs[(1, 1e-7)] - outs[(1, 0.0)]).max()
    noise_exact = np.abs(outs[(0, 1e-7)] - outs[(0, 0.0)]).max()
    assert noise_exact < 1e-5
    assert 1e-3 < noise_bf16 < 3e-2, noise_bf16
