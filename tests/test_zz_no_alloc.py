"""The allocation-free acceptance entry point (static device scratch) against the ordinary one, through the
C ABI: identical outcomes on two calls in a row, the second with a smaller input; size limits are errors."""
import numpy as np
import pytest
import torch

from paper_2511_13587_amd import synth

pytestmark = pytest.mark.gpu


def run_both(pair, shape, parent, seed, mode=0):
    vb_dev = pair.dev
    T, V, B = shape.n_nodes + 1, shape.v_eff, shape.n_prompts
    rng = np.random.default_rng(seed)
    raw = rng.standard_normal((2 * B, T, V)).astype(np.float32)
    q, toks = synth.make_draft(shape, parent, seed)
    u = synth.make_uniforms(shape, shape.n_nodes, seed)
    args = (shape.n_nodes, parent, None, torch.from_numpy(raw).to(vb_dev), torch.from_numpy(toks).to(vb_dev), torch.from_numpy(q).to(vb_dev),
            torch.from_numpy(u).to(vb_dev), mode)
    outs = []
    for fn in (pair.ctx.vvs_accept_from_logits, pair.ctx.vvs_accept_from_logits_noalloc):
        a = torch.full((B,), -7, dtype=torch.int32, device=vb_dev)
        path = torch.full((B, 64), -7, dtype=torch.int32, device=vb_dev)
        nxt = torch.full((B,), -7, dtype=torch.int32, device=vb_dev)
        fn(*args, a, path, nxt)
        torch.cuda.synchronize()
        outs.append((a.cpu().numpy(), path.cpu().numpy(), nxt.cpu().numpy()))
    for x, y in zip(*outs):
        assert (x == y).all()
    assert (outs[1][0] >= 0).all() and (outs[1][2] >= shape.logit_lo).all()
    return outs[1]


def test_noalloc_accept_matches_workspace_accept():
    import gpu_common as gc
    # first call: the 26-node tree of the XL workload, 6 prompts, 16384 ids (about 2.7 M scratch floats)
    big = synth.XL_TREE.replace(n_layers=1, d_model=64, n_heads=1, d_ff=64, n_prompts=6, prefix_len=1)
    pair = gc.Pair(big, with_oracle=False)
    parent = synth.tree_parents(big.tree_widths, big.n_nodes)
    run_both(pair, big, parent, 1)
    pair.close()
    # second call, smaller: a chain of 4 over 1024 ids, one prompt; the array still holds the first call's data
    small = synth.TINY
    pair = gc.Pair(small, with_oracle=False)
    run_both(pair, small, synth.tree_parents(None, small.n_nodes), 2)
    pair.close()
    # relaxed mode, and the first size again
    nbr = synth.make_codebook_neighbours(big.vocab, 50)
    big_r = big.replace(relax_k=50, relax_delta=0.2)
    pair = gc.Pair(big_r, with_oracle=False)
    pair.set_neighbors(nbr)
    run_both(pair, big_r, parent, 3, mode=1)
    pair.close()


def test_noalloc_accept_rejects_what_does_not_fit():
    import gpu_common as gc
    vb = gc.vb
    shape = synth.XL_TREE.replace(n_layers=1, d_model=64, n_heads=1, d_ff=64, n_prompts=12, prefix_len=1)   # 12 * 27 * 16384 floats > 4 Mi
    pair = gc.Pair(shape, with_oracle=False)
    parent = synth.tree_parents(shape.tree_widths, shape.n_nodes)
    T, V, B = shape.n_nodes + 1, shape.v_eff, shape.n_prompts
    dev = pair.dev
    z = lambda *s, dt=torch.float32: torch.zeros(s, dtype=dt, device=dev)
    with pytest.raises(vb.VvsError) as e:
        pair.ctx.vvs_accept_from_logits_noalloc(shape.n_nodes, parent, None, z(2 * B, T, V), z(B, T - 1, dt=torch.int32), z(B, T, V), z(B, T, 2), 0,
                                                pair.accept_len, pair.path, pair.next_token)
    assert e.value.status == vb.VVS_ESIZE
    torch.cuda.synchronize()
    pair.close()
