"""GPU edge cases through the C ABI, against the CPU checker: degenerate distributions in the
acceptance stage, the largest tree a call may carry, bushy sibling groups, several prompts at ragged
progress with some of them finished, and a second prefill on a used context."""
import numpy as np
import pytest
import torch

from paper_2511_13587_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gc():
    from tests import gpu_common
    return gpu_common


def run_accept(gc, pair, shape, parent, raw, toks, q, u, mode=0, nbr=None):
    from oracle import vvs_oracle as vo
    dev = pair.dev
    N = len(parent)
    B = shape.n_prompts
    pair.ctx.vvs_accept_from_logits(N, parent, None, torch.from_numpy(np.ascontiguousarray(raw, dtype=np.float32)).to(dev),
                                    torch.from_numpy(np.ascontiguousarray(toks, dtype=np.int32)).to(dev),
                                    torch.from_numpy(np.ascontiguousarray(q, dtype=np.float32)).to(dev),
                                    torch.from_numpy(np.ascontiguousarray(u, dtype=np.float32)).to(dev), mode,
                                    pair.accept_len, pair.path, pair.next_token)
    torch.cuda.synchronize()
    out = (pair.accept_len.cpu().numpy(), pair.path.cpu().numpy(), pair.next_token.cpu().numpy())
    T, V = N + 1, shape.v_eff
    lc, lu = raw.reshape(B, 2, T, V)[:, 0].astype(np.float64), raw.reshape(B, 2, T, V)[:, 1].astype(np.float64)
    p = vo.softmax(lu + shape.cfg_scale * (lc - lu))
    a_o, paths_o, next_o, traces = [], [], [], []
    for b in range(B):
        tr = {}
        a, path, nxt = vo.decide(p[b], q[b].astype(np.float64), toks[b] - shape.logit_lo, parent, u[b].astype(np.float64),
                                 10 ** 9, mode, nbr, shape.relax_k, shape.relax_delta, shape.logit_lo, trace=tr)
        a_o.append(a); paths_o.append(path); next_o.append(shape.logit_lo + nxt); traces.append(tr)
    return out, (np.array(a_o), paths_o, np.array(next_o)), traces


def test_accept_stage_degenerate_distributions(gc):
    """Zero draft mass on the drafted id (accept iff the target has mass there), zero target mass,
    a draft distribution that the sibling draws exhaust, a target that equals the draft (residual
    without mass), one-hot targets: decisions equal the checker's exactly (every margin is wide)."""
    shape = synth.TINY.replace(n_layers=1, d_model=64, n_heads=2, d_ff=64, n_prompts=4, prefix_len=1, n_nodes=4, cfg_scale=1.0)
    pair = gc.Pair(shape, with_oracle=False)
    V, B = shape.v_eff, shape.n_prompts
    parent = np.array([0, 0, 0, 1], dtype=np.int32)             # three siblings below the root, node 4 below node 1
    T = 5
    NEG = -1.0e4                                                 # exp underflows to an exact 0 in fp32 and in float64
    lc = np.full((B, T, V), NEG, dtype=np.float32)
    toks = np.zeros((B, 4), dtype=np.int32)
    q = np.zeros((B, T, V), dtype=np.float32)
    u = np.full((B, T, 2), 0.5, dtype=np.float32)
    # prompt 0: siblings 10, 11, 12; draft mass only on those three; target: all mass on id 12 -> 10 and 11 are rejected
    # (target 0 there), the draft renormalises twice, 12 is accepted; below node... path [0, 3]
    toks[0] = [10, 11, 12, 13]
    q[0, 0, [10, 11, 12]] = [0.5, 0.3, 0.2]
    lc[0, 0, 12] = 0.0
    lc[0, 3, 40] = 0.0                                           # node 3 is a leaf: the next token comes from its target = id 40
    # prompt 1: the draft gives the drafted id no mass at all, the target does -> accepted at once (u * 0 < p)
    toks[1] = [20, 21, 22, 23]
    q[1, 0, [21, 22, 30]] = [0.3, 0.3, 0.4]
    lc[1, 0, [20, 31]] = [0.0, 0.0]                              # target 0.5 / 0.5 on ids 20 and 31
    q[1, 1, 23] = 1.0                                            # node 1's child (node 4, id 23): draft sure, target elsewhere -> rejected
    lc[1, 1, 50] = 0.0
    # prompt 2: neither draft nor target has mass on the drafted ids: 0/0 rejects all three, the draft is exhausted after
    # its own support is gone; the residual equals the target
    toks[2] = [60, 61, 62, 63]
    q[2, 0, 70] = 1.0
    lc[2, 0, [80, 81]] = [0.0, 0.0]
    u[2, 0, 1] = 0.75                                            # terminal draw at the root: second half of the CDF -> id 81
    # prompt 3: target == draft on two ids; drafted id 90 rejected by a large uniform -> residual has no mass -> the target stays
    toks[3] = [90, 91, 92, 93]
    q[3, 0, [90, 91]] = [0.5, 0.5]
    lc[3, 0, [90, 91]] = [0.0, 0.0]
    u[3, 1, 0] = 0.999                                           # rejects node 1 (id 90): u * 0.5 < 0.5 is false only for u >= 1 -> accepted
    lc[:, :, 0] = np.where(np.all(lc == NEG, axis=2), 0.0, lc[:, :, 0])   # rows nobody set: all mass on id 0
    lu = lc.copy()                                               # cfg scale 1 and equal rows: mixed = lc
    raw = np.stack([lc, lu], axis=1).reshape(2 * B, T, V)
    out, oout, traces = run_accept(gc, pair, shape, parent, raw, toks, q, u)
    for b in range(B):
        assert out[0][b] == oout[0][b], (b, out[0], oout[0])
        assert list(out[1][b][:out[0][b] + 1]) == list(oout[1][b]), (b, out[1][b][:6], oout[1][b])
        assert out[2][b] == oout[2][b], (b, out[2], oout[2])
    assert list(oout[1][0]) == [0, 3] and oout[2][0] == 40
    assert oout[0][1] == 1 and oout[2][1] == 50
    assert oout[0][2] == 0 and oout[2][2] == 81
    pair.close()


@pytest.mark.parametrize("kind", ["chain", "star", "random"])
def test_largest_tree_fp32(gc, kind):
    """63 draft nodes (64 query tokens per row, the most a call may carry): a chain, a root with 63
    children (63 sibling draws without replacement), a random tree.  Logits 1e-4 and decisions
    against the checker."""
    N = 63
    shape = synth.TINY.replace(n_nodes=N, grid_h=12, grid_w=12)
    rng = np.random.default_rng(9)
    parent = {"chain": np.arange(N), "star": np.zeros(N, dtype=np.int64),
              "random": np.array([int(rng.integers(0, j)) for j in range(1, N + 1)])}[kind].astype(np.int32)
    pair = gc.Pair(shape, gain_jitter=0.1)
    pair.prefill(n_forced=10)
    q, toks = synth.make_draft(shape, parent, 0)
    u = synth.make_uniforms(shape, N, 0)
    state = torch.from_numpy(pair.ctx.vvs_read_state()).to(pair.dev)
    out, oout = pair.verify(parent, toks, q, u)
    gc.check_logits(pair, kind)
    gc.decisions_match(out, oout, pair.oracle.traces, shape.logit_lo)
    pair.ctx.vvs_set_state(state)                                # drop this verify (not committed) on both sides
    pair.oracle.last = None
    # a draft that follows the target: long accepted paths
    q2, toks2 = synth.make_draft(shape.replace(draft_noise_std=0.2), parent, 1, base_logits=pair.oracle.mixed_logits.astype(np.float32))
    out, oout = pair.verify(parent, toks2, q2, synth.make_uniforms(shape, N, 1))
    gc.decisions_match(out, oout, pair.oracle.traces, shape.logit_lo)
    if (out[0] == oout[0]).all() and (out[2] == oout[2]).all():
        pair.commit()
        st = pair.ctx.vvs_read_state()
        assert st[0, 0] == pair.oracle.kv_len(0) and st[1, 0] == pair.oracle.n_emitted[0]
        S = pair.oracle.kv_len(0)
        k, v = pair.ctx.vvs_debug_kv(shape.n_layers - 1, 1, S)
        assert np.abs(k.cpu().numpy() - pair.oracle.kc[1][shape.n_layers - 1].reshape(S, -1)).max() < 1e-4
        assert np.abs(v.cpu().numpy() - pair.oracle.vc[1][shape.n_layers - 1].reshape(S, -1)).max() < 1e-4
    pair.close()


def test_ragged_prompts_some_finished_fp32(gc):
    """Three prompts on a 3 x 3 grid driven to the end: they accept different numbers of tokens per
    call, so their cache lengths diverge and they finish in different calls; a finished prompt must
    return accept_len 0 / next -1 and stay untouched while the others go on.  Then a second prefill on
    the same context starts over."""
    shape = synth.TINY.replace(n_prompts=3, grid_h=3, grid_w=3, n_nodes=3)
    pair = gc.Pair(shape, gain_jitter=0.1)
    first, ofirst, _ = pair.prefill()
    assert (first == ofirst).all()
    parent = np.array([0, 0, 1], dtype=np.int32)
    seen_ragged = seen_finished_with_running = False
    for it in range(12):
        q, toks = synth.make_draft(shape, parent, it)
        if it % 2:                                               # every other call: a draft close to the target of the previous call
            q, toks = synth.make_draft(shape.replace(draft_noise_std=0.3), parent, it, base_logits=pair.oracle.mixed_logits.astype(np.float32))
        u = synth.make_uniforms(shape, 3, it)
        out, oout = pair.verify(parent, toks, q, u)
        gc.check_logits(pair, f"call {it}")
        gc.decisions_match(out, oout, pair.oracle.traces, shape.logit_lo)
        if not ((out[0] == oout[0]).all() and (out[2] == oout[2]).all()):
            break
        done = pair.oracle.n_emitted >= shape.grid
        for b in range(3):
            if done[b]:
                assert out[0][b] == 0 and out[2][b] == -1
        seen_finished_with_running |= bool(done.any() and not done.all())
        pair.commit()
        st = pair.ctx.vvs_read_state()
        for b in range(3):
            assert st[0, b] == pair.oracle.kv_len(b) and st[1, b] == pair.oracle.n_emitted[b] and st[2, b] == pair.oracle.pending[b]
        seen_ragged |= len(set(int(x) for x in st[0])) > 1
        if done.all():
            break
    assert seen_ragged and seen_finished_with_running
    assert (pair.oracle.n_emitted == shape.grid).all()
    for row in range(shape.n_rows):
        S = pair.oracle.kv_len(row // 2)
        k, v = pair.ctx.vvs_debug_kv(0, row, S)
        assert np.abs(k.cpu().numpy() - pair.oracle.kc[row][0].reshape(S, -1)).max() < 1e-4
        assert np.abs(v.cpu().numpy() - pair.oracle.vc[row][0].reshape(S, -1)).max() < 1e-4
    # a second prefill resets everything, the feature rings included
    first2, ofirst2, _ = pair.prefill(n_forced=2)
    assert (first2 == ofirst2).all()
    st = pair.ctx.vvs_read_state()
    assert (st[0] == shape.prefix_len + 2).all() and (st[1] == 3).all()
    feats, count = pair.ctx.vvs_read_features()
    assert (count == 1).all()
    for row in range(shape.n_rows):
        assert np.abs(feats[row, 0] - pair.oracle.features(row)[0]).max() < 1e-4
    pair.close()


def test_rerun_is_bit_identical_bf16(gc):
    """No kernel of the path uses atomics or an order that depends on scheduling: the same verify call on
    the same state gives bit-identical logits, probabilities and outcome, and so does the same drafting
    call (XL width, 2 layers, the 26-node tree)."""
    shape = synth.XL_TREE.replace(n_layers=2)
    parent = synth.tree_parents(shape.tree_widths, shape.n_nodes)
    pair = gc.Pair(shape, with_oracle=False)
    pair.prefill(n_forced=45, run_oracle=False)
    state = torch.from_numpy(pair.ctx.vvs_read_state()).to(pair.dev)
    q, toks = synth.make_draft(shape, parent, 0)
    u = synth.make_uniforms(shape, shape.n_nodes, 0)
    runs = []
    for _ in range(3):
        pair.ctx.vvs_set_state(state)
        out, _ = pair.verify(parent, toks, q, u, run_oracle=False, mask=synth.ancestor_mask(parent))
        raw, mixed, probs = pair.gpu_logits()
        runs.append((out, raw, probs))
    for out, raw, probs in runs[1:]:
        assert np.array_equal(raw, runs[0][1]) and np.array_equal(probs, runs[0][2])
        assert all(np.array_equal(a, b) for a, b in zip(out, runs[0][0]))
    pair.commit(run_oracle=False)
    vb = gc.vb
    n_exp = len(set(int(p) for p in parent if p > 0))
    dctx = vb.Context(vb.make_config(shape.replace(n_layers=1), max_nodes=5 + n_exp - 1, feature_slots=0, draft_input=1))
    dctx.load_weights_from_host(synth.make_drafter_weights(shape, pair.w), synth.drafter_weight_names())
    recent = torch.from_numpy(np.random.default_rng(2).integers(0, shape.vocab, (shape.n_prompts, 5)).astype(np.int32)).to(pair.dev)
    got = []
    for _ in range(3):
        tok = torch.zeros((shape.n_prompts, shape.n_nodes), dtype=torch.int32, device=pair.dev)
        dq = torch.zeros((shape.n_prompts, shape.n_nodes + 1, shape.v_eff), dtype=torch.float32, device=pair.dev)
        dctx.vvs_draft(pair.ctx, shape.n_nodes, parent, None, 5, recent, 0, None, tok, dq)
        torch.cuda.synchronize()
        got.append((tok.cpu().numpy(), dq.cpu().numpy()))
    for tok, dq in got[1:]:
        assert np.array_equal(tok, got[0][0]) and np.array_equal(dq, got[0][1])
    dctx.close()
    pair.close()


def test_hip_graph_replay_of_a_whole_step_bf16(gc):
    """A step (roll back the state, draft, verify, commit) is captured once into a HIP graph - the library only
    launches kernels, it records no memset or copy node - and replayed several times with eager work and
    synchronisations in between; every replay must reproduce the eager results bit for bit."""
    shape = synth.XL_TREE.replace(n_layers=2)
    parent = synth.tree_parents(shape.tree_widths, shape.n_nodes)
    mask = synth.ancestor_mask(parent)
    N, B = shape.n_nodes, shape.n_prompts
    pair = gc.Pair(shape, with_oracle=False)
    pair.prefill(n_forced=45, run_oracle=False)
    vb = gc.vb
    dev = pair.dev
    n_exp = len(set(int(p) for p in parent if p > 0))
    dctx = vb.Context(vb.make_config(shape.replace(n_layers=1), max_nodes=1 + n_exp - 1, feature_slots=0, draft_input=1))
    dctx.load_weights_from_host(synth.make_drafter_weights(shape, pair.w), synth.drafter_weight_names())
    state = torch.from_numpy(pair.ctx.vvs_read_state()).to(dev)
    recent = torch.from_numpy(pair.ctx.vvs_read_state()[2:3].T.copy()).to(dev)          # the pending tokens
    u = torch.from_numpy(synth.make_uniforms(shape, N, 0)).to(dev)
    tok = torch.zeros((B, N), dtype=torch.int32, device=dev)
    dq = torch.zeros((B, N + 1, shape.v_eff), dtype=torch.float32, device=dev)

    def step():
        pair.ctx.vvs_set_state(state)
        dctx.vvs_draft(pair.ctx, N, parent, None, 1, recent, 0, None, tok, dq)
        pair.ctx.vvs_verify(N, parent, mask, tok, dq, u, 0, pair.accept_len, pair.path, pair.next_token)
        pair.ctx.vvs_kv_commit()

    def snapshot():
        torch.cuda.synchronize()
        k, v = pair.ctx.vvs_debug_kv(1, 3, int(state[0, 1].item()) + 4)
        return [t.cpu().numpy().copy() for t in (tok, dq, pair.accept_len, pair.path, pair.next_token, k, v)] + [pair.ctx.vvs_read_state()]

    step()          # the first commit replaces the prefill's feature by the committed path's: from the second
    step()          # step on, the newest cached feature - the drafter's input here - is the same every time
    want = snapshot()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                                          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for i in range(3):
        tok.fill_(-1)
        dq.fill_(0.5)
        pair.accept_len.fill_(77)
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert np.array_equal(a, b), f"replay {i} differs from the eager step"
        step()                                                          # eager work between the replays
        for a, b in zip(snapshot(), want):
            assert np.array_equal(a, b)
    dctx.close()
    pair.close()


@pytest.mark.parametrize("mode", [0, 1])
def test_fill_probe_reads_the_region_it_is_given(gc, mode):
    """The L1 fill probe (a measurement aid): its checksum says that thread 0 of every workgroup read exactly the blocks
    the declaration describes, for a region that is not a multiple of the 8 blocks x waves in flight; the direct-to-LDS
    variant leaves 0; arguments out of range are refused before any launch."""
    vb = gc.vb
    ctx = vb.Context(vb.make_config(synth.TINY))
    n_blocks, waves, reps, wgs = 40, 3, 2, 5                  # 40 KiB: 24 blocks per round, then 16
    words = np.random.default_rng(7).integers(0, 2**32, size=n_blocks * 256, dtype=np.uint64).astype(np.uint32)
    src = torch.from_numpy(words.view(np.int32)).to(ctx.device)
    def expected(first_block, blocks):
        want = 0
        if mode == 0:
            for _ in range(reps):
                for blk in range(0, blocks, waves * 8):
                    for u in range(8):
                        b = first_block + min(blk + u * waves, blocks - 1)
                        want = (want + int(words[b * 256] ^ words[b * 256 + 1] ^ words[b * 256 + 2] ^ words[b * 256 + 3])) & 0xFFFFFFFF
        return want
    sink = ctx.vvs_debug_fill_probe(src, reps, mode, wgs, waves).cpu().numpy().view(np.uint32)
    assert (sink == expected(0, n_blocks)).all()
    # a region of 8 blocks of its own per workgroup
    sink = ctx.vvs_debug_fill_probe(src, reps, mode, wgs, waves, region_bytes=8192, wg_stride_bytes=8192).cpu().numpy().view(np.uint32)
    assert [int(v) for v in sink] == [expected(8 * w, 8) for w in range(wgs)]
    with pytest.raises(vb.VvsError):
        ctx.vvs_debug_fill_probe(src, reps, mode, wgs, 17)
    with pytest.raises(vb.VvsError):
        ctx.vvs_debug_fill_probe(src[:1000], reps, mode, wgs, waves)
    ctx.close()


@pytest.mark.parametrize("case", ["xl_27_tokens", "xl_61_tokens_few_prompts", "xl_61_tokens_many_prompts", "head_size_128"])
def test_which_launches_a_layer_takes(gc, case):
    """The launch plan is part of what the library promises to measure with (vvs_timing_read): a verify call runs the q/k/v
    projection and the attention of a layer as one launch at head size 64 with up to 32 tokens per row, and with up to 64
    tokens while there are at most 512 (head, prompt) pairs; otherwise, and at head size 128, as separate launches."""
    vb = gc.vb
    if case == "xl_27_tokens":
        shape, fused_attention = synth.XL_TREE.replace(n_layers=2, n_prompts=2), True
    elif case == "xl_61_tokens_few_prompts":
        shape, fused_attention = synth.XL_STRESS.replace(n_layers=2, n_prompts=2), True
    elif case == "xl_61_tokens_many_prompts":
        shape, fused_attention = synth.XL_STRESS.replace(n_layers=1, n_prompts=26), False     # 520 pairs
    else:
        shape, fused_attention = synth.SEVEN_B.replace(n_layers=2, d_model=1024, n_heads=8, d_ff=2752), False
    parent = synth.tree_parents(shape.tree_widths, shape.n_nodes)
    pair = gc.Pair(shape, with_oracle=False)
    pair.prefill(n_forced=10, run_oracle=False)
    q, toks = synth.make_draft(shape, parent, 0)
    u = synth.make_uniforms(shape, shape.n_nodes, 0)
    pair.ctx.vvs_timing_enable(True)
    pair.verify(parent, toks, q, u, run_oracle=False)
    n_attention, _ = pair.ctx.vvs_timing_read(vb.VVS_K_ATTENTION)
    pair.ctx.vvs_timing_enable(False)
    assert n_attention == (0 if fused_attention else shape.n_layers)
