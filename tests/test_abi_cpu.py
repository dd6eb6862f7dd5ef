"""Host-side checks of libvvs that need no GPU: the library loads, exports every function that
include/vvs.h declares, sizes buffers sensibly, and rejects bad shapes and bad draft trees before
anything could be launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2511_13587_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_13587_amd", "libvvs.so")


@pytest.fixture(scope="module")
def binding():
    if not os.path.exists(LIB):
        from paper_2511_13587_amd import build
        build.build(verbose=False)
    from paper_2511_13587_amd import binding as b
    return b


def declared_functions():
    text = open(os.path.join(ROOT, "include", "vvs.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vvs_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(binding):
    names = declared_functions()
    assert {"vvs_prefill", "vvs_verify", "vvs_kv_commit"} <= set(names)
    raw = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(raw, n), f"{n} declared in vvs.h but not exported"
    assert set(binding.EXPORTS) == set(names)


def test_query_sizes_for_the_five_workloads(binding):
    for shape in synth.SHAPES.values():
        cfg = binding.make_config(shape)
        kv, ws, pw = binding.vvs_query_sizes(cfg)
        esz = 2 if shape.dtype == synth.DTYPE_BF16 else 4
        n_par = shape.n_layers * (4 * shape.d_model ** 2 + 3 * shape.d_model * shape.d_ff)
        assert pw >= esz * (n_par + shape.d_model * shape.v_eff + shape.vocab * shape.d_model)
        assert pw < 1.05 * esz * (n_par + shape.d_model * shape.v_eff + (shape.vocab + 1001) * shape.d_model) + (1 << 20)
        slots = shape.prefix_len + shape.grid + 64
        assert kv >= 2 * esz * shape.n_layers * shape.n_rows * slots * shape.d_model
        assert kv % 256 == 0 and ws % 256 == 0 and pw % 256 == 0 and ws > 0


@pytest.mark.parametrize("field,value,status", [
    ("d_ff", 2000, -3),        # bf16: not a multiple of 64
    ("n_heads", 7, -1),        # does not divide d_model
    ("logit_hi", 99999, -1),   # slice outside the vocabulary
    ("max_nodes", 64, -3),     # more than VVS_MAX_T - 1 draft nodes
    ("dtype", 5, -1),
    ("n_prompts", 0, -1),
    ("relax_k", 65, -3),
])
def test_query_sizes_rejects_bad_shapes(binding, field, value, status):
    cfg = binding.make_config(synth.B_SHAPE)
    setattr(cfg, field, value)
    with pytest.raises(binding.VvsError) as e:
        binding.vvs_query_sizes(cfg)
    assert e.value.status == status


def test_head_size_rules(binding):
    cfg = binding.make_config(synth.B_SHAPE.replace(n_heads=24))       # bf16 with head size 32
    with pytest.raises(binding.VvsError):
        binding.vvs_query_sizes(cfg)
    cfg = binding.make_config(synth.TINY.replace(d_model=120, n_heads=4))  # fp32, head size 30
    with pytest.raises(binding.VvsError):
        binding.vvs_query_sizes(cfg)
    binding.vvs_query_sizes(binding.make_config(synth.TINY))


def test_check_tree_accepts_the_workload_trees(binding):
    for shape in (synth.XL_TREE, synth.XL_STRESS, synth.B_SHAPE):
        parent = synth.tree_parents(shape.tree_widths, shape.n_nodes)
        mask = synth.ancestor_mask(parent)
        for p, m in ((parent, mask), (parent, None), (None, mask)):
            st, depth, pout = binding.vvs_check_tree(shape.n_nodes, p, m)
            assert st == 0
            assert (depth == synth.node_depths(parent)).all() and (pout == parent).all()
    st, depth, pout = binding.vvs_check_tree(5, None, None)     # both NULL: a chain
    assert st == 0 and (depth == np.arange(6)).all() and (pout == np.arange(5)).all()
    st, depth, _ = binding.vvs_check_tree(0, None, None)
    assert st == 0 and depth.tolist() == [0]


def test_check_tree_rejects_malformed_input(binding):
    assert binding.vvs_check_tree(3, np.array([0, 2, 1]), None)[0] == -1        # parent after child
    assert binding.vvs_check_tree(3, np.array([0, -1, 1]), None)[0] == -1
    assert binding.vvs_check_tree(64, np.zeros(64, dtype=np.int32), None)[0] == -3
    assert binding.vvs_check_tree(-1, None, None)[0] == -3
    parent = np.array([0, 0, 1])
    mask = synth.ancestor_mask(parent)
    bad = mask.copy(); bad[3, 2] = 1                                            # sibling marked visible
    assert binding.vvs_check_tree(3, parent, bad)[0] == -1
    bad = mask.copy(); bad[2, 0] = 0                                            # root hidden
    assert binding.vvs_check_tree(3, parent, bad)[0] == -1
    assert binding.vvs_check_tree(3, None, bad)[0] == -1
    bad = mask.copy(); bad[1, 3] = 1                                            # looks ahead
    assert binding.vvs_check_tree(3, parent, bad)[0] == -1
    assert binding.vvs_check_tree(3, np.array([0, 1, 2]), mask)[0] == -1        # mask of another tree


def test_select_unverified_and_skip_rules_match_the_checker(binding):
    """Host-only logic of the verification-free step (Section 4.2, Eq. 1; Section 4.4; Algorithm 1):
    the library's answers equal the CPU checker's on random trees and uniforms."""
    from oracle import vvs_schedule as vs
    rng = np.random.default_rng(5)
    for trial in range(200):
        n = int(rng.integers(0, 40))
        parent = np.array([int(rng.integers(0, j)) for j in range(1, n + 1)], dtype=np.int32)
        u = np.float32(rng.random())
        if u >= 1.0:
            u = np.float32(0.5)
        st, kept = binding.vvs_select_unverified(n, parent if n else None, None, float(u))
        assert st == binding.VVS_OK
        assert list(kept) == vs.select_unverified(parent, float(u)), (parent, u)
    # the synthetic benchmark trees, from the ancestor mask alone
    for widths, n in (((4, 6, 6, 4, 3, 3), 26), ((8, 12, 12, 10, 8, 6, 4), 60)):
        parent = synth.tree_parents(widths, n)
        st, kept = binding.vvs_select_unverified(n, None, synth.ancestor_mask(parent), 0.37)
        assert st == binding.VVS_OK and list(kept) == vs.select_unverified(parent, np.float32(0.37))
    st, _ = binding.vvs_select_unverified(3, np.array([0, 0, 1], dtype=np.int32), None, 1.0)
    assert st == binding.VVS_EINVAL
    st, _ = binding.vvs_select_unverified(3, np.array([0, 2, 1], dtype=np.int32), None, 0.5)       # parent after child
    assert st == binding.VVS_EINVAL
    for i in range(0, 6):
        for t in range(20):
            assert binding.vvs_skip_uniform(t, i) == vs.skip_uniform(t, i)
    for s, thr, last in ((0.81, 0.8, True), (0.8, 0.8, True), (0.79, 0.8, True), (0.99, 0.8, False)):
        assert binding.vvs_skip_dynamic(s, thr, last) == vs.skip_dynamic(np.float32(s), np.float32(thr), last)
