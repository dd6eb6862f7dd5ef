"""Pins for the CPU checker's acceptance procedure (oracle/vvs_oracle.py: decide, inverse_cdf,
relaxed_target) against what the paper and the mathematics fix (Section 2, "Speculative Decoding"):
hand-worked numbers, the closed form min(1, p/q), losslessness by exhaustive enumeration, and the
invariants of the relaxed rule.

The probabilities of the procedure's outcomes are *measured from the procedure itself*: an outcome
is a step function of each uniform, so its breakpoints are found by bisection on calls of `decide`
(no formula of the procedure is retyped here)."""
import itertools
import os

import numpy as np
import pytest

from oracle.vvs_oracle import decide, inverse_cdf, relaxed_target

ONE = 1.0 - 2.0 ** -53     # largest uniform below 1
GOLD = os.path.join(os.path.dirname(__file__), "golden", "sd_worked_example.txt")


def read_golden():
    out = {}
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out[k] = np.array([float(t) for t in v])
    return out


def sup_true(f):
    """sup{u in [0,1): f(u)} for f true on [0, t) and false on [t, 1)."""
    if f(ONE):
        return 1.0
    if not f(0.0):
        return 0.0
    lo, hi = 0.0, ONE
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if f(mid):
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def step_measure(g, V):
    """g(u) -> id is non-decreasing in u; returns the length of {u: g(u) = y} for every y."""
    cdf = np.array([sup_true(lambda u, y=y: g(u) <= y) for y in range(V)])
    return np.diff(np.concatenate([[0.0], cdf]))


def chain1(p0, q0, x, u_acc, u_term0, u_term1=0.5, p1=None, **kw):
    """One drafted token x below the root."""
    V = len(p0)
    p_rows = np.stack([p0, p0 if p1 is None else p1])
    q_rows = np.stack([q0, q0])
    u = np.array([[0.5, u_term0], [u_acc, u_term1]])
    return decide(p_rows, q_rows, np.array([x]), np.array([0]), u, cap=10, **kw)


def accept_prob(p0, q0, x, **kw):
    return sup_true(lambda u: chain1(p0, q0, x, u, 0.5, **kw)[0] == 1)


def reject_dist(p0, q0, x, **kw):
    return step_measure(lambda u: chain1(p0, q0, x, ONE, u, **kw)[2], len(p0))


def rand_dist(rng, V, sparsity=0.0):
    w = rng.random(V) ** 2
    if sparsity:
        w[rng.random(V) < sparsity] = 0.0
        w[rng.integers(V)] += 0.1
    return w / w.sum()


# ------------------------------------------------------------------------------------------------
def test_golden_worked_example():
    g = read_golden()
    for p, q, acc, res, tot in ((g["p"], g["q"], g["accept"], g["resid"], g["total_accept"]),
                                (g["p2"], g["q2"], g["accept2"], g["resid2"], g["total_accept2"])):
        V = len(p)
        got_acc = np.array([accept_prob(p, q, x) for x in range(V)])
        assert np.allclose(got_acc, acc, atol=1e-12)
        assert abs(float(np.dot(q, got_acc)) - float(tot[0])) < 1e-12
        for x in range(V):
            if got_acc[x] < 1.0:
                assert np.allclose(reject_dist(p, q, x), res, atol=1e-12)


def test_golden_relaxed_example():
    g = read_golden()
    p, q = g["p2"], g["q2"]
    nbr = np.array([[2, 1], [0, 2], [1, 0]])
    num, pt = relaxed_target(p.copy(), 0, nbr[0], 2, 0.35)
    assert abs(num - g["relaxed_num"][0]) < 1e-15
    assert np.allclose(pt, g["relaxed_target"], atol=1e-15)
    kw = dict(mode=1, nbr=nbr, relax_k=2, relax_delta=0.35)
    assert abs(accept_prob(p, q, 0, **kw) - g["relaxed_accept"][0]) < 1e-12
    # after a relaxed rejection the replacement comes from the positive part of (modified target - q)
    # = (0, 0.3, 0) -> id 1 with certainty
    assert np.allclose(reject_dist(p, q, 0, **kw), [0.0, 1.0, 0.0], atol=1e-12)


@pytest.mark.parametrize("V", [2, 3, 7, 50])
def test_accept_closed_form(V):
    rng = np.random.default_rng(V)
    for _ in range(5):
        p, q = rand_dist(rng, V), rand_dist(rng, V)
        thr = np.array([accept_prob(p, q, x) for x in range(V)])
        assert np.allclose(thr, np.minimum(1.0, p / q), atol=1e-12)
        # overall acceptance = sum_x min(p, q) = 1 - TV(p, q)
        assert abs(np.dot(q, thr) - (1.0 - 0.5 * np.abs(p - q).sum())) < 1e-12


def test_zero_mass_conventions():
    p = np.array([0.5, 0.5, 0.0, 0.0])
    q = np.array([0.0, 0.5, 0.5, 0.0])
    assert accept_prob(p, q, 0) == 1.0      # draft mass 0, target mass > 0: always accepted
    assert accept_prob(p, q, 2) == 0.0      # target mass 0: never accepted
    assert accept_prob(p, q, 3) == 0.0      # 0/0 rejects


def test_identical_and_disjoint():
    rng = np.random.default_rng(5)
    V, K = 9, 4
    p_rows = np.stack([rand_dist(rng, V) for _ in range(K + 1)])
    toks = rng.integers(0, V, size=K)
    parent = np.arange(K)
    for trial in range(20):
        u = rng.random((K + 1, 2))
        a, path, nxt = decide(p_rows, p_rows, toks, parent, u, cap=100)     # q == p: accept all
        assert a == K and path == list(range(K + 1))
        assert nxt == inverse_cdf(p_rows[K], u[K, 1])                         # bonus from the last row
    # the bonus token follows the last target distribution
    g = lambda uu: decide(p_rows, p_rows, toks, parent, np.array([[0.5, 0.5]] * K + [[0.5, uu]]), cap=100)[2]
    assert np.allclose(step_measure(g, V), p_rows[K], atol=1e-12)
    # disjoint supports: reject at the first node, replacement drawn from p itself
    p = np.array([0.3, 0.7, 0.0, 0.0])
    q = np.array([0.0, 0.0, 0.4, 0.6])
    assert accept_prob(p, q, 2) == 0.0 and accept_prob(p, q, 3) == 0.0
    assert np.allclose(reject_dist(p, q, 3), p, atol=1e-12)


@pytest.mark.parametrize("V", [2, 3, 4, 6, 8])
def test_lossless_single_draft(V):
    """Emitted-token marginal of draft-one/verify-one equals the target exactly."""
    rng = np.random.default_rng(100 + V)
    for sparsity in (0.0, 0.4):
        p, q = rand_dist(rng, V, sparsity), rand_dist(rng, V, sparsity)
        out = np.zeros(V)
        for x in range(V):
            if q[x] == 0:
                continue
            t = accept_prob(p, q, x)
            out[x] += q[x] * t
            if t < 1.0:
                out += q[x] * (1.0 - t) * reject_dist(p, q, x)
        assert np.allclose(out, p, atol=1e-12)


def _sibling_outcome(p0, q0, xs, u_acc, u_term):
    m = len(xs)
    V = len(p0)
    p_rows = np.stack([p0] * (m + 1))
    q_rows = np.stack([q0] * (m + 1))
    u = np.full((m + 1, 2), 0.5)
    u[1:, 0] = u_acc
    u[0, 1] = u_term
    a, path, nxt = decide(p_rows, q_rows, np.array(xs), np.zeros(m, dtype=int), u, cap=10)
    return a, path, nxt


@pytest.mark.parametrize("V,m", [(3, 2), (4, 2), (5, 3), (6, 3)])
def test_lossless_siblings(V, m):
    """m children of the root, drawn from q without replacement and tried in order: the first
    emitted token still follows the target exactly (tree rule)."""
    rng = np.random.default_rng(1000 + 10 * V + m)
    p, q = rand_dist(rng, V), rand_dist(rng, V)
    out = np.zeros(V)
    for xs in itertools.permutations(range(V), m):
        w, rem = 1.0, 1.0
        for x in xs:
            w *= q[x] / rem
            rem -= q[x]
        reach = w                       # probability mass of reaching child i with all earlier rejected
        for i in range(m):
            def acc(u, i=i):
                ua = np.full(m, ONE)
                ua[i] = u
                a, path, _ = _sibling_outcome(p, q, xs, ua, 0.5)
                return a == 1 and path[1] == i + 1
            t = sup_true(acc)
            out[xs[i]] += reach * t
            reach *= (1.0 - t)
            if reach == 0.0:
                break
        if reach > 0.0:
            out += reach * step_measure(lambda u: _sibling_outcome(p, q, xs, np.full(m, ONE), u)[2], V)
    assert np.allclose(out, p, atol=1e-11)


@pytest.mark.parametrize("V", [2, 3, 4])
def test_lossless_two_level_chain(V):
    """Chain of two drafts: the joint law of the first two generated tokens equals
    p(x1) p(x2 | x1).  (When the first draft is rejected the call emits one token and the second
    comes from the next call, i.e. from the target itself.)"""
    rng = np.random.default_rng(7 + V)
    p0, q0 = rand_dist(rng, V), rand_dist(rng, V)
    p1 = np.stack([rand_dist(rng, V) for _ in range(V)])      # target after first token y
    q1 = np.stack([rand_dist(rng, V) for _ in range(V)])
    p2 = rand_dist(rng, V)
    joint = np.zeros((V, V))
    parent = np.array([0, 1])
    for x1 in range(V):
        for x2 in range(V):
            w = q0[x1] * q1[x1, x2]
            p_rows = np.stack([p0, p1[x1], p2])
            q_rows = np.stack([q0, q1[x1], q0])

            def run(u1, u2, t0=0.5, t1=0.5):
                u = np.array([[0.5, t0], [u1, t1], [u2, 0.5]])
                return decide(p_rows, q_rows, np.array([x1, x2]), parent, u, cap=10)
            t1 = sup_true(lambda u: run(u, 0.0)[0] >= 1)
            t2 = sup_true(lambda u: run(0.0, u)[0] == 2)
            joint[x1, x2] += w * t1 * t2
            if t2 < 1.0:
                joint[x1] += w * t1 * (1 - t2) * step_measure(lambda u: run(0.0, ONE, t1=u)[2], V)
            if t1 < 1.0:
                r0 = step_measure(lambda u: run(ONE, 0.0, t0=u)[2], V)
                joint += w * (1 - t1) * (r0[:, None] * p1)
    assert np.allclose(joint, p0[:, None] * p1, atol=1e-11)


def test_emits_at_least_one_and_plain_ar():
    rng = np.random.default_rng(3)
    V = 11
    p = rand_dist(rng, V)
    # no draft at all: plain AR sampling from the target, one token per pass
    g = lambda u: decide(p[None], p[None], np.zeros(0, dtype=int), np.zeros(0, dtype=int),
                         np.array([[0.5, u]]), cap=5)
    a, path, nxt = g(0.3)
    assert a == 0 and path == [0]
    assert np.allclose(step_measure(lambda u: g(u)[2], V), p, atol=1e-12)
    for _ in range(50):
        K = int(rng.integers(1, 6))
        p_rows = np.stack([rand_dist(rng, V) for _ in range(K + 1)])
        q_rows = np.stack([rand_dist(rng, V) for _ in range(K + 1)])
        a, path, nxt = decide(p_rows, q_rows, rng.integers(0, V, K), np.arange(K), rng.random((K + 1, 2)), cap=99)
        assert 0 <= a <= K and len(path) == a + 1 and 0 <= nxt < V


def test_cap_stops_the_walk_and_samples_from_unmodified_target():
    rng = np.random.default_rng(11)
    V, K = 6, 3
    p_rows = np.stack([rand_dist(rng, V) for _ in range(K + 1)])
    toks = rng.integers(0, V, K)
    u = np.zeros((K + 1, 2))        # u = 0 accepts everything that has target mass
    a, path, _ = decide(p_rows, p_rows, toks, np.arange(K), u, cap=1)
    assert a == 1 and path == [0, 1]
    g = lambda uu: decide(p_rows, p_rows, toks, np.arange(K), np.array([[0, 0], [0, uu], [0, 0], [0, 0]], dtype=float), cap=1)[2]
    assert np.allclose(step_measure(g, V), p_rows[1], atol=1e-12)
    g0 = lambda uu: decide(p_rows, p_rows, toks, np.arange(K), np.array([[0, uu]] + [[0, 0]] * K, dtype=float), cap=0)
    assert g0(0.5)[0] == 0
    assert np.allclose(step_measure(lambda uu: g0(uu)[2], V), p_rows[0], atol=1e-12)


def test_uniforms_are_indexed_by_node():
    """A draw that the walk does not consult cannot change the outcome."""
    rng = np.random.default_rng(21)
    V = 8
    parent = np.array([0, 0, 1, 1, 2])        # root -> {1, 2}; 1 -> {3, 4}; 2 -> {5}
    T = 6
    for _ in range(40):
        p_rows = np.stack([rand_dist(rng, V) for _ in range(T)])
        q_rows = np.stack([rand_dist(rng, V) for _ in range(T)])
        toks = np.array([1, 2, 3, 4, 5])
        u = rng.random((T, 2))
        a, path, nxt = decide(p_rows, q_rows, toks, parent, u, cap=9)
        consulted_term = path[-1]
        u2 = u.copy()
        for j in range(T):
            if j != consulted_term:
                u2[j, 1] = rng.random()
        on_path_or_tried = set()
        for node in path:
            for c in range(1, T):
                if parent[c - 1] == node:
                    on_path_or_tried.add(c)
        for c in range(1, T):
            if c not in on_path_or_tried:
                u2[c, 0] = rng.random()
        assert decide(p_rows, q_rows, toks, parent, u2, cap=9) == (a, path, nxt)
        # path is a root-to-node chain of the tree
        for i in range(1, len(path)):
            assert parent[path[i] - 1] == path[i - 1]


def test_inverse_cdf_edges():
    p = np.array([0.0, 0.2, 0.0, 0.5, 0.3, 0.0])
    assert inverse_cdf(p, 0.0) == 1            # never an id without mass
    assert inverse_cdf(p, 0.19999) == 1
    assert inverse_cdf(p, 0.2) == 3            # running sum must EXCEED u * total
    assert inverse_cdf(p, 0.6999) == 3
    assert inverse_cdf(p, 0.71) == 4
    assert inverse_cdf(p, ONE) == 4
    assert inverse_cdf(p * 3.0, 0.71) == 4     # scale-free: unnormalised input allowed
    assert np.allclose(step_measure(lambda u: inverse_cdf(p, u), 6), p, atol=1e-12)


# ------------------------------------------------------------------------------------------------ relaxed rule
def _nbr_table(rng, V, k):
    return np.stack([rng.permutation(np.delete(np.arange(V), x))[:k] for x in range(V)])


def test_relaxed_reduces_to_strict():
    rng = np.random.default_rng(31)
    V, K, k = 16, 4, 5
    nbr = _nbr_table(rng, V, k)
    for _ in range(100):
        p_rows = np.stack([rand_dist(rng, V) for _ in range(K + 1)])
        q_rows = np.stack([rand_dist(rng, V) for _ in range(K + 1)])
        toks, u = rng.integers(0, V, K), rng.random((K + 1, 2))
        strict = decide(p_rows, q_rows, toks, np.arange(K), u, cap=99)
        assert decide(p_rows, q_rows, toks, np.arange(K), u, cap=99, mode=1, nbr=nbr, relax_k=k, relax_delta=0.0) == strict
        assert decide(p_rows, q_rows, toks, np.arange(K), u, cap=99, mode=1, nbr=nbr, relax_k=0, relax_delta=0.5) == strict


def test_relaxed_invariants():
    rng = np.random.default_rng(32)
    V, k = 24, 6
    nbr = _nbr_table(rng, V, k)
    for _ in range(50):
        p, q = rand_dist(rng, V), rand_dist(rng, V)
        x = int(rng.integers(V))
        prev = accept_prob(p, q, x)
        for delta in (0.05, 0.1, 0.2, 0.4, 0.8):
            num, pt = relaxed_target(p.copy(), x, nbr[x], k, delta)
            assert abs(pt.sum() - 1.0) < 1e-12 and (pt >= 0).all()
            assert 0.5 * np.abs(pt - p).sum() <= delta + 1e-12          # total-variation budget
            assert num >= p[x]
            t = accept_prob(p, q, x, mode=1, nbr=nbr, relax_k=k, relax_delta=delta)
            assert t >= prev - 1e-12                                      # non-decreasing in delta
            assert abs(t - min(1.0, num / q[x])) < 1e-12
            prev = t
        # budget >= 1: every neighbour is absorbed
        num, _ = relaxed_target(p.copy(), x, nbr[x], k, 1.0)
        assert abs(num - (p[x] + p[nbr[x]].sum())) < 1e-15
        # prefix rule: stops at the first neighbour that would exceed the budget (no skipping ahead)
        p2 = np.full(V, 0.0)
        p2[x], p2[nbr[x][0]], p2[nbr[x][1]], p2[nbr[x][2]] = 0.1, 0.05, 0.6, 0.25
        num, pt = relaxed_target(p2, x, nbr[x], k, 0.3)
        assert abs(num - 0.15) < 1e-15 and pt[nbr[x][2]] == 0.25


def test_relaxed_is_strict_against_modified_target():
    """Relaxed acceptance = strict acceptance against the modified target (absorbed neighbour mass
    moved onto the drafted id): same accept probability, same replacement law."""
    rng = np.random.default_rng(33)
    V, k = 12, 4
    nbr = _nbr_table(rng, V, k)
    for _ in range(10):
        p, q = rand_dist(rng, V), rand_dist(rng, V)
        x = int(rng.integers(V))
        kw = dict(mode=1, nbr=nbr, relax_k=k, relax_delta=0.25)
        _, pt = relaxed_target(p.copy(), x, nbr[x], k, 0.25)
        assert abs(accept_prob(p, q, x, **kw) - accept_prob(pt, q, x)) < 1e-12
        if accept_prob(pt, q, x) < 1:
            assert np.allclose(reject_dist(p, q, x, **kw), reject_dist(pt, q, x), atol=1e-12)
