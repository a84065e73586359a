"""Pins for the sampled-acceptance oracle (oracle/verify_sample.py) against what the mathematics
fixes: losslessness (the emitted tokens follow the target distribution, Section 1), the greedy
walk as the limit T -> 0 (Section 3.1), plain inverse-CDF sampling when nothing is drafted, and
exact acceptance probabilities on a uniform grid."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import ddd_oracle as O
from oracle.verify_sample import verify_sample


def make_tree(parents, tokens, m=None):
    """Tree with index 0 = root; parents[i-1], tokens[i-1] describe tree index i."""
    n_sel = len(parents)
    m = n_sel if m is None else m
    tree_token = np.full(m + 1, -1, np.int32)
    parent_idx = np.full(m + 1, -1, np.int32)
    pos = np.zeros(m + 1, np.int32)
    mask = np.zeros((m + 1, m + 1), np.uint8)
    tree_token[0] = 0
    mask[0, 0] = 1
    for i in range(1, n_sel + 1):
        p = parents[i - 1]
        assert 0 <= p < i
        parent_idx[i] = p
        tree_token[i] = tokens[i - 1]
        pos[i] = pos[p] + 1
        mask[i] = mask[p]
        mask[i, i] = 1
    sel = np.full(m, -1, np.int32)
    sel[:n_sel] = np.arange(1, n_sel + 1)
    return O.Tree(m=m, n_sel=n_sel, sel_node=sel, tree_token=tree_token, pos=pos, parent_idx=parent_idx, mask=mask)


def test_no_children_is_inverse_cdf_sampling():
    """A tree that is only the root: the bonus token is a plain categorical draw by inverse CDF,
    checked against scipy's softmax + searchsorted."""
    rng = np.random.default_rng(3)
    V = 50
    tree = make_tree([], [], m=4)
    logits = rng.normal(0, 2, (5, V)).astype(np.float32)
    for T in (0.5, 1.0, 2.0):
        cdf = np.cumsum(softmax(logits[0].astype(np.float64) / T))
        for u in rng.random(200):
            ln, path, bonus = verify_sample(tree, logits, T, np.zeros(5), np.full(5, u), D=3)
            assert ln == 0 and path.tolist() == [0, -1, -1, -1]
            assert bonus == int(np.searchsorted(cdf, u, side="right"))


def test_single_child_accept_probability_on_a_grid():
    """One child with token x: over a midpoint grid of N uniforms the number accepted is N p(x)
    to within one grid cell."""
    rng = np.random.default_rng(4)
    V, N = 12, 2000
    logits = rng.normal(0, 1.5, (2, V)).astype(np.float32)
    for x in (0, 5, 11):
        tree = make_tree([0], [x])
        p = softmax(logits[0].astype(np.float64) / 0.8)[x]
        acc = 0
        for i in range(N):
            ua = np.array([0.0, (i + 0.5) / N])
            ln, _, bonus = verify_sample(tree, logits, 0.8, ua, np.full(2, 0.3), D=2)
            acc += ln
            if ln == 0:
                assert bonus != x          # a rejected token is never emitted as the bonus
        assert abs(acc - p * N) <= 1.0


def test_lossless_first_and_second_token():
    """Monte Carlo over the uniforms on a two-level tree: the first emitted token is distributed as
    softmax(root logits / T), and given that it was the drafted child x1 the second one as
    softmax(logits after x1 / T).  5-sigma binomial bounds."""
    rng = np.random.default_rng(5)
    V, T, N = 6, 1.3, 40000
    #      idx:      1  2  3  4  5
    parents = [0, 0, 1, 1, 2]
    tokens = [2, 4, 1, 3, 2]
    tree = make_tree(parents, tokens)
    logits = rng.normal(0, 1.2, (6, V)).astype(np.float32)
    first = np.zeros(V)
    second_after_1 = np.zeros(V)
    n1 = 0
    ua = rng.random((N, 6))
    ub = rng.random((N, 6))
    for t in range(N):
        ln, path, bonus = verify_sample(tree, logits, T, ua[t], ub[t], D=2)
        emitted = [int(tree.tree_token[i]) for i in path[1:ln + 1]] + [bonus]
        first[emitted[0]] += 1
        if ln >= 1 and path[1] == 1:
            n1 += 1
            second_after_1[emitted[1]] += 1
    p0 = softmax(logits[0].astype(np.float64) / T)
    p1 = softmax(logits[1].astype(np.float64) / T)
    assert np.all(np.abs(first / N - p0) < 5 * np.sqrt(p0 * (1 - p0) / N) + 1e-9)
    assert n1 > 1000
    assert np.all(np.abs(second_after_1 / n1 - p1) < 5 * np.sqrt(p1 * (1 - p1) / n1) + 1e-9)


def test_low_temperature_is_the_greedy_walk():
    """T -> 0: the target distribution is a point mass at the argmax, so the result equals the
    greedy accept walk whatever the uniforms are."""
    rng = np.random.default_rng(6)
    V = 40
    for trial in range(30):
        n_sel = int(rng.integers(3, 15))
        parents, tokens = [], []
        for i in range(1, n_sel + 1):
            p = int(rng.integers(0, i))
            used = {tokens[j] for j in range(len(parents)) if parents[j] == p}
            tok = int(rng.choice([t for t in range(V) if t not in used]))
            parents.append(p)
            tokens.append(tok)
        tree = make_tree(parents, tokens)
        logits = rng.normal(0, 1, (n_sel + 1, V)).astype(np.float32)
        # make half of the nodes agree with one of their children
        for i in range(n_sel + 1):
            kids = [c for c in range(1, n_sel + 1) if parents[c - 1] == i]
            if kids and rng.random() < 0.7:
                logits[i, tokens[int(rng.choice(kids)) - 1]] = 9.0
        D = int(tree.pos.max()) + 1
        g = O.verify_accept(tree, np.argmax(logits, axis=1).astype(np.int32), D)
        s = verify_sample(tree, logits, 1e-3, rng.random(n_sel + 1) * 0.999, rng.random(n_sel + 1), D)
        assert s[0] == g[0] and s[1].tolist() == g[1].tolist() and s[2] == g[2]


def test_extreme_uniforms():
    """u_accept = 0 accepts the first child at every level (it has positive probability);
    u_accept close to 1 rejects every child, and u_bonus = 0 then emits the smallest token that is
    not one of the root's children."""
    rng = np.random.default_rng(7)
    V = 10
    tree = make_tree([0, 0, 1, 3], [0, 1, 5, 6])
    logits = rng.normal(0, 1, (5, V)).astype(np.float32)
    ln, path, _ = verify_sample(tree, logits, 1.0, np.zeros(5), np.full(5, 0.5), D=3)
    assert ln == 3 and path.tolist() == [0, 1, 3, 4]
    ln, path, bonus = verify_sample(tree, logits, 1.0, np.full(5, 1.0 - 1e-12), np.zeros(5), D=3)
    assert ln == 0 and bonus == 2


def test_margins_are_reported_for_every_decision():
    rng = np.random.default_rng(8)
    tree = make_tree([0, 0], [1, 2])
    logits = rng.normal(0, 1, (3, 8)).astype(np.float32)
    mg = []
    ln, _, bonus = verify_sample(tree, logits, 1.0, np.full(3, 1.0 - 1e-12), np.full(3, 0.5), D=2, margins=mg)
    assert ln == 0 and len(mg) == 2 + (2 if bonus > 0 else 1) and all(x >= 0 for x in mg)


def test_rejects_non_positive_temperature():
    tree = make_tree([], [], m=1)
    with pytest.raises(ValueError):
        verify_sample(tree, np.zeros((2, 4), np.float32), 0.0, np.zeros(2), np.zeros(2), D=1)
