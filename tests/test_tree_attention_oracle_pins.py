"""Pins of the tree-attention oracle (oracle/tree_attention.py); no GPU."""
import math

import numpy as np

from oracle import bruteforce as BF
from oracle import tree_attention as OT


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _chain_mask(parent):
    n = len(parent)
    return np.array(BF.closure_mask(parent, n), dtype=np.uint8)


def test_root_alone_and_padding():
    T, nh, d, L = 4, 2, 8, 3
    q, kt, vt = _rand((T, nh, d), 0), _rand((T, nh, d), 1), _rand((T, nh, d), 2)
    kp, vp = _rand((L, nh, d), 3), _rand((L, nh, d), 4)
    mask = _chain_mask([-1, 0, 1, 1])
    out = OT.tree_attention(q, kt, vt, kp, vp, mask, n_sel=2)
    assert np.all(out[3] == 0.0)                                   # padding row
    # no prompt, root only: the root sees itself alone, so its output is its own value
    out0 = OT.tree_attention(q, kt, vt, kp[:0], vp[:0], mask, n_sel=3)
    assert np.allclose(out0[0], vt[0], atol=1e-15)


def test_two_keys_is_a_sigmoid():
    T, nh, d = 2, 1, 16
    q, kt, vt = _rand((T, nh, d), 5), _rand((T, nh, d), 6), _rand((T, nh, d), 7)
    mask = _chain_mask([-1, 0])
    out = OT.tree_attention(q, kt, vt, np.zeros((0, nh, d)), np.zeros((0, nh, d)), mask, n_sel=1)
    gap = (q[1, 0] @ kt[0, 0] - q[1, 0] @ kt[1, 0]) / math.sqrt(d)
    p0 = 1.0 / (1.0 + math.exp(-gap))
    assert np.allclose(out[1, 0], p0 * vt[0, 0] + (1 - p0) * vt[1, 0], atol=1e-14)


def test_equal_keys_give_the_mean_and_invisible_nodes_do_not_matter():
    T, nh, d, L = 5, 2, 8, 4
    q = _rand((T, nh, d), 8)
    kt = np.tile(_rand((1, nh, d), 9), (T, 1, 1))
    kp = np.tile(kt[:1], (L, 1, 1))
    vt, vp = _rand((T, nh, d), 10), _rand((L, nh, d), 11)
    parent = [-1, 0, 0, 1, 2]
    mask = _chain_mask(parent)
    out = OT.tree_attention(q, kt, vt, kp, vp, mask, n_sel=4)
    # node 3 sees the prompt and nodes 0, 1, 3 with equal scores
    want = (vp.sum(axis=0) + vt[0] + vt[1] + vt[3]) / (L + 3)
    assert np.allclose(out[3], want, atol=1e-13)
    # changing a node outside the visible set (a sibling branch) changes nothing for node 3
    kt2, vt2 = kt.copy(), vt.copy()
    kt2[2] += 100.0
    vt2[4] -= 50.0
    out2 = OT.tree_attention(q, kt2, vt2, kp, vp, mask, n_sel=4)
    assert np.array_equal(out2[3], out[3]) and np.array_equal(out2[1], out[1])
    assert not np.array_equal(out2[4], out[4])                     # node 4 does see node 2


def test_against_dense_attention_with_minus_infinity():
    """The same numbers from a dense score matrix with -inf at the masked entries."""
    T, nh, d, L = 7, 3, 16, 5
    q, kt, vt = _rand((T, nh, d), 12), _rand((T, nh, d), 13), _rand((T, nh, d), 14)
    kp, vp = _rand((L, nh, d), 15), _rand((L, nh, d), 16)
    parent = [-1, 0, 0, 1, 1, 2, 5]
    mask = _chain_mask(parent)
    out = OT.tree_attention(q, kt, vt, kp, vp, mask, n_sel=6)
    for h in range(nh):
        K = np.concatenate([kp[:, h], kt[:, h]], axis=0)
        V = np.concatenate([vp[:, h], vt[:, h]], axis=0)
        S = q[:, h] @ K.T / math.sqrt(d)
        bias = np.concatenate([np.zeros((T, L)), np.where(mask != 0, 0.0, -np.inf)], axis=1)
        S = S + bias
        P = np.exp(S - S.max(axis=1, keepdims=True))
        P = P / P.sum(axis=1, keepdims=True)
        assert np.allclose(out[:, h], P @ V, atol=1e-13)
