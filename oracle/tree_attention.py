"""CPU oracle for tree attention in the verification pass: what consumes the final tree's mask.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import it.  It shares no code with the HIP path and never calls it.  Plain
numpy in fp64.

Section 1 (EAGLE paragraph): the whole draft tree is fed to the target model in one pass, with
the attention mask adjusted so that a tree node sees the prompt, its ancestors and itself.  For
one sequence, head h and tree node i (tree index order, 0 = root):

    s_j   = q_i . k_j / sqrt(d)        over the L prompt keys and the tree keys j with mask[i][j] = 1
    out_i = sum_j softmax(s)_j v_j

Queries and keys arrive already rotated (position = prompt length + depth is the caller's
business, the tree's `pos` gives the depth).  Tree indices past n_sel are padding: their output
is zero.  The paper treats the target model as a black box, so there are no reference numbers:
the arithmetic is pinned by special cases and brute force in the tests.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def tree_attention(q: np.ndarray, k_tree: np.ndarray, v_tree: np.ndarray, k_prompt: np.ndarray,
                   v_prompt: np.ndarray, mask: np.ndarray, n_sel: int) -> np.ndarray:
    """q, k_tree, v_tree: float64 [T, nh, d]; k_prompt, v_prompt: float64 [L, nh, d];
    mask: [T, T] with mask[i][j] != 0 iff tree node j is i or an ancestor of i.  Returns [T, nh, d]."""
    T, nh, d = q.shape
    L = k_prompt.shape[0]
    out = np.zeros((T, nh, d), dtype=np.float64)
    for i in range(min(T, n_sel + 1)):
        vis = [j for j in range(T) if mask[i][j]]
        for h in range(nh):
            K = np.concatenate([k_prompt[:, h, :], k_tree[vis, h, :]], axis=0)
            V = np.concatenate([v_prompt[:, h, :], v_tree[vis, h, :]], axis=0)
            s = K @ q[i, h] / np.sqrt(float(d))
            s = s - np.max(s)
            p = np.exp(s)
            p = p / np.sum(p)
            out[i, h] = p @ V
    return out
