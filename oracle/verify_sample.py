"""CPU oracle for sampled (temperature > 0) acceptance of the final draft tree.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import it.  It shares no code with the HIP path and never calls it.  Plain
numpy in fp64.

The paper measures at temperature 0 only (Section 3.1) and names the verification process as
future work (Section 4); what it fixes is that speculative decoding is lossless: the emitted
tokens are distributed as the target model's own (Section 1).  The rule below is the reading
taken here for temperature T > 0.

The drafted children of a tree node are a deterministic function of the context (the top-k of
the draft scores, then the top-m rerank), so as a proposal each child x is a point mass.
Speculative sampling with a point-mass proposal accepts x with probability p(x) and, when it
rejects, continues with p restricted to the tokens other than x and renormalised.  Applied to the
children of the current node in tree-index order, with p = softmax(target logits / T):

  rem = 1
  for each child c (token x_c):  accept c  iff  u_accept[c] * rem < p(x_c);
                                 else  rem -= p(x_c)  and  p(x_c) := 0
  no child accepted (or the node is a leaf): emit the bonus token, the smallest token j with
       sum_{i <= j} p(i) > u_bonus[node] * rem            (inverse CDF of the residual)

Every emitted token then has exactly the distribution p of its context: the first child is
emitted with probability p(x_1), the second with (1 - p(x_1)) * p(x_2) / (1 - p(x_1)) = p(x_2),
and so on, and the bonus token covers the rest.  As T -> 0 the rule becomes the greedy walk.

The uniforms are inputs (one per tree node for its acceptance test, one per tree node for the
bonus draw at that node), so that both sides of a parity test consume the same numbers.

Weights are kept unnormalised: w_j = exp((x_j - max x) / T), rem starts at sum_j w_j.  The tests
that compare a second implementation against this one use `margins` to make sure that no decision
sits within summation-order rounding of its threshold.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np


def verify_sample(tree, target_logits: np.ndarray, temperature: float, u_accept: np.ndarray,
                  u_bonus: np.ndarray, D: int, margins: List[float] | None = None
                  ) -> Tuple[int, np.ndarray, int]:
    """(accept_len, accept_path int32[D+1] of tree indices (-1 padded, starts with 0), bonus_token).

    tree: oracle.ddd_oracle.Tree;  target_logits fp32 [m+1, V], row i = the target model's logits
    after tree node i;  u_accept, u_bonus fp64 [m+1] in [0, 1).
    If `margins` is a list, the relative distance of every decision from its threshold is appended.
    """
    T = float(temperature)
    if not T > 0.0:
        raise ValueError("temperature must be positive")
    n = tree.n_sel + 1
    path = np.full(D + 1, -1, np.int32)
    path[0] = 0
    cur, length = 0, 0
    while True:
        x = np.asarray(target_logits[cur], dtype=np.float32).astype(np.float64)
        w = np.exp((x - np.max(x)) / T)
        total = float(np.sum(w))
        rem = total
        nxt = -1
        for c in range(1, n):
            if tree.parent_idx[c] != cur:
                continue
            tok = int(tree.tree_token[c])
            lhs = float(u_accept[c]) * rem
            if margins is not None:
                margins.append(abs(lhs - w[tok]) / total)
            if lhs < w[tok]:
                nxt = c
                break
            rem -= w[tok]
            w[tok] = 0.0
        if nxt < 0:
            break
        cur = nxt
        length += 1
        path[length] = cur
    thr = float(u_bonus[cur]) * rem
    cum = np.cumsum(w)
    over = np.nonzero(cum > thr)[0]
    if over.size:
        bonus = int(over[0])
        if margins is not None:
            margins.append(abs(cum[bonus] - thr) / total)
            if bonus > 0:
                margins.append(abs(cum[bonus - 1] - thr) / total)
    else:
        # rounding left no prefix above the threshold: the last token that still has weight,
        # and if the children covered everything, the target's most likely token
        pos = np.nonzero(w > 0.0)[0]
        bonus = int(pos[-1]) if pos.size else int(np.argmax(x))
        if margins is not None:
            margins.append(0.0)
    return length, path, bonus
