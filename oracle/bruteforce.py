"""Brute-force cross-checks for the CPU oracle (test infrastructure only).

Each function restates one part of the draft round in a deliberately different
form from ddd_oracle.py, so that an indexing or ordering mistake in either one
shows up as a disagreement:

* global_topk_over_kV   - the next beam as a full sort of all k*V scored
                          continuations (Section 1, EAGLE-2 paragraph) instead of
                          "row top-k, then top-k of k*k".
* closure_mask          - the tree mask as the reflexive-transitive closure of
                          the parent relation, by Warshall's algorithm.
* accept_len_enumerate  - the accept length as the maximum, over every root-to-
                          node path of the tree, of the matched prefix length.
* round_by_paths        - a whole round keyed by token paths held in
                          dictionaries (no node ids, no pool arrays).
"""
from __future__ import annotations

from typing import Callable, Dict, List, Sequence, Tuple

import numpy as np


def global_topk_over_kV(logprobsum: np.ndarray, logits_rows: np.ndarray, lse_rows: np.ndarray, k: int):
    """Top-k of all k*V continuations by (score desc, token asc, parent slot asc).

    Returns a list of (parent_slot, token, score_f32).
    """
    R, V = logits_rows.shape
    cands = []
    for i in range(R):
        lp = (logits_rows[i].astype(np.float64) - float(lse_rows[i])).astype(np.float32)
        sc = (np.float32(logprobsum[i]) + lp).astype(np.float32)
        for v in range(V):
            cands.append((-float(sc[v]), v, i, np.float32(sc[v])))
    cands.sort(key=lambda c: (c[0], c[1], c[2]))
    return [(c[2], c[1], c[3]) for c in cands[:k]], cands


def closure_mask(parent_idx: Sequence[int], n: int) -> np.ndarray:
    """Reflexive-transitive closure of i -> parent_idx[i] over tree indices 0..n-1 (Warshall)."""
    reach = np.zeros((n, n), dtype=bool)
    for i in range(n):
        reach[i, i] = True
        p = int(parent_idx[i])
        if p >= 0:
            reach[i, p] = True
    for mid in range(n):
        for i in range(n):
            if reach[i, mid]:
                reach[i] |= reach[mid]
    return reach.astype(np.uint8)


def accept_len_enumerate(parent_idx: Sequence[int], tree_token: Sequence[int], n: int,
                         target_argmax: Sequence[int]) -> Tuple[int, int]:
    """(accept length, tree index of the last accepted node) by enumerating every root-to-node path."""
    best_len, best_node = 0, 0
    for node in range(n):
        path = []
        a = node
        while a != -1:
            path.append(a)
            a = int(parent_idx[a])
        path.reverse()                      # root ... node
        ok = True
        for prev, cur in zip(path[:-1], path[1:]):
            if int(tree_token[cur]) != int(target_argmax[prev]):
                ok = False
                break
        if ok and len(path) - 1 > best_len:
            best_len, best_node = len(path) - 1, node
    return best_len, best_node


PathLogitsFn = Callable[[Tuple[int, ...]], np.ndarray]


def round_by_paths(path_logits: PathLogitsFn, V: int, k: int, D: int, m: int, t: float, check_mask: int):
    """A DDD round keyed by token paths.

    path_logits(path) -> fp32[V] logits of the draft call whose input ends at `path`
    (() for the prompt).  Returns (beams per step as lists of paths, pool dict
    path -> (score, creation index), chosen tree paths, steps, P per step).
    """
    def lse_of(z):
        z = z.astype(np.float64)
        M = z.max()
        return M + np.log(np.exp(z - M).sum())

    score: Dict[Tuple[int, ...], np.float32] = {(): np.float32(0.0)}
    created: Dict[Tuple[int, ...], int] = {(): 0}
    beams: List[List[Tuple[int, ...]]] = []
    Ps: List[float] = []

    def children_of(path, parent_score):
        z = path_logits(path)
        lse = lse_of(z)
        lp = (z.astype(np.float64) - lse).astype(np.float32)
        sc = (np.float32(parent_score) + lp).astype(np.float32)
        ranked = sorted(range(V), key=lambda v: (-float(z[v]), v))[:k]
        return z, sc, ranked

    # prompt call
    z, sc, ranked = children_of((), np.float32(0.0))
    # at the first step the score is the logprob itself (0 + lp is exact)
    for v in ranked:
        score[(v,)] = sc[v]
        created[(v,)] = len(created)
    beam = [(v,) for v in ranked]
    beams.append(beam)
    steps = 1

    def conf(beam):
        return float(sum(np.exp(np.float64(score[p])) for p in beam))

    while True:
        P = conf(beam)
        Ps.append(P)
        if steps >= D:
            break
        if (check_mask >> steps) & 1 and P < float(np.float32(t)):
            break
        allc = []
        for i, p in enumerate(beam):
            z, sc, ranked = children_of(p, score[p])
            for v in ranked:
                score[p + (v,)] = sc[v]
                created[p + (v,)] = len(created)
            for v in range(V):
                allc.append((-float(sc[v]), v, i, p + (v,)))
        allc.sort(key=lambda c: (c[0], c[1], c[2]))
        beam = [c[3] for c in allc[:k]]
        beams.append(beam)
        steps += 1

    nodes = [p for p in score if p != ()]
    nodes.sort(key=lambda p: (-float(score[p]), created[p]))
    chosen = sorted(nodes[: min(m, len(nodes))], key=lambda p: created[p])
    return beams, score, created, chosen, steps, Ps
