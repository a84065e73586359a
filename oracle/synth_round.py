"""Glue between the seeded input generators and the CPU oracle (test infrastructure only).

Runs oracle rounds on the synthetic workloads: the stand-in draft body is the
counter-based hidden-state generator, the stand-in target model is the hashed
target argmax.  No method arithmetic lives here.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

import synth
from . import ddd_oracle as O


def make_draft_body(wl: synth.Workload, skey: int, plant_dir: Optional[np.ndarray]):
    def body(s, beam, pool):
        if beam is None:
            return synth.root_hidden(wl, skey, plant_dir)
        parents = [int(pool.parent[n]) for n in beam.node]
        return synth.hidden_rows(wl, skey, parents, beam.token, s, plant_dir)
    return body


def oracle_round(wl: synth.Workload, W_bits: np.ndarray, plant_dir: Optional[np.ndarray], b: int, rnd: int,
                 threshold: Optional[float] = None, logits_fn=None, keep_logits: bool = False):
    """One oracle round for sequence b of round rnd; returns (RoundResult, target_argmax, accept tuple)."""
    skey = synth.stream_key(wl.seed, b, rnd)
    t = wl.threshold if threshold is None else threshold
    res = O.run_round(W_bits, wl.k, wl.D, wl.m, t, wl.check_mask, make_draft_body(wl, skey, plant_dir),
                      root_token=wl.root_token, logits_fn=logits_fn, keep_logits=keep_logits)
    tree_nodes = [0] + [int(n) for n in res.tree.sel_node[: res.tree.n_sel]]
    tgt = np.full(wl.m + 1, -1, np.int32)
    tgt[: len(tree_nodes)] = synth.target_argmax_for_tree(wl, skey, res.pool.token, res.pool.parent,
                                                          res.pool.n_nodes, tree_nodes)
    acc = O.verify_accept(res.tree, tgt, wl.D)
    return res, tgt, acc
