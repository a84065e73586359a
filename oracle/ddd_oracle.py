"""CPU oracle for one Dynamic Depth Decoding (DDD) draft round.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and
the benchmark's cpu_baseline leg may import it.  It shares no code with the HIP
path and never calls it.  Everything is plain numpy in fp64 (results rounded
once to fp32 where the method stores fp32), written step by step in the order
and notation of the paper so it can be checked against the paper by eye.

The method is a heuristic procedure (beam-search drafting with a confidence
stop), so the oracle *is* the algorithm:

* Section 1 (EAGLE-2 paragraph): the draft tree grows by beam search; after
  each draft-model run the top-k token sequences, ranked by the sum of their
  logprobs, become the next draft input.
* Section 2: the draft output goes through a logsoftmax; Eq. 1 defines the
  heuristic H = log(sum_i exp(logprobsum[i])) over the beam.
* Algorithm 1: run on the prompt, build the beam, then for step = 1..n-1:
  if step is in S and H < x, stop; otherwise run the draft model on the beam,
  build the new beam, add the parents' logprobsum to the new logprobs.
* Section 1 (speculative decoding / EAGLE paragraphs) and Section 3.1
  (temperature 0): the whole tree goes to the target model under a tree
  attention mask; tokens are verified until one is incorrect and the token
  that should follow the correct prefix is emitted.

Readings taken where the paper is silent or inconsistent (each also listed in
the design notes of the repository):

R1  Eq. 1 prints the sum as i = 0..w; a beam has w entries, so i = 0..w-1.
R2  The threshold is taken in the probability domain: P = sum_i exp(logprobsum[i]),
    continue iff P >= t, with t = exp(x).  "H < x" (strict) stops, equality continues.
R3  Loop index `step` = number of draft calls already made.  The test at index
    `step` uses the beam produced by call number `step`, before call step+1.
    Bit s of check_mask <=> s in S.
R4  n (max draft calls incl. the prompt call) is called D here; depth of the
    tree <= D.
R5  "EAGLE-2's algorithm": per-row top-k of the logprobs, add the parent's
    logprobsum, global top-k of the k*k candidates is the next beam; *all* k*k
    candidates enter the node pool that the final tree is chosen from.
R6  Row top-k ranks by the fp32 logit (descending), ties by lower token id.
R7  Beam select ranks by (score descending, token id ascending, flat index
    i*k+j ascending).
R8  The final tree is the m best pool nodes (root excluded) by (score
    descending, node id ascending), listed in ascending node id; the root is
    tree index 0.  m counts draft nodes only.
R9  pos = depth (root 0); mask[i][j] = 1 iff j is i or an ancestor of i.
R10 accept_len counts accepted draft tokens; the bonus token is the target's
    argmax after the last accepted node.
R11 Arithmetic: bf16 inputs; logits = fp64 dot product rounded once to fp32;
    lse in fp64 from the fp32 logits; logprob = fp32(logit - lse); score =
    one IEEE fp32 add; the stop-test sum in fp64 in index order.

Parity status: every function below is pinned by the CPU tests (library
special cases, closed forms, invariants, brute force, a hand-worked example);
none is "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np


# --------------------------------------------------------------------------
# bf16 decode (exact)
# --------------------------------------------------------------------------
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# LM-head projection  (Section 1: the draft model reuses the target's LM head)
# --------------------------------------------------------------------------
def lmhead_logits(W_bits: np.ndarray, hid_bits: np.ndarray, chunk: int = 4096) -> np.ndarray:
    """logits[r,v] = fp32( sum_h W[v,h] * hid[r,h] ), the sum taken in fp64.

    W_bits uint16[V,H] and hid_bits uint16[R,H] are bf16 bit patterns.
    """
    V, H = W_bits.shape
    R = hid_bits.shape[0]
    x = bf16_to_f64(hid_bits)                       # [R,H]
    out = np.empty((R, V), dtype=np.float32)
    for v0 in range(0, V, chunk):
        v1 = min(V, v0 + chunk)
        Wc = bf16_to_f64(W_bits[v0:v1])             # [c,H]
        out[:, v0:v1] = (x @ Wc.T).astype(np.float32)
    return out


def lmhead_logits_loops(W_bits: np.ndarray, hid_bits: np.ndarray) -> np.ndarray:
    """Same definition as lmhead_logits written as explicit loops (small inputs only)."""
    V, H = W_bits.shape
    R = hid_bits.shape[0]
    W = bf16_to_f64(W_bits)
    x = bf16_to_f64(hid_bits)
    out = np.empty((R, V), dtype=np.float32)
    for r in range(R):
        for v in range(V):
            acc = 0.0
            for h in range(H):
                acc += float(W[v, h]) * float(x[r, h])
            out[r, v] = np.float32(acc)
    return out


# --------------------------------------------------------------------------
# logsoftmax  (Section 2: the draft output is turned into logprobs by a logsoftmax)
# --------------------------------------------------------------------------
def logsumexp_row(logits_f32: np.ndarray) -> float:
    """lse = M + log(sum_v exp(logit[v] - M)), M = max, in fp64."""
    z = np.asarray(logits_f32, dtype=np.float64)
    M = float(np.max(z))
    return M + float(np.log(np.sum(np.exp(z - M))))


def logprobs_row(logits_f32: np.ndarray, lse: Optional[float] = None) -> np.ndarray:
    """logprob[v] = fp32( fp64(logit[v]) - lse )."""
    if lse is None:
        lse = logsumexp_row(logits_f32)
    return (np.asarray(logits_f32, dtype=np.float64) - float(lse)).astype(np.float32)


# --------------------------------------------------------------------------
# per-row top-k   (reading R6)
# --------------------------------------------------------------------------
def row_topk(logits_f32: np.ndarray, k: int) -> np.ndarray:
    """Token ids of the k largest logits; order (logit descending, token id ascending)."""
    z = np.asarray(logits_f32, dtype=np.float32)
    ids = np.arange(z.shape[0])
    order = np.lexsort((ids, -z.astype(np.float64)))     # last key is primary
    return order[:k].astype(np.int32)


# --------------------------------------------------------------------------
# Eq. 1 and the stop test  (Algorithm 1, the `if step in S` block; readings R1-R3)
# --------------------------------------------------------------------------
def beam_confidence(logprobsum_f32: Sequence[float]) -> float:
    """P = sum_i exp(logprobsum[i]) over the beam, fp64, in index order.  H of Eq. 1 is log P."""
    P = 0.0
    for v in np.asarray(logprobsum_f32, dtype=np.float32):
        P += float(np.exp(np.float64(v)))
    return P


def heuristic_H(logprobsum_f32: Sequence[float]) -> float:
    """Eq. 1 as printed (log domain)."""
    return float(np.log(beam_confidence(logprobsum_f32)))


def depth_continue(logprobsum_f32: Sequence[float], steps_done: int, D: int, t: float,
                   check_mask: int) -> Tuple[bool, float]:
    """Decision taken after `steps_done` draft calls: (continue?, P).

    Continue iff another call is allowed (steps_done < D) and either the step is
    not in S or P >= t.  t is the fp32 threshold widened to fp64.
    """
    P = beam_confidence(logprobsum_f32)
    if steps_done >= D:
        return False, P
    if (check_mask >> steps_done) & 1:
        if P < float(np.float32(t)):
            return False, P
    return True, P


# --------------------------------------------------------------------------
# node pool and beam  (Section 1, EAGLE-2 paragraph; Algorithm 1, the beam update;
#                      readings R5, R7)
# --------------------------------------------------------------------------
@dataclass
class Pool:
    k: int
    D: int
    token: np.ndarray = None      # int32[Nmax]
    parent: np.ndarray = None     # int32[Nmax]
    depth: np.ndarray = None      # int32[Nmax]
    score: np.ndarray = None      # fp32[Nmax]
    n_nodes: int = 1

    def __post_init__(self):
        n = 1 + self.k + (self.D - 1) * self.k * self.k
        self.token = np.full(n, -1, np.int32)
        self.parent = np.full(n, -1, np.int32)
        self.depth = np.zeros(n, np.int32)
        self.score = np.zeros(n, np.float32)

    @property
    def capacity(self) -> int:
        return self.token.shape[0]


@dataclass
class Beam:
    node: np.ndarray            # int32[k] pool ids
    token: np.ndarray           # int32[k]
    parent_slot: np.ndarray     # int32[k] slot in the previous beam (0 at the first step)
    logprobsum: np.ndarray      # fp32[k]


def beam_first(pool: Pool, root_token: int, tok: np.ndarray, lp: np.ndarray) -> Beam:
    """Algorithm 1, before the loop: the prompt call's top-k tokens become nodes 1..k and the beam."""
    k = pool.k
    pool.token[0] = root_token
    pool.parent[0] = -1
    pool.depth[0] = 0
    pool.score[0] = np.float32(0.0)
    for j in range(k):
        nid = 1 + j
        pool.token[nid] = tok[j]
        pool.parent[nid] = 0
        pool.depth[nid] = 1
        pool.score[nid] = np.float32(lp[j])
    pool.n_nodes = 1 + k
    return Beam(node=np.arange(1, 1 + k, dtype=np.int32), token=np.array(tok[:k], np.int32),
                parent_slot=np.zeros(k, np.int32), logprobsum=np.array(lp[:k], np.float32))


def beam_expand(pool: Pool, beam: Beam, s: int, tok: np.ndarray, lp: np.ndarray) -> Beam:
    """One loop iteration of Algorithm 1 after the draft call number s+1 (s >= 1 calls were made before).

    tok[i][j], lp[i][j]: rank-j token / logprob of the row of beam slot i.
    Appends the k*k candidates (i-major) to the pool, then selects the new beam.
    """
    k = pool.k
    base = 1 + k + (s - 1) * k * k
    cand = []
    for i in range(k):
        for j in range(k):
            nid = base + i * k + j
            sc = np.float32(np.float32(beam.logprobsum[i]) + np.float32(lp[i][j]))   # one fp32 add
            pool.token[nid] = tok[i][j]
            pool.parent[nid] = beam.node[i]
            pool.depth[nid] = s + 1
            pool.score[nid] = sc
            cand.append((-float(sc), int(tok[i][j]), i * k + j))
    pool.n_nodes = base + k * k
    cand.sort()                                   # score desc, token asc, flat index asc
    pick = [c[2] for c in cand[:k]]
    return Beam(node=np.array([base + f for f in pick], np.int32),
                token=np.array([pool.token[base + f] for f in pick], np.int32),
                parent_slot=np.array([f // k for f in pick], np.int32),
                logprobsum=np.array([pool.score[base + f] for f in pick], np.float32))


# --------------------------------------------------------------------------
# final tree: top-m rerank, mask, positions   (Section 1, EAGLE paragraph; readings R8, R9)
# --------------------------------------------------------------------------
@dataclass
class Tree:
    m: int
    n_sel: int
    sel_node: np.ndarray       # int32[m], pool ids ascending, -1 padded
    tree_token: np.ndarray     # int32[m+1], index 0 = root
    pos: np.ndarray            # int32[m+1]
    parent_idx: np.ndarray     # int32[m+1], index into this list, root -1
    mask: np.ndarray           # uint8[m+1,m+1]


def tree_finalize(pool: Pool, m: int) -> Tree:
    N = pool.n_nodes - 1
    m_eff = min(m, N)
    ids = list(range(1, pool.n_nodes))
    ids.sort(key=lambda n: (-float(pool.score[n]), n))
    chosen = sorted(ids[:m_eff])
    sel_node = np.full(m, -1, np.int32)
    sel_node[:m_eff] = chosen
    tree_nodes = [0] + chosen
    index_of = {n: i for i, n in enumerate(tree_nodes)}
    tree_token = np.full(m + 1, -1, np.int32)
    pos = np.zeros(m + 1, np.int32)
    parent_idx = np.full(m + 1, -1, np.int32)
    mask = np.zeros((m + 1, m + 1), np.uint8)
    for i, n in enumerate(tree_nodes):
        tree_token[i] = pool.token[n]
        pos[i] = pool.depth[n]
        parent_idx[i] = index_of[int(pool.parent[n])] if n != 0 else -1
        a = n
        while a != -1:                     # walk to the root, marking self and ancestors
            mask[i, index_of[int(a)]] = 1
            a = int(pool.parent[a])
    return Tree(m=m, n_sel=m_eff, sel_node=sel_node, tree_token=tree_token, pos=pos,
                parent_idx=parent_idx, mask=mask)


# --------------------------------------------------------------------------
# greedy accept walk   (Section 1, speculative-decoding paragraph; Section 3.1; reading R10)
# --------------------------------------------------------------------------
def verify_accept(tree: Tree, target_argmax: np.ndarray, D: int) -> Tuple[int, np.ndarray, int]:
    """(accept_len, accept_path int32[D+1] of tree indices (-1 padded, starts with 0), bonus_token)."""
    n = tree.n_sel + 1
    path = np.full(D + 1, -1, np.int32)
    cur = 0
    path[0] = 0
    length = 0
    while True:
        nxt = -1
        for c in range(1, n):
            if tree.parent_idx[c] == cur and tree.tree_token[c] == target_argmax[cur]:
                nxt = c
                break
        if nxt < 0:
            break
        cur = nxt
        length += 1
        path[length] = cur
    return length, path, int(target_argmax[cur])


# --------------------------------------------------------------------------
# the round   (Algorithm 1)
# --------------------------------------------------------------------------
@dataclass
class StepRecord:
    hid_bits: np.ndarray        # uint16[R,H] fed to the LM head
    logits: Optional[np.ndarray]  # fp32[R,V] (kept only if keep_logits)
    lse: np.ndarray             # fp64[R]
    tok: np.ndarray             # int32[R,k]
    lp: np.ndarray              # fp32[R,k]
    beam: Beam                  # beam after this step
    P: float                    # confidence after this step
    cont: bool                  # decision after this step


@dataclass
class RoundResult:
    pool: Pool
    steps: int
    records: List[StepRecord]
    tree: Tree


LogitsFn = Callable[[int, np.ndarray], Tuple[np.ndarray, Optional[np.ndarray]]]
DraftBodyFn = Callable[[int, Optional[Beam], Pool], np.ndarray]


def lmhead_topk(logits: np.ndarray, k: int, lse_in: Optional[np.ndarray] = None):
    """Rows of logits -> (tok int32[R,k], lp fp32[R,k], lse fp64[R])."""
    R = logits.shape[0]
    tok = np.empty((R, k), np.int32)
    lp = np.empty((R, k), np.float32)
    lse = np.empty(R, np.float64)
    for r in range(R):
        lse[r] = logsumexp_row(logits[r]) if lse_in is None else float(lse_in[r])
        tok[r] = row_topk(logits[r], k)
        lp[r] = (logits[r][tok[r]].astype(np.float64) - lse[r]).astype(np.float32)
    return tok, lp, lse


def run_round(W_bits: Optional[np.ndarray], k: int, D: int, m: int, t: float, check_mask: int,
              draft_body: DraftBodyFn, root_token: int = 1,
              logits_fn: Optional[LogitsFn] = None, keep_logits: bool = False) -> RoundResult:
    """One DDD draft round for one sequence.

    draft_body(s, beam, pool) returns the bf16 hidden rows for draft call number
    s+1 (beam is None for the prompt call, one row; k rows afterwards).
    logits_fn(s, hid_bits) may supply (logits fp32[R,V], lse or None) instead of
    the oracle's own projection (used to replay another implementation's logits).
    """
    pool = Pool(k=k, D=D)
    records: List[StepRecord] = []

    def project(s, hid):
        if logits_fn is not None:
            return logits_fn(s, hid)
        return lmhead_logits(W_bits, hid), None

    # Algorithm 1, before the loop: prompt call, first beam, logprobsum
    hid = draft_body(0, None, pool)
    logits, lse_in = project(0, hid)
    tok, lp, lse = lmhead_topk(logits, k, lse_in)
    beam = beam_first(pool, root_token, tok[0], lp[0])
    steps = 1
    cont, P = depth_continue(beam.logprobsum, steps, D, t, check_mask)
    records.append(StepRecord(hid, logits if keep_logits else None, lse, tok, lp, beam, P, cont))

    # Algorithm 1, the for loop: step = number of calls already made
    while cont:
        s = steps
        hid = draft_body(s, beam, pool)
        logits, lse_in = project(s, hid)
        tok, lp, lse = lmhead_topk(logits, k, lse_in)
        beam = beam_expand(pool, beam, s, tok, lp)
        steps += 1
        cont, P = depth_continue(beam.logprobsum, steps, D, t, check_mask)
        records.append(StepRecord(hid, logits if keep_logits else None, lse, tok, lp, beam, P, cont))

    tree = tree_finalize(pool, m)
    return RoundResult(pool=pool, steps=steps, records=records, tree=tree)
