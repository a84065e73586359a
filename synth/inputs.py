"""Counter-based synthetic inputs shaped like the paper's workloads.

The paper evaluates on MT-bench with Vicuna / LLaMA2-Chat targets and EAGLE
draft heads (Section 3.1).  None of those are available, so everything here is
seeded and synthetic and only mirrors the *shapes*: hidden size, vocabulary,
beam width w (called k here), maximum number of draft calls n (called D) and
final tree size.

Recipe (all integer arithmetic is modulo 2**64):

* LM head ``W[V,H]``: N(0, sigma_w**2) from ``numpy.random.default_rng(seed)``
  in fp32, rounded to bf16 with round-to-nearest-even.  Optional duplicated row
  pairs (row b := row a) give bit-identical logits for the tie-break tests.
* Hidden state of a tree node: a counter-based pseudo-Gaussian.  The key of a
  sequence/round is ``stream_key(seed, b, round)``; the key of a node is
  ``node_key(skey, parent_node_id, token_id)``; element ``e`` draws
  ``z = mix64(nkey + (e+1)*GOLD)`` and sums the four 16-bit fields of ``z``
  (an Irwin-Hall(4) variate, centred: integer in [-131070, 131070], standard
  deviation 65536/sqrt(3)).  One int->fp32 conversion (exact), one fp32
  multiply by ``scale = gain*(1+0.3*depth)/(65536/sqrt(3))``, optionally one
  fp32 add of a "plant" direction, then one RNE rounding to bf16.  No
  transcendental functions are used, so a second implementation of the same
  recipe (for example inside a GPU kernel) reproduces it bit for bit.
* Plant: with probability ``plant_round_p`` per round (and independently
  ``plant_row_p`` per row) the hidden state is shifted along
  ``plant_gain * W[tok] / ||W[tok]||**2`` so that ``logit[tok]`` rises by about
  ``plant_gain``.
* Target argmax for a tree node: a 24-bit hash ``u`` of (skey, pool node id);
  ``u < 0.70`` -> the token of the node's rank-0 child, ``u < 0.85`` -> the
  rank-1 child, otherwise (or when the node has no children in the pool) a
  hash-uniform token.

Nothing in this module projects, normalises, ranks or selects anything.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Optional, Sequence, Tuple

import numpy as np

M64 = (1 << 64) - 1
GOLD = 0x9E3779B97F4A7C15
C_SEQ = 0xD1B54A32D192ED03
C_ROUND_PLANT = 0xA5A5A5A5A5A5A5A5
C_ROW_PLANT = 0x5A5A5A5A5A5A5A5A
C_TARGET = 0x7A67E7
ROOT_PARENT = 0xFFFFFFFF
IH4_STD = 65536.0 / math.sqrt(3.0)
U24_070 = int(0.70 * (1 << 24))
U24_085 = int(0.85 * (1 << 24))


# --------------------------------------------------------------------------
# bf16 helpers (bit manipulation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern (uint16), round-to-nearest-even. Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit pattern (uint16) -> fp32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# integer hashing
# --------------------------------------------------------------------------
def mix64(z):
    """SplitMix64 finaliser on python ints or uint64 arrays."""
    if isinstance(z, np.ndarray):
        z = z.astype(np.uint64, copy=True)
        z ^= z >> np.uint64(30)
        z *= np.uint64(0xBF58476D1CE4E5B9)
        z ^= z >> np.uint64(27)
        z *= np.uint64(0x94D049BB133111EB)
        z ^= z >> np.uint64(31)
        return z
    z &= M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def stream_key(seed: int, b: int, rnd: int) -> int:
    """Key of (seed, sequence b, round rnd)."""
    a = mix64((seed * GOLD + rnd + 1) & M64)
    return mix64(a ^ (((b + 1) * C_SEQ) & M64))


def node_key(skey: int, parent_node: int, token: int) -> int:
    """Key of the tree node reached from pool node ``parent_node`` by ``token``."""
    pt = ((parent_node & 0xFFFFFFFF) << 32) | (token & 0xFFFFFFFF)
    return mix64(skey ^ mix64(pt))


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    V: int
    k: int
    D: int                 # maximum number of LM-head steps per round (paper's n)
    m: int                 # final tree size (draft nodes, root excluded)
    threshold: float       # probability-domain stop threshold t (paper's x = log t)
    sigma_w: float
    gain: float            # hidden-state gain G
    check_mask: int = 0xFFFFFFFF   # bit s set => stop test after the s-th LM-head step
    seed: int = 0
    root_token: int = 1
    plant_round_p: float = 0.0
    plant_row_p: float = 0.0
    plant_gain: float = 8.0
    n_plant: int = 0
    dup_pairs: Tuple[Tuple[int, int], ...] = ()
    plant_on_dups: bool = False    # plant tokens are the first rows of dup_pairs

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)

    @property
    def pool_capacity(self) -> int:
        return 1 + self.k + (self.D - 1) * self.k * self.k

    def scale(self, depth: int) -> np.float32:
        return np.float32(self.gain * (1.0 + 0.3 * depth) / IH4_STD)

    def plant_round_p24(self) -> int:
        return int(self.plant_round_p * (1 << 24))

    def plant_row_p24(self) -> int:
        return int(self.plant_row_p * (1 << 24))


WORKLOADS = {
    "tiny": Workload("tiny", B=1, H=256, V=1000, k=4, D=6, m=16, threshold=0.35,
                     sigma_w=0.05, gain=5.0),
    "7b_b1": Workload("7b_b1", B=1, H=4096, V=32000, k=10, D=10, m=60, threshold=0.3,
                      sigma_w=0.02, gain=3.5),
    "13b_b1": Workload("13b_b1", B=1, H=5120, V=32000, k=10, D=10, m=60, threshold=0.3,
                       sigma_w=0.02, gain=3.5, plant_round_p=0.25, plant_gain=8.0, n_plant=16),
    "7b_b64": Workload("7b_b64", B=64, H=4096, V=32000, k=10, D=10, m=60, threshold=0.3,
                       sigma_w=0.02, gain=3.5),
    "large_vocab": Workload("large_vocab", B=8, H=4096, V=128256, k=16, D=12, m=80, threshold=0.2,
                            sigma_w=0.02, gain=3.5, plant_row_p=0.01, plant_gain=24.0, n_plant=8,
                            dup_pairs=tuple((1000 + 997 * i, 70000 + 1009 * i) for i in range(8)),
                            plant_on_dups=True),
}


# The paper's own parameter settings as variants of a workload (configuration only).  The values are also
# kept, with their citations, in tests/golden/paper_parameters.json.
PAPER_MODES = ("paper", "strict", "eagle2")
PAPER_X = -0.3               # Section 3.2: threshold in the log domain


def paper_mode(wl: Workload, mode: str) -> Workload:
    """`paper`: Section 3.2's DDD setting, n = 11 draft calls at most, checks after calls 5, 7 and 9,
    x = -0.3, i.e. t = fl32(exp(x)) in the probability domain; `strict`: the same with the check after every
    call (the "DDD + Strict" row of Table 1, S = {1..10}); `eagle2`: EAGLE-2's fixed depth of 6 calls and no
    check (Section 3.2).  The beam width of all three is the paper's w = 10, which the 7B / 13B workloads have."""
    t = float(np.float32(math.exp(PAPER_X)))
    if mode == "paper":
        return wl.with_(D=11, check_mask=(1 << 5) | (1 << 7) | (1 << 9), threshold=t)
    if mode == "strict":
        return wl.with_(D=11, check_mask=0x7FE, threshold=t)
    if mode == "eagle2":
        return wl.with_(D=6, check_mask=0, threshold=0.0)
    raise ValueError(f"unknown mode {mode!r}")


# --------------------------------------------------------------------------
# LM head
# --------------------------------------------------------------------------
def make_lm_head(V: int, H: int, sigma_w: float, seed: int = 0,
                 dup_pairs: Sequence[Tuple[int, int]] = ()) -> np.ndarray:
    """bf16 bit patterns (uint16) of W[V,H] ~ N(0, sigma_w**2); row b := row a for (a,b) in dup_pairs."""
    rng = np.random.default_rng(seed)
    out = np.empty((V, H), dtype=np.uint16)
    step = max(1, (1 << 24) // H)
    for v0 in range(0, V, step):
        v1 = min(V, v0 + step)
        blk = rng.standard_normal((v1 - v0, H), dtype=np.float32) * np.float32(sigma_w)
        out[v0:v1] = f32_to_bf16_bits(blk)
    for a, b in dup_pairs:
        out[b] = out[a]
    return out


# --------------------------------------------------------------------------
# stand-in draft layer: weights and prompt context (random numbers only, no arithmetic of the layer)
# --------------------------------------------------------------------------
def _normal_bits(rng, shape, sigma: float) -> np.ndarray:
    rows = shape[0]
    out = np.empty(shape, dtype=np.uint16)
    step = max(1, (1 << 24) // max(1, int(np.prod(shape[1:]))))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        blk = rng.standard_normal((r1 - r0,) + tuple(shape[1:]), dtype=np.float32) * np.float32(sigma)
        out[r0:r1] = f32_to_bf16_bits(blk)
    return out


def make_body_weights(V: int, H: int, F: int, seed: int = 0) -> dict:
    """bf16 bit patterns / fp32 gains of a one-layer draft body: embedding E[V,H], Wfc[H,2H], g1[H],
    Wqkv[3H,H] (q, k, v rows), Wo[H,H], g2[H], Wgu[2F,H] (gate and up rows alternating), Wd[H,F].  Variances are
    1/fan_in, so activations stay of order one."""
    rng = np.random.default_rng(1000 + seed)
    return {
        "E": _normal_bits(rng, (V, H), 1.0),
        "Wfc": _normal_bits(rng, (H, 2 * H), (2 * H) ** -0.5),
        "g1": (1.0 + 0.1 * rng.standard_normal(H)).astype(np.float32),
        "Wqkv": _normal_bits(rng, (3 * H, H), H ** -0.5),
        "Wo": _normal_bits(rng, (H, H), H ** -0.5),
        "g2": (1.0 + 0.1 * rng.standard_normal(H)).astype(np.float32),
        "Wgu": _normal_bits(rng, (2 * F, H), H ** -0.5),
        "Wd": _normal_bits(rng, (H, F), F ** -0.5),
    }


def make_prompt_context(L: int, H: int, seed: int = 0) -> dict:
    """Cached keys K[L,H], values V[L,H] of L prompt positions and the feature f_root[H] of the last
    prompt token, all bf16 bit patterns ~ N(0,1)."""
    rng = np.random.default_rng(2000 + seed)
    return {"K": _normal_bits(rng, (L, H), 1.0), "V": _normal_bits(rng, (L, H), 1.0),
            "f_root": _normal_bits(rng, (1, H), 1.0)[0]}


def make_random_tree(m: int, n_sel: int, k: int, V: int, max_depth: int, seed: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """A random draft-tree shape for the acceptance tests: (tree_token[m+1], parent_idx[m+1]) with
    index 0 the root, parents before children, at most k children per node, no node deeper than
    max_depth and distinct tokens among the children of one node; entries past n_sel are -1."""
    rng = np.random.default_rng(3000 + seed)
    tok = np.full(m + 1, -1, np.int32)
    par = np.full(m + 1, -1, np.int32)
    tok[0] = int(rng.integers(0, V))
    n_kids = np.zeros(m + 1, np.int64)
    depth = np.zeros(m + 1, np.int64)
    used = [set() for _ in range(m + 1)]
    for i in range(1, n_sel + 1):
        open_nodes = np.nonzero((n_kids[:i] < k) & (depth[:i] < max_depth))[0]
        if open_nodes.size == 0:
            raise ValueError("n_sel nodes do not fit a tree of this width and depth")
        # favour recent nodes a little so that trees get some depth
        p = int(open_nodes[min(len(open_nodes) - 1, int(len(open_nodes) * rng.random() ** 0.6))])
        t = int(rng.integers(0, V))
        while t in used[p]:
            t = int(rng.integers(0, V))
        used[p].add(t)
        n_kids[p] += 1
        depth[i] = depth[p] + 1
        par[i], tok[i] = p, t
    return tok, par


def make_target_logits(tree_token: np.ndarray, parent_idx: np.ndarray, n_sel: int, V: int, seed: int = 0,
                       sigma: float = 2.0, boost: float = 13.0, agree: float = 0.8) -> np.ndarray:
    """Stand-in target logits fp32 [m+1, V] for sampled acceptance: N(0, sigma) noise, and with
    probability `agree` a node's row favours the token of one of its children by `boost`, so that
    accepted paths have a realistic length."""
    rng = np.random.default_rng(4000 + seed)
    T = tree_token.shape[0]
    x = (rng.standard_normal((T, V), dtype=np.float32) * np.float32(sigma)).astype(np.float32)
    for i in range(n_sel + 1):
        kids = np.nonzero(parent_idx[1:n_sel + 1] == i)[0] + 1
        if kids.size and rng.random() < agree:
            x[i, tree_token[int(rng.choice(kids))]] += np.float32(boost)
    return x


def make_plant_table(W_bits: np.ndarray, wl: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """(plant_tokens int32[n_plant], plant_dir fp32[n_plant,H]) or empty arrays."""
    if wl.n_plant <= 0:
        return np.zeros((0,), np.int32), np.zeros((0, W_bits.shape[1]), np.float32)
    if wl.plant_on_dups:
        toks = np.array([a for a, _ in wl.dup_pairs][: wl.n_plant], dtype=np.int32)
    else:
        rng = np.random.default_rng(wl.seed + 12345)
        toks = np.sort(rng.choice(wl.V, size=wl.n_plant, replace=False)).astype(np.int32)
    rows = bf16_bits_to_f32(W_bits[toks]).astype(np.float64)
    d = wl.plant_gain * rows / np.sum(rows * rows, axis=1, keepdims=True)
    return toks, d.astype(np.float32)


# --------------------------------------------------------------------------
# hidden states
# --------------------------------------------------------------------------
def _plant_index(skey: int, nkey: int, wl: Workload) -> int:
    """Index into the plant table for this row, or -1."""
    if wl.n_plant <= 0:
        return -1
    ur = mix64(skey ^ C_ROUND_PLANT)
    if (ur >> 40) < wl.plant_round_p24():
        return int((ur & 0xFFFF) % wl.n_plant)
    un = mix64(nkey ^ C_ROW_PLANT)
    if (un >> 40) < wl.plant_row_p24():
        return int((un & 0xFFFF) % wl.n_plant)
    return -1


def hidden_row(wl: Workload, skey: int, parent_node: int, token: int, depth: int,
               plant_dir: Optional[np.ndarray] = None) -> np.ndarray:
    """bf16 bits (uint16[H]) of the hidden state of the node (parent_node --token-->), at ``depth``."""
    nk = node_key(skey, parent_node, token)
    e = np.arange(1, wl.H + 1, dtype=np.uint64)
    z = mix64(np.uint64(nk) + e * np.uint64(GOLD))
    s = ((z & np.uint64(0xFFFF)) + ((z >> np.uint64(16)) & np.uint64(0xFFFF))
         + ((z >> np.uint64(32)) & np.uint64(0xFFFF)) + (z >> np.uint64(48))).astype(np.int64) - 131070
    val = s.astype(np.float32) * wl.scale(depth)
    p = _plant_index(skey, nk, wl)
    if p >= 0:
        assert plant_dir is not None
        val = val + plant_dir[p]
    return f32_to_bf16_bits(val)


def hidden_rows(wl: Workload, skey: int, parent_nodes, tokens, depth: int,
                plant_dir: Optional[np.ndarray] = None) -> np.ndarray:
    """Stack of hidden_row() for several (parent, token) pairs: uint16[R,H]."""
    with np.errstate(over="ignore"):
        return np.stack([hidden_row(wl, skey, int(p), int(t), depth, plant_dir)
                         for p, t in zip(parent_nodes, tokens)])


def root_hidden(wl: Workload, skey: int, plant_dir: Optional[np.ndarray] = None) -> np.ndarray:
    with np.errstate(over="ignore"):
        return hidden_row(wl, skey, ROOT_PARENT, wl.root_token, 0, plant_dir)[None, :]


# --------------------------------------------------------------------------
# synthetic target model: greedy next token after every tree node
# --------------------------------------------------------------------------
def target_argmax_for_tree(wl: Workload, skey: int, pool_token: np.ndarray, pool_parent: np.ndarray,
                           n_nodes: int, tree_nodes: Sequence[int]) -> np.ndarray:
    """int32[len(tree_nodes)]: the stand-in target's argmax after each listed pool node."""
    out = np.empty(len(tree_nodes), dtype=np.int32)
    par = np.asarray(pool_parent[:n_nodes])
    for i, n in enumerate(tree_nodes):
        n = int(n)
        tk = mix64(skey ^ mix64((C_TARGET + n) & M64))
        u = tk >> 40
        uni = int((tk & 0xFFFFFFFF) % wl.V)
        kids = np.nonzero(par == n)[0]          # ascending id == ascending rank
        if u < U24_070 and len(kids) >= 1:
            out[i] = pool_token[kids[0]]
        elif U24_070 <= u < U24_085 and len(kids) >= 2:
            out[i] = pool_token[kids[1]]
        else:
            out[i] = uni
    return out
