"""CPU oracle for the stand-in draft-model body (an EAGLE-shaped draft layer with synthetic weights).

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and the benchmark's
cpu_baseline leg may import it.  It shares no code with the HIP path and never calls it.  Plain
numpy in fp64, written out step by step.

What it models (Section 1, EAGLE paragraph: the draft model takes the token sequence and the
target's feature sequence, runs one transformer decoder layer, and reuses the target's LM head;
Section 1, EAGLE-2 paragraph: every beam node is one input row whose context is the prompt plus
the node's ancestors in the draft tree, i.e. tree attention):

  row input   x0 = [ E[token] , f_parent ]                      (2H, bf16: an exact concatenation)
  r0 = x0 Wfc^T                                                 (H)
  xn = bf16( rmsnorm(r0) * g1 )
  [q,k,v] = xn Wqkv^T ; q,k rotated to position L + depth (RoPE, rotate-half pairing, base 10000)
  k,v -> bf16 (what later rows see)
  o = bf16( softmax_j( q.k_j / sqrt(d) ) v_j ) per head, j over the L prompt positions, the row's
      ancestors in the draft tree and the row itself
  r1 = r0 + o Wo^T
  xn2 = bf16( rmsnorm(r1) * g2 )
  [gate, up] = xn2 Wgu^T ; a = bf16( silu(gate) * up )
  h = bf16( r1 + a Wd^T )      -> the hidden row the LM head projects, and the feature f of this node

The trained EAGLE weights are not available, so nothing here says anything about acceptance
quality: parity unpinned against the paper's model; the arithmetic of each step is pinned by
closed forms and brute force in the tests (rotation invariants, softmax over an explicit visible
set, rmsnorm scale, silu values).

bf16 rounding points are part of the definition (the HIP path feeds bf16 operands to the matrix
cores and stores bf16 keys/values); between them this file computes in fp64 where the HIP path
computes in fp32, so comparisons are within a tolerance, not bit-exact.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

HEAD_DIM = 128
ROPE_BASE = 10000.0
RMS_EPS = 1e-6


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round to fp32, then to bf16 (nearest even).  Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float64).astype(np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def round_bf16(x: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f64(f64_to_bf16_bits(x))


def rmsnorm(x: np.ndarray, g: np.ndarray) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * g, per row."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + RMS_EPS) * g


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def rope(x: np.ndarray, pos: int) -> np.ndarray:
    """Rotary embedding of x[..., n_heads*HEAD_DIM] at integer position pos.

    Inside each head, element i (< d/2) is paired with element i + d/2 and the pair is rotated by
    the angle pos * base^(-2i/d).
    """
    d = HEAD_DIM
    shp = x.shape
    xh = x.reshape(shp[:-1] + (shp[-1] // d, d))
    i = np.arange(d // 2, dtype=np.float64)
    ang = float(pos) * ROPE_BASE ** (-2.0 * i / d)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = xh[..., : d // 2], xh[..., d // 2:]
    out = np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)
    return out.reshape(shp)


def attention_row(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """One query row against its visible keys: q[H], K[n,H], V[n,H] -> o[H]; heads of HEAD_DIM."""
    d = HEAD_DIM
    nh = q.shape[0] // d
    qh = q.reshape(nh, d)
    Kh = K.reshape(K.shape[0], nh, d)
    Vh = V.reshape(V.shape[0], nh, d)
    o = np.empty((nh, d), dtype=np.float64)
    for h in range(nh):
        s = Kh[:, h, :] @ qh[h] / np.sqrt(float(d))
        s = s - np.max(s)
        p = np.exp(s)
        p = p / np.sum(p)
        o[h] = p @ Vh[:, h, :]
    return o.reshape(-1)


@dataclass
class LayerWeights:
    E_bits: np.ndarray      # uint16 [V,H]   token embedding
    Wfc_bits: np.ndarray    # uint16 [H,2H]
    g1: np.ndarray          # fp32 [H]
    Wqkv_bits: np.ndarray   # uint16 [3H,H]  rows: q, then k, then v
    Wo_bits: np.ndarray     # uint16 [H,H]
    g2: np.ndarray          # fp32 [H]
    Wgu_bits: np.ndarray    # uint16 [2F,H]  row 2i: gate i, row 2i+1: up i
    Wd_bits: np.ndarray     # uint16 [H,F]


@dataclass
class Prompt:
    K_bits: np.ndarray      # uint16 [L,H]  keys of the prompt positions (as cached: already rotated)
    V_bits: np.ndarray      # uint16 [L,H]
    f_root_bits: np.ndarray  # uint16 [H]   the target's feature at the last prompt token


def layer_rows(w: LayerWeights, x0_bits: np.ndarray, pos: int, visible_K: List[np.ndarray],
               visible_V: List[np.ndarray]):
    """The layer for R rows at one position.  visible_K[r] / visible_V[r]: float64 [n_r,H] keys and
    values (already bf16-rounded) the row sees besides itself.  Returns (h_bits, k_bits, v_bits)."""
    R, H2 = x0_bits.shape
    H = H2 // 2
    x0 = bf16_bits_to_f64(x0_bits)
    r0 = x0 @ bf16_bits_to_f64(w.Wfc_bits).T
    xn = round_bf16(rmsnorm(r0, w.g1.astype(np.float64)))
    qkv = xn @ bf16_bits_to_f64(w.Wqkv_bits).T
    q = rope(qkv[:, :H], pos)
    k_bits = f64_to_bf16_bits(rope(qkv[:, H:2 * H], pos))
    v_bits = f64_to_bf16_bits(qkv[:, 2 * H:])
    k, v = bf16_bits_to_f64(k_bits), bf16_bits_to_f64(v_bits)
    o = np.empty((R, H), dtype=np.float64)
    for r in range(R):
        K = np.concatenate([visible_K[r], k[r:r + 1]], axis=0)
        V = np.concatenate([visible_V[r], v[r:r + 1]], axis=0)
        o[r] = attention_row(q[r], K, V)
    o = round_bf16(o)
    r1 = r0 + o @ bf16_bits_to_f64(w.Wo_bits).T
    xn2 = round_bf16(rmsnorm(r1, w.g2.astype(np.float64)))
    gu = xn2 @ bf16_bits_to_f64(w.Wgu_bits).T
    a = round_bf16(silu(gu[:, 0::2]) * gu[:, 1::2])
    h = r1 + a @ bf16_bits_to_f64(w.Wd_bits).T
    return f64_to_bf16_bits(h), k_bits, v_bits


class StandInBody:
    """draft_body(s, beam, pool) for oracle.ddd_oracle.run_round: keeps, per draft call, the rows'
    features, keys, values and parent slots, and builds each row's visible set by walking the
    parent slots back to the prompt call."""

    def __init__(self, w: LayerWeights, prompt: Prompt, root_token: int):
        self.w, self.prompt, self.root_token = w, prompt, int(root_token)
        self.L = prompt.K_bits.shape[0]
        self.Kp = bf16_bits_to_f64(prompt.K_bits)
        self.Vp = bf16_bits_to_f64(prompt.V_bits)
        self.h: List[np.ndarray] = []        # per call: uint16 [R,H]
        self.k: List[np.ndarray] = []
        self.v: List[np.ndarray] = []
        self.parent: List[np.ndarray] = []   # per call s >= 1: parent slot in call s-1 of each row

    def _chain(self, s: int, slot: int):
        """(call, row) pairs of the ancestors of row `slot` of call s, nearest first."""
        out = []
        while s >= 1:
            p = int(self.parent[s - 1][slot])
            out.append((s - 1, p))
            s, slot = s - 1, p
        return out

    def __call__(self, s: int, beam, pool) -> np.ndarray:
        H = self.prompt.f_root_bits.shape[0]
        if s == 0:
            self.h, self.k, self.v, self.parent = [], [], [], []
            tokens = np.array([self.root_token])
            feats = self.prompt.f_root_bits[None, :]
            parents = None
        else:
            tokens = np.asarray(beam.token)
            parents = np.asarray(beam.parent_slot, dtype=np.int64)   # all 0 for the call after the prompt call
            feats = self.h[s - 1][parents]
            self.parent.append(parents)
        x0 = np.concatenate([self.w.E_bits[tokens], feats], axis=1).astype(np.uint16)
        vis_K, vis_V = [], []
        for r in range(len(tokens)):
            anc = self._chain(s, r)[::-1]     # root call first
            Ks = [self.Kp] + [bf16_bits_to_f64(self.k[c][j:j + 1]) for c, j in anc]
            Vs = [self.Vp] + [bf16_bits_to_f64(self.v[c][j:j + 1]) for c, j in anc]
            vis_K.append(np.concatenate(Ks, axis=0))
            vis_V.append(np.concatenate(Vs, axis=0))
        h_bits, k_bits, v_bits = layer_rows(self.w, x0, self.L + s, vis_K, vis_V)
        self.h.append(h_bits)
        self.k.append(k_bits)
        self.v.append(v_bits)
        return h_bits
