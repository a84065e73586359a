"""Pins of the stand-in draft-layer oracle (oracle/body.py) against closed forms, invariants and brute
force; no GPU.  The layer itself has no reference outputs to compare with (EAGLE's trained weights are not
available): what is pinned is the arithmetic of every step."""
import math

import numpy as np

import synth
from oracle import body as OB
from oracle import bruteforce as BF
from oracle import ddd_oracle as O


def _weights(V=50, H=256, F=384, seed=0):
    w = synth.make_body_weights(V, H, F, seed)
    return OB.LayerWeights(w["E"], w["Wfc"], w["g1"], w["Wqkv"], w["Wo"], w["g2"], w["Wgu"], w["Wd"])


def _prompt(L=5, H=256, seed=0):
    p = synth.make_prompt_context(L, H, seed)
    return OB.Prompt(p["K"], p["V"], p["f_root"])


def test_bf16_rounding_is_nearest_even():
    # 1 + 2^-8 lies halfway between 1 and 1 + 2^-7: ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 lies halfway between 1 + 2^-7 and 1 + 2^-6: even is 1 + 2^-6
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -2.5, 0.0])
    got = OB.round_bf16(x)
    assert list(got) == [1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -2.5, 0.0]


def test_rmsnorm_closed_forms():
    x = np.array([[3.0, -4.0, 0.0, 0.0]])             # mean square 25/4
    y = OB.rmsnorm(x, np.ones(4))
    assert np.allclose(y, x / math.sqrt(6.25 + OB.RMS_EPS), rtol=0, atol=1e-15)
    rng = np.random.default_rng(0)
    z = rng.standard_normal((3, 64)) * 7.0
    g = rng.standard_normal(64)
    yz = OB.rmsnorm(z, g)
    assert np.allclose(np.mean((yz / g) ** 2, axis=1), 1.0, atol=1e-6)          # unit mean square before the gain
    assert np.allclose(OB.rmsnorm(5.0 * z, g), yz, atol=1e-6)                     # scale invariant (up to eps)


def test_silu_values():
    assert OB.silu(np.array([0.0]))[0] == 0.0
    assert abs(OB.silu(np.array([1.0]))[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(OB.silu(np.array([-1.0]))[0] + 1.0 / (1.0 + math.e)) < 1e-15
    assert abs(OB.silu(np.array([40.0]))[0] - 40.0) < 1e-12


def test_rope_is_a_rotation_that_depends_on_relative_position():
    rng = np.random.default_rng(1)
    q = rng.standard_normal(2 * OB.HEAD_DIM)
    k = rng.standard_normal(2 * OB.HEAD_DIM)
    assert np.array_equal(OB.rope(q, 0), q)                                      # position 0: identity
    for pos in (1, 17, 300):
        rq = OB.rope(q, pos)
        for h in range(2):                                                        # norms kept per head
            sl = slice(h * OB.HEAD_DIM, (h + 1) * OB.HEAD_DIM)
            assert abs(np.linalg.norm(rq[sl]) - np.linalg.norm(q[sl])) < 1e-12
    # <R_m q, R_n k> depends on m - n only
    a = OB.rope(q, 40) @ OB.rope(k, 33)
    b = OB.rope(q, 107) @ OB.rope(k, 100)
    assert abs(a - b) < 1e-9
    # one pair written out by hand: element 0 pairs with element d/2, angle = pos (frequency 1)
    e = np.zeros(OB.HEAD_DIM)
    e[0] = 1.0
    r = OB.rope(e, 2)
    assert abs(r[0] - math.cos(2.0)) < 1e-15 and abs(r[OB.HEAD_DIM // 2] - math.sin(2.0)) < 1e-15
    # last pair: angle = pos * base^(-(d-2)/d)
    e = np.zeros(OB.HEAD_DIM)
    e[OB.HEAD_DIM // 2 - 1] = 1.0
    ang = 3.0 * OB.ROPE_BASE ** (-(OB.HEAD_DIM - 2.0) / OB.HEAD_DIM)
    r = OB.rope(e, 3)
    assert abs(r[OB.HEAD_DIM // 2 - 1] - math.cos(ang)) < 1e-15 and abs(r[OB.HEAD_DIM - 1] - math.sin(ang)) < 1e-15


def test_attention_row_special_cases():
    rng = np.random.default_rng(2)
    H = 2 * OB.HEAD_DIM
    q = rng.standard_normal(H)
    V = rng.standard_normal((4, H))
    # a single visible key: the output is its value, whatever the score
    assert np.allclose(OB.attention_row(q, rng.standard_normal((1, H)), V[:1]), V[0], atol=1e-15)
    # equal keys: equal weights, the mean of the values
    K = np.tile(rng.standard_normal((1, H)), (4, 1))
    assert np.allclose(OB.attention_row(q, K, V), V.mean(axis=0), atol=1e-12)
    # two keys, one head's score gap written out: weights sigmoid(+-gap)
    K = rng.standard_normal((2, H))
    o = OB.attention_row(q, K, V[:2])
    for h in range(2):
        sl = slice(h * OB.HEAD_DIM, (h + 1) * OB.HEAD_DIM)
        gap = (q[sl] @ K[0, sl] - q[sl] @ K[1, sl]) / math.sqrt(OB.HEAD_DIM)
        p0 = 1.0 / (1.0 + math.exp(-gap))
        assert np.allclose(o[sl], p0 * V[0, sl] + (1 - p0) * V[1, sl], atol=1e-12)


def test_layer_with_silent_attention_and_mlp_is_the_fc_projection():
    """Wo = 0 and Wd = 0 remove both residual branches: h = bf16(x0 Wfc^T), a plain matrix product."""
    w = _weights()
    w.Wo_bits = np.zeros_like(w.Wo_bits)
    w.Wd_bits = np.zeros_like(w.Wd_bits)
    p = _prompt()
    rng = np.random.default_rng(3)
    x0 = synth.f32_to_bf16_bits(rng.standard_normal((3, 512)).astype(np.float32))
    vis = [OB.bf16_bits_to_f64(p.K_bits)] * 3
    visv = [OB.bf16_bits_to_f64(p.V_bits)] * 3
    h, _, _ = OB.layer_rows(w, x0, 5, vis, visv)
    want = O.lmhead_logits(w.Wfc_bits, x0)            # the LM-head oracle is the same contraction
    assert np.array_equal(h, synth.f32_to_bf16_bits(want))


def test_tree_attention_sees_exactly_the_ancestors():
    """StandInBody against a dense recomputation: every row's visible set, taken from the transitive closure
    of the parent pointers (brute force), must give the same output rows."""
    V, H, F, k = 50, 256, 384, 3
    w, p = _weights(V, H, F), _prompt(4, H)
    body = OB.StandInBody(w, p, root_token=7)

    class B:  # the fields of a beam the body reads
        def __init__(self, token, parent_slot):
            self.token, self.parent_slot = np.array(token), np.array(parent_slot)

    beams = [None, B([1, 2, 3], [0, 0, 0]), B([4, 5, 6], [2, 0, 2]), B([7, 8, 9], [1, 1, 0])]
    rows = [body(s, b, None) for s, b in enumerate(beams)]
    assert rows[0].shape == (1, H) and rows[3].shape == (k, H)
    # global node ids: call 0 row 0 -> 0; call s row j -> 1 + (s-1)*k + j
    nid = lambda s, j: 0 if s == 0 else 1 + (s - 1) * k + j
    n = 1 + 3 * k
    parent = [-1] * n
    for s in range(1, 4):
        for j in range(k):
            ps = int(beams[s].parent_slot[j])
            parent[nid(s, j)] = nid(s - 1, ps if s > 1 else 0)
    mask = BF.closure_mask(parent, n)                  # mask[i][j] = j is i or an ancestor of i
    allK = np.concatenate([body.k[s] for s in range(4)], axis=0)
    allV = np.concatenate([body.v[s] for s in range(4)], axis=0)
    Kp, Vp = OB.bf16_bits_to_f64(p.K_bits), OB.bf16_bits_to_f64(p.V_bits)
    s = 3
    feats = body.h[s - 1][beams[s].parent_slot]
    x0 = np.concatenate([w.E_bits[beams[s].token], feats], axis=1).astype(np.uint16)
    vis_K, vis_V = [], []
    for j in range(k):
        me = nid(s, j)
        anc = [i for i in range(n) if mask[me][i] and i != me]
        vis_K.append(np.concatenate([Kp, OB.bf16_bits_to_f64(allK[anc])], axis=0))
        vis_V.append(np.concatenate([Vp, OB.bf16_bits_to_f64(allV[anc])], axis=0))
        assert len(anc) == s                                                     # one ancestor per earlier call
    h, _, _ = OB.layer_rows(w, x0, p.K_bits.shape[0] + s, vis_K, vis_V)
    assert np.array_equal(h, rows[3])
    # a sibling's key must not be visible: adding it changes the row
    j = 0
    wrong_K = [np.concatenate([vis_K[j], OB.bf16_bits_to_f64(allK[nid(3, 1):nid(3, 1) + 1])], axis=0)] + vis_K[1:]
    wrong_V = [np.concatenate([vis_V[j], OB.bf16_bits_to_f64(allV[nid(3, 1):nid(3, 1) + 1])], axis=0)] + vis_V[1:]
    h2, _, _ = OB.layer_rows(w, x0, p.K_bits.shape[0] + s, wrong_K, wrong_V)
    assert not np.array_equal(h2[0], rows[3][0])


def test_body_drives_a_round():
    """The body plugs into the round oracle; rows have the right shapes and every call extends the history."""
    V, H, F, k, D = 200, 256, 384, 4, 4
    w, p = _weights(V, H, F), _prompt(6, H)
    W_lm = synth.make_lm_head(V, H, 0.05, seed=9)
    body = OB.StandInBody(w, p, root_token=3)
    res = O.run_round(W_lm, k, D, 8, 0.0, 0xFFFFFFFF, body, root_token=3)
    assert res.steps == D
    assert [r.shape[0] for r in body.h] == [1] + [k] * (D - 1)
    assert all(len(body._chain(s, 0)) == s for s in range(D))
