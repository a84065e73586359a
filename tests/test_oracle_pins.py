"""Pins for the CPU oracle: library special cases, closed forms, invariants, brute force and a
hand-worked example.  None of these tests touches the GPU or the HIP library."""
import json
import math
import os

import numpy as np
import pytest
import scipy.special

import synth
from oracle import ddd_oracle as O
from oracle import bruteforce as BF
from oracle import synth_round as SR

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _bits(x):
    return synth.f32_to_bf16_bits(np.asarray(x, np.float32))


# ----------------------------------------------------------------------------------------------
# logits
# ----------------------------------------------------------------------------------------------
def test_logits_match_explicit_loops_and_library_matmul():
    rng = np.random.default_rng(1)
    W = _bits(rng.standard_normal((37, 24)) * 0.3)
    x = _bits(rng.standard_normal((3, 24)))
    a = O.lmhead_logits(W, x, chunk=16)           # chunk boundary inside V
    b = O.lmhead_logits_loops(W, x)
    c = (synth.bf16_bits_to_f32(x).astype(np.float64) @ synth.bf16_bits_to_f32(W).astype(np.float64).T)
    assert a.dtype == np.float32 and a.shape == (3, 37)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_allclose(a.astype(np.float64), c, rtol=0, atol=1e-6)
    assert np.max(np.abs(a.astype(np.float64) - c)) <= np.max(np.abs(c)) * 2.0 ** -24


def test_logits_exact_on_small_integers_and_not_transposed():
    # integers are exact in bf16 and the dot products are exact in fp32
    W = np.array([[1, 2, 3, 4], [0, -1, 0, 2], [5, 0, 0, 0]], np.float32)      # V=3, H=4
    x = np.array([[1, 0, 0, 0], [1, 1, 1, 1]], np.float32)                      # R=2
    got = O.lmhead_logits(_bits(W), _bits(x))
    want = np.array([[1, 0, 5], [10, 1, 5]], np.float32)                         # [R,V]
    np.testing.assert_array_equal(got, want)


def test_bf16_decode_is_exact():
    vals = np.array([1.0, -2.5, 0.00390625, 3.0e38, -1.0e-30], np.float32)
    bits = synth.f32_to_bf16_bits(vals)
    back = O.bf16_to_f64(bits)
    # decode(bits) must be the fp32 whose upper 16 bits are `bits`
    assert np.array_equal(back.astype(np.float32).view(np.uint32) >> 16, bits.astype(np.uint32))
    assert back[0] == 1.0 and back[1] == -2.5 and back[2] == 0.00390625


# ----------------------------------------------------------------------------------------------
# logsoftmax
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("scale", [0.1, 3.0, 40.0])
def test_logsoftmax_invariants_and_scipy(scale):
    rng = np.random.default_rng(2)
    z = (rng.standard_normal(5000) * scale).astype(np.float32)
    lse = O.logsumexp_row(z)
    lp = O.logprobs_row(z)
    assert lp.dtype == np.float32
    assert np.all(lp <= 0)
    assert abs(scipy.special.logsumexp(lp.astype(np.float64))) <= 1e-6      # each row has logsumexp 0
    np.testing.assert_allclose(lp, scipy.special.log_softmax(z.astype(np.float64)), rtol=2.0 ** -23, atol=1e-7)
    assert abs(lse - scipy.special.logsumexp(z.astype(np.float64))) <= 1e-10


def test_logsoftmax_closed_forms():
    assert abs(O.logsumexp_row(np.zeros(8, np.float32)) - math.log(8)) < 1e-14
    z = np.array([1000.0, 1000.0], np.float32)                    # no overflow
    assert abs(O.logsumexp_row(z) - (1000 + math.log(2))) < 1e-12
    z = np.array([0.0, -1e4], np.float32)
    assert abs(O.logsumexp_row(z)) < 1e-12


# ----------------------------------------------------------------------------------------------
# row top-k
# ----------------------------------------------------------------------------------------------
def test_row_topk_full_sort_and_ties_lower_id():
    rng = np.random.default_rng(3)
    z = rng.standard_normal(2000).astype(np.float32)
    z[17] = z[900] = z[5] = z.max() + 1.0        # planted three-way tie at the top
    z[1500] = z[40]                                # and one somewhere else
    got = O.row_topk(z, 12)
    want = sorted(range(2000), key=lambda v: (-float(z[v]), v))[:12]
    assert list(got) == want
    assert list(got[:3]) == [5, 17, 900]
    assert len(set(got.tolist())) == 12


def test_row_topk_descending_values():
    z = np.array([0.5, 2.0, -1.0, 2.0, 7.0], np.float32)
    assert list(O.row_topk(z, 4)) == [4, 1, 3, 0]


# ----------------------------------------------------------------------------------------------
# Eq. 1 / stop test
# ----------------------------------------------------------------------------------------------
def test_eq1_closed_forms():
    lps = np.log(np.array([0.5, 0.25], np.float64)).astype(np.float32)
    assert abs(O.beam_confidence(lps) - 0.75) < 1e-7
    assert abs(O.heuristic_H(lps) - math.log(0.75)) < 1e-7
    # one sequence: H is its logprobsum
    assert abs(O.heuristic_H(np.array([-1.25], np.float32)) + 1.25) < 1e-12
    # w equal entries: H = logprobsum + log w
    assert abs(O.heuristic_H(np.full(10, -3.0, np.float32)) - (-3.0 + math.log(10))) < 1e-12


def test_stop_test_semantics():
    lps = np.log(np.array([0.5, 0.25])).astype(np.float32)      # P = 0.75
    all_steps = 0xFFFFFFFF
    assert O.depth_continue(lps, 1, 6, 0.7, all_steps)[0] is True
    assert O.depth_continue(lps, 1, 6, 0.8, all_steps)[0] is False
    assert O.depth_continue(lps, 1, 6, 0.8, 0)[0] is True                # step not in S: no test
    assert O.depth_continue(lps, 1, 6, 0.8, 1 << 2)[0] is True           # S = {2}, step 1 not tested
    assert O.depth_continue(lps, 2, 6, 0.8, 1 << 2)[0] is False
    assert O.depth_continue(lps, 6, 6, 0.0, all_steps)[0] is False       # n calls made: loop is over
    # equality continues (the paper stops on H < x, strictly)
    one = np.array([0.0], np.float32)                                    # P = 1 exactly
    assert O.depth_continue(one, 1, 6, 1.0, all_steps)[0] is True
    assert O.depth_continue(one, 1, 6, np.nextafter(np.float32(1.0), np.float32(2.0)), all_steps)[0] is False


def test_log_domain_form_agrees_with_probability_domain():
    with open(os.path.join(GOLD, "paper_parameters.json")) as f:
        pp = json.load(f)
    x = pp["x"]
    t = math.exp(x)
    assert abs(t - pp["t_equiv"]) < 1e-15
    rng = np.random.default_rng(4)
    n_checked = 0
    for _ in range(500):
        lps = (-rng.exponential(1.5, size=pp["w"])).astype(np.float32)
        H = O.heuristic_H(lps)
        if abs(H - x) < 1e-6:
            continue
        n_checked += 1
        mask = sum(1 << s for s in pp["S"])
        cont, P = O.depth_continue(lps, 5, pp["n"], t, mask)
        assert cont == (not (H < x))
    assert n_checked > 400


def test_workload_modes_carry_the_papers_parameters():
    """The configurations the benchmark's --mode and the GPU mode tests run are Section 3.2's numbers."""
    with open(os.path.join(GOLD, "paper_parameters.json")) as f:
        pp = json.load(f)
    base = synth.WORKLOADS["7b_b1"]
    assert base.k == pp["w"]
    paper, strict, eagle2 = (synth.paper_mode(base, m) for m in synth.PAPER_MODES)
    assert paper.D == strict.D == pp["n"] and eagle2.D == pp["eagle2_depth"]
    assert [s for s in range(32) if (paper.check_mask >> s) & 1] == pp["S"]
    assert [s for s in range(32) if (strict.check_mask >> s) & 1] == pp["strict_S"]
    assert paper.threshold == strict.threshold == float(np.float32(pp["t_equiv"]))
    assert eagle2.threshold == 0.0
    # and the oracle's stop test under them: stops only at a step of S, and never when no step is checked
    lps = np.full(pp["w"], -6.0, np.float32)                   # P = 10 e^-6, far below t
    for done in range(1, pp["n"]):
        assert O.depth_continue(lps, done, paper.D, paper.threshold, paper.check_mask)[0] == (done not in pp["S"])
        assert O.depth_continue(lps, done, strict.D, strict.threshold, strict.check_mask)[0] is False
    for done in range(1, eagle2.D):
        assert O.depth_continue(lps, done, eagle2.D, eagle2.threshold, eagle2.check_mask)[0] is True
    assert O.depth_continue(lps, eagle2.D, eagle2.D, eagle2.threshold, eagle2.check_mask)[0] is False


# ----------------------------------------------------------------------------------------------
# the hand-worked round
# ----------------------------------------------------------------------------------------------
def _hand_logits_fn(g, pool_ref):
    probs = {tuple(int(c) for c in key.split(",") if c != ""): np.array(v, np.float64)
             for key, v in g["probs"].items()}

    def path_of(pool, node):
        p = []
        while node != 0:
            p.append(int(pool.token[node]))
            node = int(pool.parent[node])
        return tuple(reversed(p))

    state = {}

    def body(s, beam, pool):
        state["paths"] = [()] if beam is None else [path_of(pool, int(n)) for n in beam.node]
        return np.zeros((len(state["paths"]), 8), np.uint16)

    def logits_fn(s, hid):
        rows = [np.log(probs[p]).astype(np.float32) for p in state["paths"]]
        return np.stack(rows), None

    return body, logits_fn


@pytest.mark.parametrize("case", ["case_t03", "case_t05"])
def test_hand_worked_round(case):
    with open(os.path.join(GOLD, "hand_round_v4_k2.json")) as f:
        g = json.load(f)
    c = g[case]
    body, logits_fn = _hand_logits_fn(g, None)
    res = O.run_round(None, g["k"], g["D"], g["m"], c["t"], 0xFFFFFFFF, body, root_token=g["root_token"],
                      logits_fn=logits_fn)
    assert res.steps == c["steps"]
    for rec, P, bn in zip(res.records, c["P"], c["beam_nodes"]):
        assert abs(rec.P - P) < 1e-6
        assert list(rec.beam.node) == bn
    if "beam_tokens" in c:
        for rec, bt, bs in zip(res.records, c["beam_tokens"], c["beam_parent_slot"]):
            assert list(rec.beam.token) == bt
            assert list(rec.beam.parent_slot) == bs
        n = res.pool.n_nodes
        assert n == len(c["pool_token"])
        assert list(res.pool.token[:n]) == c["pool_token"]
        assert list(res.pool.parent[:n]) == c["pool_parent"]
        assert list(res.pool.depth[:n]) == c["pool_depth"]
        np.testing.assert_allclose(np.exp(res.pool.score[:n].astype(np.float64)), c["pool_prob"], rtol=1e-6)
    tr = res.tree
    assert tr.n_sel == len(c["sel_node"])
    assert list(tr.sel_node[: tr.n_sel]) == c["sel_node"]
    assert list(tr.tree_token[: tr.n_sel + 1]) == c["tree_token"]
    assert list(tr.pos[: tr.n_sel + 1]) == c["pos"]
    assert list(tr.parent_idx[: tr.n_sel + 1]) == c["parent_idx"]
    assert tr.mask[: tr.n_sel + 1, : tr.n_sel + 1].tolist() == c["mask"]
    for v in c.get("verify", []):
        ln, path, bonus = O.verify_accept(tr, np.array(v["target_argmax"], np.int32), g["D"])
        assert ln == v["accept_len"] and bonus == v["bonus"]
        assert list(path[: ln + 1]) == v["path"] and np.all(path[ln + 1:] == -1)


# ----------------------------------------------------------------------------------------------
# rounds on the synthetic tiny workload: structural invariants
# ----------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def tiny():
    wl = synth.WORKLOADS["tiny"]
    W = synth.make_lm_head(wl.V, wl.H, wl.sigma_w, wl.seed)
    return wl, W


def _check_round_invariants(wl, res):
    k, pool = wl.k, res.pool
    # node count = k + (steps-1) k^2 (+ root)
    assert pool.n_nodes == 1 + k + (res.steps - 1) * k * k
    assert 1 <= res.steps <= wl.D
    prev_beam = None
    prevP = 1.0 + 1e-6
    for s, rec in enumerate(res.records):
        # beam confidence is a probability mass, non-increasing over steps
        assert 0.0 <= rec.P <= 1.0 + 1e-6
        assert rec.P <= prevP + 1e-6
        prevP = rec.P
        assert len(set(rec.beam.node.tolist())) == k
        for i in range(k):
            n = int(rec.beam.node[i])
            assert pool.depth[n] == s + 1
            assert pool.score[n] == rec.beam.logprobsum[i]
            if prev_beam is not None:
                assert pool.parent[n] == prev_beam.node[rec.beam.parent_slot[i]]
                # logprobsum never increases from parent to child
                assert rec.beam.logprobsum[i] <= prev_beam.logprobsum[rec.beam.parent_slot[i]]
        if s >= 1:
            # the new beam is the top-k of the k*k candidates by full sort
            base = 1 + k + (s - 1) * k * k
            ids = sorted(range(base, base + k * k),
                         key=lambda n: (-float(pool.score[n]), int(pool.token[n]), n))
            assert list(rec.beam.node) == ids[:k]
        prev_beam = rec.beam
    # every non-root node: parent exists, one level up, and was in the beam of the previous step
    for n in range(1, pool.n_nodes):
        p = int(pool.parent[n])
        assert 0 <= p < n and pool.depth[p] == pool.depth[n] - 1
        if pool.depth[n] >= 2:
            assert p in res.records[pool.depth[n] - 2].beam.node.tolist()
    # score of a node = sum of the logprobs on its path (recomputed in fp64)
    for n in range(1, pool.n_nodes, max(1, pool.n_nodes // 40)):
        tot, a = 0.0, n
        while a != 0:
            d = int(pool.depth[a])
            rec = res.records[d - 1]
            p = int(pool.parent[a])
            row = 0 if d == 1 else res.records[d - 2].beam.node.tolist().index(p)
            j = rec.tok[row].tolist().index(int(pool.token[a]))
            tot += float(rec.lp[row][j])
            a = p
        assert abs(tot - float(pool.score[n])) < 1e-5
    # stop decisions
    for s, rec in enumerate(res.records):
        steps_done = s + 1
        want = steps_done < wl.D and not (((wl.check_mask >> steps_done) & 1) and rec.P < np.float32(wl.threshold))
        assert rec.cont == want
    assert res.records[-1].cont is False
    assert all(r.cont for r in res.records[:-1])


def _check_tree(wl, res):
    pool, tr = res.pool, res.tree
    N = pool.n_nodes - 1
    assert tr.n_sel == min(wl.m, N)
    ids = sorted(range(1, pool.n_nodes), key=lambda n: (-float(pool.score[n]), n))[: tr.n_sel]
    assert sorted(ids) == tr.sel_node[: tr.n_sel].tolist()
    assert np.all(tr.sel_node[tr.n_sel:] == -1)
    sel = set(tr.sel_node[: tr.n_sel].tolist()) | {0}
    for n in sel - {0}:
        assert int(pool.parent[n]) in sel                       # parent-closed
    n = tr.n_sel + 1
    np.testing.assert_array_equal(tr.mask[:n, :n], BF.closure_mask(tr.parent_idx, n))
    assert np.all(tr.mask[n:, :] == 0) and np.all(tr.mask[:, n:] == 0)
    assert np.all(tr.mask[:n, 0] == 1)                          # root is everyone's ancestor
    assert np.all(np.triu(tr.mask[:n, :n], 1) == 0)             # parents precede children
    assert np.array_equal(tr.mask[:n, :n].sum(axis=1), tr.pos[:n] + 1)
    for i in range(1, n):
        assert tr.pos[i] == tr.pos[tr.parent_idx[i]] + 1
        assert tr.tree_token[i] == pool.token[tr.sel_node[i - 1]]


def test_tiny_rounds_invariants_and_accept_bruteforce(tiny):
    wl, W = tiny
    depths = set()
    for rnd in range(24):
        res, tgt, (ln, path, bonus) = SR.oracle_round(wl, W, None, 0, rnd)
        depths.add(res.steps)
        _check_round_invariants(wl, res)
        _check_tree(wl, res)
        n = res.tree.n_sel + 1
        bl, bn = BF.accept_len_enumerate(res.tree.parent_idx, res.tree.tree_token, n, tgt)
        assert ln == bl and path[ln] == bn and bonus == tgt[bn]
        assert 0 <= ln <= res.steps
    assert len(depths) >= 4          # the workload exercises early stop and full depth


def test_threshold_extremes_and_empty_S(tiny):
    wl, W = tiny
    r0, _, _ = SR.oracle_round(wl, W, None, 0, 3, threshold=0.0)
    assert r0.steps == wl.D                                  # t = 0 never stops: fixed depth (EAGLE-2)
    r1, _, _ = SR.oracle_round(wl, W, None, 0, 3, threshold=1.5)
    assert r1.steps == 1                                     # t > 1 always stops after the prompt call
    r2, _, _ = SR.oracle_round(wl.with_(check_mask=0), W, None, 0, 3, threshold=1.5)
    assert r2.steps == wl.D                                  # S empty: never tested
    # the first `steps` records of a stopped round equal the prefix of the fixed-depth round
    r3, _, _ = SR.oracle_round(wl, W, None, 0, 3)
    for a, b in zip(r3.records, r0.records):
        assert list(a.beam.node) == list(b.beam.node)
        assert a.P == b.P


def test_taking_over_one_stop_decision_leaves_the_earlier_calls_alone(tiny):
    """The replay comparisons may take one borderline stop decision over from the other side; the parameters they
    use for that must change nothing before the call in question and decide that call as asked."""
    from replay_util import take_over_stop_decision
    wl, W = tiny
    seen = 0
    for rnd in range(12):
        base, _, _ = SR.oracle_round(wl, W, None, 0, rnd)
        s = base.steps
        if s < wl.D:                                         # stopped after call s: force it to go on
            mask, t = take_over_stop_decision(wl.check_mask, wl.threshold, s, True)
            r, _, _ = SR.oracle_round(wl.with_(check_mask=mask), W, None, 0, rnd, threshold=t)
            assert r.steps > s
            for a, b in zip(base.records, r.records):
                assert list(a.beam.node) == list(b.beam.node) and a.P == b.P
            seen += 1
        if s >= 2:                                           # went on after call s - 1: force it to stop there
            mask, t = take_over_stop_decision(wl.check_mask, wl.threshold, s - 1, False)
            r, _, _ = SR.oracle_round(wl.with_(check_mask=mask), W, None, 0, rnd, threshold=t)
            assert r.steps == s - 1
            for a, b in zip(r.records, base.records):
                assert list(a.beam.node) == list(b.beam.node) and a.P == b.P
            seen += 1
    assert seen >= 8


def test_m_at_least_N_selects_everything(tiny):
    wl, W = tiny
    res, _, _ = SR.oracle_round(wl.with_(m=200), W, None, 0, 1)
    N = res.pool.n_nodes - 1
    assert res.tree.n_sel == N
    assert res.tree.sel_node[:N].tolist() == list(range(1, N + 1))


def test_k1_is_a_greedy_chain():
    wl = synth.WORKLOADS["tiny"].with_(k=1, m=8, D=5, threshold=0.0)
    W = synth.make_lm_head(wl.V, wl.H, wl.sigma_w, wl.seed)
    res, tgt, _ = SR.oracle_round(wl, W, None, 0, 0, keep_logits=True)
    assert res.steps == 5 and res.pool.n_nodes == 6
    # k = 1: P is the product of the top-1 probabilities, and every token is the row argmax
    prod = 1.0
    for s, rec in enumerate(res.records):
        z = rec.logits[0].astype(np.float64)
        p = np.exp(z - scipy.special.logsumexp(z))
        assert rec.tok[0][0] == int(np.argmax(z))
        prod *= p.max()
        assert abs(rec.P - prod) < 1e-6
    n = res.tree.n_sel + 1
    np.testing.assert_array_equal(res.tree.mask[:n, :n], np.tril(np.ones((n, n), np.uint8)))
    # target that always agrees -> whole chain accepted; first disagreement cuts it
    tgt = np.full(wl.m + 1, -1, np.int32)
    tgt[: n - 1] = res.tree.tree_token[1:n]
    tgt[n - 1] = 77
    assert O.verify_accept(res.tree, tgt, wl.D)[0] == 5
    tgt[2] = (tgt[2] + 1) % wl.V
    ln, path, bonus = O.verify_accept(res.tree, tgt, wl.D)
    assert ln == 2 and bonus == tgt[2]


def test_V_equals_k_gives_unit_mass():
    rng = np.random.default_rng(7)
    z = rng.standard_normal((1, 6)).astype(np.float32)
    res = O.run_round(None, 6, 2, 4, 0.0, 0xFFFFFFFF, lambda s, b, p: np.zeros((1 if b is None else 6, 4), np.uint16),
                      logits_fn=lambda s, hid: (np.repeat(z, hid.shape[0], axis=0), None))
    assert abs(res.records[0].P - 1.0) < 1e-6


# ----------------------------------------------------------------------------------------------
# whole round against the path-keyed brute force, and beam select against the k*V full sort
# ----------------------------------------------------------------------------------------------
def _path_logits_factory(V, seed, sharp):
    def f(path):
        h = 1469598103934665603
        for tkn in (seed,) + tuple(path):
            h = ((h ^ (tkn + 11)) * 1099511628211) % (1 << 64)
        rng = np.random.default_rng(h % (1 << 32))
        return (rng.standard_normal(V) * sharp).astype(np.float32)
    return f


@pytest.mark.parametrize("seed", range(12))
def test_round_matches_path_keyed_bruteforce(seed):
    rng = np.random.default_rng(100 + seed)
    V = int(rng.integers(5, 40)); k = int(rng.integers(1, 5)); D = int(rng.integers(1, 5))
    k = min(k, V)
    m = int(rng.integers(1, 30)); t = float(rng.choice([0.0, 0.2, 0.5, 0.8]))
    mask = int(rng.choice([0xFFFFFFFF, 0b1010, 0]))
    plog = _path_logits_factory(V, seed, float(rng.choice([1.0, 3.0, 6.0])))
    state = {}

    def path_of(pool, node):
        p = []
        while node != 0:
            p.append(int(pool.token[node])); node = int(pool.parent[node])
        return tuple(reversed(p))

    def body(s, beam, pool):
        state["paths"] = [()] if beam is None else [path_of(pool, int(n)) for n in beam.node]
        return np.zeros((len(state["paths"]), 4), np.uint16)

    res = O.run_round(None, k, D, m, t, mask, body, logits_fn=lambda s, hid: (np.stack([plog(p) for p in state["paths"]]), None))
    try:
        beams, score, created, chosen, steps, Ps = BF.round_by_paths(plog, V, k, D, m, t, mask)
    except KeyError:
        pytest.skip("two distinct logits of one row rounded to the same score at the beam cut")
    assert steps == res.steps
    for rec, bp, P in zip(res.records, beams, Ps):
        assert [path_of(res.pool, int(n)) for n in rec.beam.node] == bp
        assert abs(rec.P - P) < 1e-12
    got = [path_of(res.pool, int(n)) for n in res.tree.sel_node[: res.tree.n_sel]]
    assert got == chosen
    for n in range(1, res.pool.n_nodes):
        assert score[path_of(res.pool, n)] == res.pool.score[n]
        assert created[path_of(res.pool, n)] == n


def test_beam_select_equals_full_sort_over_kV():
    rng = np.random.default_rng(9)
    k, V = 4, 300
    pool = O.Pool(k=k, D=3)
    z0 = (rng.standard_normal((1, V)) * 3).astype(np.float32)
    tok, lp, lse = O.lmhead_topk(z0, k)
    beam = O.beam_first(pool, 1, tok[0], lp[0])
    z1 = (rng.standard_normal((k, V)) * 3).astype(np.float32)
    tok1, lp1, lse1 = O.lmhead_topk(z1, k)
    nb = O.beam_expand(pool, beam, 1, tok1, lp1)
    top, _ = BF.global_topk_over_kV(beam.logprobsum, z1, lse1, k)
    assert [(int(a), int(b)) for a, b in zip(nb.parent_slot, nb.token)] == [(i, v) for i, v, _ in top]
    assert [np.float32(s) for s in nb.logprobsum] == [s for _, _, s in top]


# ----------------------------------------------------------------------------------------------
# planted mistakes: the pins above must notice them
# ----------------------------------------------------------------------------------------------
def test_pins_catch_planted_mistakes(monkeypatch, tiny):
    wl, W = tiny

    def run_checks():
        res, tgt, (ln, path, bonus) = SR.oracle_round(wl, W, None, 0, 5, threshold=0.0)
        _check_round_invariants(wl.with_(threshold=0.0), res)
        _check_tree(wl, res)
        n = res.tree.n_sel + 1
        bl, bn = BF.accept_len_enumerate(res.tree.parent_idx, res.tree.tree_token, n, tgt)
        assert ln == bl and path[ln] == bn

    run_checks()                                               # the unmodified oracle passes

    # (1) ascending instead of descending row top-k
    good = O.row_topk
    monkeypatch.setattr(O, "row_topk", lambda z, k: good(-np.asarray(z), k))
    with pytest.raises((AssertionError, KeyError, ValueError, IndexError)):
        run_checks()
    monkeypatch.setattr(O, "row_topk", good)

    # (2) dropped parent term in the score
    good_expand = O.beam_expand

    def bad_expand(pool, beam, s, tok, lp):
        zero = O.Beam(beam.node, beam.token, beam.parent_slot, np.zeros_like(beam.logprobsum))
        return good_expand(pool, zero, s, tok, lp)
    monkeypatch.setattr(O, "beam_expand", bad_expand)
    with pytest.raises((AssertionError, KeyError, ValueError, IndexError)):
        run_checks()
    monkeypatch.setattr(O, "beam_expand", good_expand)

    # (3) wrong sign in the logsoftmax
    good_lp = O.logsumexp_row
    monkeypatch.setattr(O, "logsumexp_row", lambda z: -good_lp(z))
    with pytest.raises((AssertionError, KeyError, ValueError, IndexError)):
        run_checks()
    monkeypatch.setattr(O, "logsumexp_row", good_lp)

    # (4) mask without the ancestors beyond the parent
    good_fin = O.tree_finalize

    def bad_fin(pool, m):
        tr = good_fin(pool, m)
        n = tr.n_sel + 1
        tr.mask[:] = 0
        for i in range(n):
            tr.mask[i, i] = 1
            if tr.parent_idx[i] >= 0:
                tr.mask[i, tr.parent_idx[i]] = 1
        return tr
    monkeypatch.setattr(O, "tree_finalize", bad_fin)
    with pytest.raises((AssertionError, KeyError, ValueError, IndexError)):
        run_checks()
    monkeypatch.setattr(O, "tree_finalize", good_fin)

    # (5) accept walk that compares with the child's own target instead of the parent's
    good_ver = O.verify_accept

    def bad_ver(tree, tgt, D):
        shifted = np.roll(np.asarray(tgt), 1)
        return good_ver(tree, shifted, D)
    monkeypatch.setattr(O, "verify_accept", bad_ver)
    with pytest.raises((AssertionError, KeyError, ValueError, IndexError)):
        run_checks()
    monkeypatch.setattr(O, "verify_accept", good_ver)
    run_checks()
