"""GPU parity of ddd_verify_sample (sampled acceptance at temperature > 0) against
oracle/verify_sample.py, through the C ABI.  Accept lengths, paths and bonus tokens are integers
and must agree exactly; both sides take every decision in fp64, and each case checks that no
decision of the oracle sits within summation-order rounding of its threshold."""
import numpy as np
import pytest

import synth
from oracle import ddd_oracle as O
from oracle.verify_sample import verify_sample

pytestmark = pytest.mark.gpu

# relative distance of a decision from its threshold below which fp64 summation order could matter
MIN_MARGIN = 1e-10


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device (an MI355X)")
    import paper_2409_00142_amd as D
    return torch, D


def _oracle_tree(tok, par, n_sel, m):
    pos = np.zeros(m + 1, np.int32)
    for i in range(1, n_sel + 1):
        pos[i] = pos[par[i]] + 1
    return O.Tree(m=m, n_sel=n_sel, sel_node=np.full(m, -1, np.int32), tree_token=tok, pos=pos, parent_idx=par,
                  mask=np.zeros((m + 1, m + 1), np.uint8))


def _run(torch, D, B, V, k, Dm, m, toks, pars, n_sels, logits, T, ua, ub):
    cfg = D.make_config(B, 256, V, k, Dm, m, 0.3)
    ctx = D.ddd_create(cfg)
    try:
        tree, tree_t = D.alloc_tree(cfg)
        tree_t["tree_token"].copy_(torch.from_numpy(np.stack(toks)).view_as(tree_t["tree_token"]))
        tree_t["parent_idx"].copy_(torch.from_numpy(np.stack(pars)).view_as(tree_t["parent_idx"]))
        tree_t["n_sel"].copy_(torch.tensor(n_sels, dtype=torch.int32))
        lg = torch.from_numpy(logits).cuda()
        alen = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        apath = torch.full((B, Dm + 1), -7, dtype=torch.int32, device="cuda")
        bonus = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        # statistics bound without the rounds' depths: accepted lengths and the round count only
        acc_hist = torch.zeros(32, dtype=torch.int64, device="cuda")
        n_rounds = torch.zeros(1, dtype=torch.int64, device="cuda")
        D.ddd_stats_bind(ctx, rounds=n_rounds, accept_hist=acc_hist)
        D.ddd_verify_sample(ctx, tree, lg, T, torch.from_numpy(ua).cuda(), torch.from_numpy(ub).cuda(), alen, apath, bonus)
        torch.cuda.synchronize()
        assert int(n_rounds.item()) == 1
        assert np.array_equal(acc_hist.cpu().numpy(), np.bincount(np.minimum(alen.cpu().numpy(), 31), minlength=32))
        return alen.cpu().numpy(), apath.cpu().numpy(), bonus.cpu().numpy()
    finally:
        D.ddd_destroy(ctx)


CASES = [
    # name, B, V, k, D, m, n_sel per sequence, temperature
    ("small_vocab_below_one_pass", 3, 1000, 4, 6, 20, [20, 11, 0], 1.0),
    ("7b_shape", 4, 32000, 10, 10, 60, [60, 60, 33, 60], 0.7),
    ("large_vocab", 2, 128256, 10, 10, 60, [60, 45], 1.0),
    ("wide_beam_many_children", 1, 5003, 100, 2, 127, [127], 1.5),
    ("cold", 2, 32000, 10, 10, 60, [60, 60], 0.05),
    ("7b_b64_shape", 64, 32000, 10, 10, 60, [60] * 40 + [37] * 24, 0.9),      # the batch the benchmark times
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_verify_sample_against_oracle(gpu, case):
    torch, D = gpu
    name, B, V, k, Dm, m, n_sels, T = case
    print(f"[case] verify_sample {name} B={B} V={V} k={k} D={Dm} m={m} n_sel={n_sels} T={T}", flush=True)
    seed = sum(map(ord, name))
    rng = np.random.default_rng(seed)
    toks, pars, lgs = [], [], []
    for b in range(B):
        tok, par = synth.make_random_tree(m, n_sels[b], k, V, Dm, seed=seed * 100 + b)
        toks.append(tok)
        pars.append(par)
        lgs.append(synth.make_target_logits(tok, par, n_sels[b], V, seed=seed * 100 + b, agree=1.0 if name == "cold" else 0.9))
    logits = np.stack(lgs)
    ua, ub = rng.random((B, m + 1)), rng.random((B, m + 1))
    T32 = float(np.float32(T))
    alen, apath, bonus = _run(torch, D, B, V, k, Dm, m, toks, pars, n_sels, logits, T32, ua, ub)
    total_len = 0
    for b in range(B):
        mg = []
        o_len, o_path, o_bonus = verify_sample(_oracle_tree(toks[b], pars[b], n_sels[b], m), logits[b], T32, ua[b], ub[b],
                                               Dm, margins=mg)
        assert min(mg) > MIN_MARGIN, f"seed gives a decision at rounding distance from its threshold: {min(mg)}"
        assert int(alen[b]) == o_len, (b, alen[b], o_len)
        assert np.array_equal(apath[b], o_path), (b, apath[b], o_path)
        assert int(bonus[b]) == o_bonus, (b, bonus[b], o_bonus)
        total_len += o_len
    if name in ("7b_shape", "cold"):
        assert total_len >= B           # the case exercises accepted paths, not only rejections


def test_verify_sample_degenerate_rows(gpu):
    """Exact-arithmetic corner cases (weights are 0 or 1, so both sides compute the same numbers):
    a child that holds all the mass is accepted for any u < 1; uniforms of exactly 1 (outside the
    documented range) reach the two fallbacks of the bonus draw."""
    torch, D = gpu
    print("[case] verify_sample degenerate rows", flush=True)
    B, V, k, Dm, m = 3, 300, 4, 3, 4
    ninf = np.float32(-np.inf)
    toks = [np.array([0, 5, 9, -1, -1], np.int32)] * B
    pars = [np.array([-1, 0, 1, -1, -1], np.int32)] * B
    n_sels = [2, 2, 2]
    logits = np.full((B, m + 1, V), ninf, np.float32)
    ua = np.full((B, m + 1), 0.999)
    ub = np.full((B, m + 1), 0.25)
    # sequence 0: all mass on the child's token at the root and at node 1, token 17 at the leaf
    logits[0, 0, 5] = 1.0
    logits[0, 1, 9] = 2.0
    logits[0, 2, 17] = 0.5
    # sequence 1: the only live token is 40 and u_bonus = 1: no prefix exceeds the threshold -> last live token
    logits[1, 0, 40] = 0.0
    ub[1, 0] = 1.0
    # sequence 2: the child holds all the mass but u_accept = 1 rejects it: nothing is left -> the row's argmax
    logits[2, 0, 5] = 3.0
    ua[2, 1] = 1.0
    alen, apath, bonus = _run(torch, D, B, V, k, Dm, m, toks, pars, n_sels, logits, 1.0, ua, ub)
    for b in range(B):
        o_len, o_path, o_bonus = verify_sample(_oracle_tree(toks[b], pars[b], 2, m), logits[b], 1.0, ua[b], ub[b], Dm)
        assert (int(alen[b]), int(bonus[b])) == (o_len, o_bonus), b
        assert np.array_equal(apath[b], o_path)
    assert (alen.tolist(), bonus.tolist()) == ([2, 0, 0], [17, 40, 5])


def test_verify_sample_cold_equals_greedy(gpu):
    """At a very low temperature the sampled walk equals ddd_verify_accept on the target's argmax."""
    torch, D = gpu
    print("[case] verify_sample cold equals greedy", flush=True)
    B, V, k, Dm, m = 2, 4000, 10, 10, 60
    toks, pars = zip(*[synth.make_random_tree(m, 60, k, V, Dm, seed=50 + b) for b in range(B)])
    logits = np.stack([synth.make_target_logits(toks[b], pars[b], 60, V, seed=60 + b) for b in range(B)])
    rng = np.random.default_rng(9)
    ua, ub = rng.random((B, m + 1)), rng.random((B, m + 1))
    cfg = D.make_config(B, 256, V, k, Dm, m, 0.3)
    ctx = D.ddd_create(cfg)
    try:
        tree, tree_t = D.alloc_tree(cfg)
        tree_t["tree_token"].copy_(torch.from_numpy(np.stack(toks)).view_as(tree_t["tree_token"]))
        tree_t["parent_idx"].copy_(torch.from_numpy(np.stack(pars)).view_as(tree_t["parent_idx"]))
        tree_t["n_sel"].copy_(torch.tensor([60] * B, dtype=torch.int32))
        mk = lambda *s: torch.zeros(*s, dtype=torch.int32, device="cuda")
        l1, p1, b1, l2, p2, b2 = mk(B), mk(B, Dm + 1), mk(B), mk(B), mk(B, Dm + 1), mk(B)
        lg = torch.from_numpy(logits).cuda()
        D.ddd_verify_sample(ctx, tree, lg, 1e-3, torch.from_numpy(ua).cuda(), torch.from_numpy(ub).cuda(), l1, p1, b1)
        D.ddd_verify_accept(ctx, tree, lg.argmax(dim=2).to(torch.int32).contiguous(), l2, p2, b2)
        torch.cuda.synchronize()
        assert torch.equal(l1, l2) and torch.equal(p1, p2) and torch.equal(b1, b2)
        assert int(l1.sum()) >= 2
    finally:
        D.ddd_destroy(ctx)


def test_verify_sample_rejects_bad_arguments(gpu):
    torch, D = gpu
    print("[case] verify_sample argument checks", flush=True)
    cfg = D.make_config(1, 256, 1000, 4, 4, 8, 0.3)
    ctx = D.ddd_create(cfg)
    try:
        tree, _ = D.alloc_tree(cfg)
        lg = torch.zeros(1, 9, 1000, device="cuda")
        u = torch.zeros(1, 9, dtype=torch.float64, device="cuda")
        i32 = lambda *s: torch.zeros(*s, dtype=torch.int32, device="cuda")
        for bad_T in (0.0, -1.0, float("nan"), float("inf")):
            with pytest.raises(D.DDDError):
                D.ddd_verify_sample(ctx, tree, lg, bad_T, u, u, i32(1), i32(1, 5), i32(1))
        with pytest.raises(D.DDDError):
            D.ddd_verify_sample(ctx, tree, None, 1.0, u, u, i32(1), i32(1, 5), i32(1))
        with pytest.raises(D.DDDError):
            D.ddd_verify_sample(ctx, tree, lg, 1.0, None, u, i32(1), i32(1, 5), i32(1))
    finally:
        D.ddd_destroy(ctx)
