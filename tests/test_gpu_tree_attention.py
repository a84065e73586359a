"""GPU parity of ddd_tree_attention (the consumer of the final tree's mask) against oracle/tree_attention.py,
through the C ABI."""
import numpy as np
import pytest

import synth
from oracle import bruteforce as BF
from oracle import tree_attention as OT

pytestmark = pytest.mark.gpu

# The weights of the second product are rounded to bf16 (2^-9 relative) before they meet the values on the
# matrix cores, and exp is the fast fp32 one; with values of order one (|v| < 5 here) the output error stays
# below 5 * 2^-9 = 1e-2.
ATTN_TOL = 1e-2


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device (an MI355X)")
    import paper_2409_00142_amd as D
    from synth import device as SD
    return torch, D, SD


def _random_tree(rng, T, n_sel):
    """parent_idx of a random tree over tree indices 0..n_sel (parents precede children), -1 padded."""
    parent = [-1] * T
    for i in range(1, n_sel + 1):
        parent[i] = int(rng.integers(0, i))
    return parent


CASES = [
    # name, B, m, n_heads, L, n_sel per sequence
    ("no_prompt_small", 1, 20, 2, 0, [20]),
    ("ragged_prompt_two_sequences", 2, 60, 4, 100, [60, 37]),
    ("two_query_tiles", 1, 127, 3, 1000, [127]),
    ("short_tree_long_prompt", 1, 60, 8, 2048, [9]),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_tree_attention_against_oracle(gpu, case):
    name, B, m, nh, L, n_sels = case
    _check_case(gpu, name, B, m, nh, L, n_sels, seed=sum(map(ord, name)))


def _random_cases(n=24, seed=9):
    """Seeded random shapes: trees of 1..128 rows, 0..2100 prompt positions (ragged against the 32-key chunks and the
    split sizes), 1..8 heads, 1..5 sequences with trees of different sizes (empty ones included)."""
    import random
    rnd = random.Random(seed)
    out = []
    while len(out) < n:
        B, m, nh = rnd.choice([1, 1, 2, 3, 5]), rnd.choice([1, 2, 20, 31, 32, 60, 63, 64, 100, 127]), rnd.choice([1, 2, 3, 8])
        L = rnd.choice([0, 1, 31, 32, 33, 100, 255, 256, 1000, 2100])
        if B * nh * (L + m) > 12000:
            continue
        out.append(("random%d" % len(out), B, m, nh, L, [rnd.randint(0, m) for _ in range(B)]))
    return out


def test_tree_attention_random_shapes(gpu):
    for i, (name, B, m, nh, L, n_sels) in enumerate(_random_cases()):
        _check_case(gpu, name, B, m, nh, L, n_sels, seed=500 + i)


def _check_case(gpu, name, B, m, nh, L, n_sels, seed):
    torch, D, SD = gpu
    T, d = m + 1, 128
    print(f"[case] tree attention {name} B={B} m={m} heads={nh} L={L} n_sel={n_sels}", flush=True)
    rng = np.random.default_rng(seed)
    bits = lambda shape: synth.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    q, kt, vt = bits((B, T, nh, d)), bits((B, T, nh, d)), bits((B, T, nh, d))
    kp, vp = bits((B, L, nh, d)), bits((B, L, nh, d))
    Tp, Lp = (T + 31) // 32 * 32, (L + 31) // 32 * 32
    vt_t = np.zeros((B, nh, d, Tp), dtype=np.uint16)
    vt_t[:, :, :, :T] = vt.transpose(0, 2, 3, 1)
    parents = [_random_tree(rng, T, n_sels[b]) for b in range(B)]
    masks = np.zeros((B, T, T), dtype=np.uint8)
    for b in range(B):
        n = n_sels[b] + 1
        masks[b, :n, :n] = np.array(BF.closure_mask(parents[b][:n], n), dtype=np.uint8)

    cfg = D.make_config(B, 256, 1000, 4, 4, m, 0.3)
    ctx = D.ddd_create(cfg)
    try:
        tree, tree_t = D.alloc_tree(cfg)
        tree_t["mask"].copy_(torch.from_numpy(masks).view_as(tree_t["mask"]))
        tree_t["n_sel"].copy_(torch.tensor(n_sels, dtype=torch.int32))
        ws = torch.empty(max(1, D.ddd_tree_attention_workspace(ctx, nh, L) // 4), dtype=torch.float32, device="cuda")
        out = torch.full((B, T, nh, d), float("nan"), dtype=torch.float32, device="cuda")
        up = SD.upload_bits
        kpk = vpk = None
        if L:
            n_packed = B * nh * (Lp // 32) * 4096
            kpk = torch.full((n_packed,), float("nan"), dtype=torch.bfloat16, device="cuda")
            vpk = torch.full((n_packed,), float("nan"), dtype=torch.bfloat16, device="cuda")
            D.ddd_kv_pack(ctx, up(kp), up(vp), L, nh, kpk, vpk)
        args = (up(q), up(kt), up(vt_t), kpk, vpk)
        D.ddd_tree_attention(ctx, tree, *args, L, nh, ws, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        D.ddd_tree_attention(ctx, tree, *args, L, nh, ws, out)     # deterministic: the same bits again
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), got)
    finally:
        D.ddd_destroy(ctx)
    f = OT.bf16_bits_to_f64
    assert not np.isnan(got).any()
    for b in range(B):
        want = OT.tree_attention(f(q[b]), f(kt[b]), f(vt[b]), f(kp[b]), f(vp[b]), masks[b], n_sels[b])
        assert np.max(np.abs(got[b] - want)) <= ATTN_TOL, float(np.max(np.abs(got[b] - want)))
        assert np.all(got[b, n_sels[b] + 1:] == 0.0)


def test_tree_attention_full_size_sampled(gpu):
    """The verification-pass shape the benchmark times (B = 64, 61 tree nodes, 32 heads, prompt 2048, one key
    split per head): the oracle recomputes sampled (sequence, head) pairs."""
    torch, D, SD = gpu
    B, m, nh, L, d = 64, 60, 32, 2048, 128
    T, Tp = m + 1, 64
    print(f"[case] tree attention full size B={B} m={m} heads={nh} L={L}, sampled heads", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(77)
    rnd = lambda *s: torch.randn(*s, device="cuda", generator=gen).to(torch.bfloat16)
    q, kt, vt = rnd(B, T, nh, d), rnd(B, T, nh, d), rnd(B, T, nh, d)
    vtt = torch.zeros(B, nh, d, Tp, device="cuda", dtype=torch.bfloat16)
    vtt[..., :T] = vt.permute(0, 2, 3, 1)
    kp, vp = rnd(B, L, nh, d), rnd(B, L, nh, d)
    rng = np.random.default_rng(78)
    n_sels = [int(x) for x in rng.integers(20, m + 1, size=B)]
    parents = [_random_tree(rng, T, n_sels[b]) for b in range(B)]
    masks = np.zeros((B, T, T), dtype=np.uint8)
    for b in range(B):
        n = n_sels[b] + 1
        masks[b, :n, :n] = np.array(BF.closure_mask(parents[b][:n], n), dtype=np.uint8)
    cfg = D.make_config(B, 256, 1000, 4, 4, m, 0.3)
    ctx = D.ddd_create(cfg)
    try:
        tree, tree_t = D.alloc_tree(cfg)
        tree_t["mask"].copy_(torch.from_numpy(masks).view_as(tree_t["mask"]))
        tree_t["n_sel"].copy_(torch.tensor(n_sels, dtype=torch.int32))
        ws = torch.empty(max(1, D.ddd_tree_attention_workspace(ctx, nh, L) // 4), dtype=torch.float32, device="cuda")
        out = torch.full((B, T, nh, d), float("nan"), dtype=torch.float32, device="cuda")
        kpk = torch.empty(B * nh * (L // 32) * 4096, dtype=torch.bfloat16, device="cuda")
        vpk = torch.empty_like(kpk)
        D.ddd_kv_pack(ctx, kp, vp, L, nh, kpk, vpk)
        D.ddd_tree_attention(ctx, tree, q, kt, vtt, kpk, vpk, L, nh, ws, out)
        torch.cuda.synchronize()
        assert not torch.isnan(out).any()
        f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
        for b, h in [(0, 0), (63, 31), (17, 5), (40, 20), (5, 30), (29, 11)]:
            want = OT.tree_attention(f64(q[b, :, h:h + 1]), f64(kt[b, :, h:h + 1]), f64(vt[b, :, h:h + 1]),
                                     f64(kp[b, :, h:h + 1]), f64(vp[b, :, h:h + 1]), masks[b], n_sels[b])
            got = out[b, :, h:h + 1].cpu().numpy().astype(np.float64)
            assert np.max(np.abs(got - want)) <= ATTN_TOL, (b, h, float(np.max(np.abs(got - want))))
            assert np.all(got[n_sels[b] + 1:] == 0.0)
    finally:
        D.ddd_destroy(ctx)
