"""GPU parity of the stand-in draft layer (include/ddd_body.h) against oracle/body.py, through the C ABI.

The layer's outputs are bf16 rows computed in fp32 on the GPU and in fp64 by the oracle, with bf16 rounding at
the same five points; a rounding tie can fall differently, so rows are compared within a tolerance stated
below, and the integers of a round are compared by replaying the GPU's logits in the oracle."""
import numpy as np
import pytest

import synth
from oracle import body as OB
from oracle import ddd_oracle as O

pytestmark = pytest.mark.gpu

# A hidden row is a sum of terms of the size of the row's rms (the residual stream, the attention and MLP
# branches), each carrying bf16 roundings (2^-9 relative) taken at five points, by fp32 arithmetic on one side
# and fp64 on the other; a tie that rounds the other way moves a term by one bf16 ulp, and a call's rows are the
# next call's inputs.  Allowed: two ulps of the element (2^-6 relative) plus 2^-5 of the row's rms.
ROW_RTOL, ROW_ATOL_RMS = 2.0 ** -6, 2.0 ** -5
LINEAR_TOL = 2e-3          # fp32 accumulation of <= 11008 products of order-one sums


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device (an MI355X)")
    import paper_2409_00142_amd as D
    from synth import device as SD
    return torch, D, SD


def _body_inputs(torch, SD, V, H, F, L, B, seed=0, root_token=3):
    wb = synth.make_body_weights(V, H, F, seed)
    pb = [synth.make_prompt_context(L, H, seed + 10 * b) for b in range(B)]
    dev_w = {n: (SD.upload_bits(wb[n]) if wb[n].dtype == np.uint16 else torch.from_numpy(wb[n]).cuda()) for n in wb}
    dev_p = {
        "K": SD.upload_bits(np.stack([p["K"] for p in pb])),
        "V": SD.upload_bits(np.stack([p["V"] for p in pb])),
        "f_root": SD.upload_bits(np.stack([p["f_root"] for p in pb])),
        "root_token": torch.full((B,), root_token, dtype=torch.int32, device="cuda"),
    }
    ow = OB.LayerWeights(wb["E"], wb["Wfc"], wb["g1"], wb["Wqkv"], wb["Wo"], wb["g2"], wb["Wgu"], wb["Wd"])
    op = [OB.Prompt(p["K"], p["V"], p["f_root"]) for p in pb]
    return dev_w, dev_p, ow, op


def _rows_close(got_bits, want_bits):
    g = synth.bf16_bits_to_f32(got_bits).astype(np.float64)
    w = synth.bf16_bits_to_f32(want_bits).astype(np.float64)
    err = np.abs(g - w)
    rms = np.sqrt(np.mean(w * w, axis=1, keepdims=True))
    assert np.all(err <= ROW_ATOL_RMS * rms + ROW_RTOL * np.abs(w)), float(err.max())
    # and most elements land on the same or the neighbouring bf16 value (fewer in later calls, whose inputs are
    # the earlier calls' rows on either side)
    assert np.mean(err <= 2.0 ** -7 * np.maximum(1.0, np.abs(w))) > 0.85


def _bits(t):
    return t.view(__import__("torch").int16).cpu().numpy().view(np.uint16)


LINEAR_CASES = [
    # name, N, K, R
    ("one_range", 300, 256, 5),
    ("two_ranges_1408", 1000, 1408, 16),          # 128*11 = 1280 + 128
    ("k8192", 520, 8192, 10),                      # 5120 + 3072
    ("k11008_ragged_N", 1037, 11008, 3),           # 5120 + 5120 + 768; N not a multiple of 16
    # more than 16 rows: the MFMA path (128 x 128 tiles when the product has few of them, wider ones otherwise)
    ("gemm_rows40", 512, 1024, 40),
    ("gemm_rows130_k8192", 520, 8192, 130),
    ("gemm_rows24_k11008_ragged_N", 1036, 11008, 24),
    ("gemm_rows330_wide_tiles", 33000, 256, 330),
]


@pytest.mark.parametrize("case", LINEAR_CASES, ids=[c[0] for c in LINEAR_CASES])
def test_body_linear_against_oracle(gpu, case):
    torch, D, SD = gpu
    name, N, K, R = case
    print(f"[case] body linear {name} N={N} K={K} R={R}", flush=True)
    rng = np.random.default_rng(sum(map(ord, name)))
    W_bits = synth.f32_to_bf16_bits((rng.standard_normal((N, K)) * K ** -0.5).astype(np.float32))
    x_bits = synth.f32_to_bf16_bits(rng.standard_normal((R, K)).astype(np.float32))
    body = D.ddd_body_create(D.ddd_body_config(max(1, (R + 3) // 4), 4, 256, 256, 10, 2, 0))
    try:
        W, x = SD.upload_bits(W_bits), SD.upload_bits(x_bits)
        y = torch.full((R, N), float("nan"), dtype=torch.float32, device="cuda")
        D.ddd_body_linear(body, W, N, K, x, R, y)
        torch.cuda.synchronize()
        y1 = y.cpu().numpy()
        D.ddd_body_linear(body, W, N, K, x, R, y, accumulate=True)
        torch.cuda.synchronize()
        y2 = y.cpu().numpy()
    finally:
        D.ddd_body_destroy(body)
    want = O.lmhead_logits(W_bits, x_bits).astype(np.float64)     # the same contraction, summed in fp64
    assert not np.isnan(y1).any()
    assert np.max(np.abs(y1 - want)) <= LINEAR_TOL
    assert np.max(np.abs(y2 - 2.0 * want)) <= 2 * LINEAR_TOL


class _Beam:
    def __init__(self, token, parent_slot):
        self.token, self.parent_slot = np.asarray(token), np.asarray(parent_slot)


@pytest.mark.parametrize("B,k", [(2, 3), (6, 3), (20, 2)], ids=lambda v: str(v))
def test_body_steps_with_scripted_beams(gpu, B, k):
    """Four calls with scripted beams (seeded tokens and parent slots); some sequences stop after call 1 or 2, and
    their rows must be left untouched from then on.  B*k <= 16: every linear is a weight stream; more rows: the
    MFMA path (B = 6: from the second call on; B = 20: for the prompt call as well)."""
    torch, D, SD = gpu
    H, F, V, L, Dm = 256, 384, 60, 7, 4
    print(f"[case] body scripted beams B={B} k={k} H={H} F={F} L={L}", flush=True)
    dev_w, dev_p, ow, op = _body_inputs(torch, SD, V, H, F, L, B)
    cfg = D.make_config(B, H, V, k, Dm, 8, 0.3)
    st, st_t = D.alloc_state(cfg)
    rng = np.random.default_rng(100 * B + k)
    beams = [None] + [[(rng.integers(0, V, k).tolist(), [0] * k if s == 1 else rng.integers(0, k, k).tolist())
                       for b in range(B)] for s in range(1, Dm)]
    stop_after = [int(rng.integers(1, Dm + 1)) if b % 2 == 1 else Dm for b in range(B)]      # calls a sequence makes
    active = [None] + [[1 if s < stop_after[b] else 0 for b in range(B)] for s in range(1, Dm)]
    body = D.ddd_body_create(D.ddd_body_config(B, k, H, F, V, Dm, L))
    obodies = [OB.StandInBody(ow, op[b], root_token=3) for b in range(B)]
    try:
        D.ddd_body_bind(body, dev_w, dev_p)
        hid = torch.zeros(B * k, H, dtype=torch.bfloat16, device="cuda")
        for s in range(Dm):
            if s >= 1:
                st_t["beam_token"].copy_(torch.tensor([t for b in range(B) for t in beams[s][b][0]], dtype=torch.int32)
                                         .view_as(st_t["beam_token"]))
                st_t["beam_parent_slot"].copy_(torch.tensor([t for b in range(B) for t in beams[s][b][1]],
                                                            dtype=torch.int32).view_as(st_t["beam_parent_slot"]))
                st_t["row_active"].copy_(torch.tensor([active[s][b] for b in range(B) for _ in range(k)],
                                                      dtype=torch.uint8).view_as(st_t["row_active"]))
            hid.fill_(7.0)                                        # sentinel: skipped rows keep it
            D.ddd_body_step(body, s, st, hid)
            torch.cuda.synchronize()
            got = _bits(hid)
            for b in range(B):
                if s == 0:
                    want = obodies[b](0, None, None)
                    _rows_close(got[b:b + 1], want)
                elif active[s][b]:
                    want = obodies[b](s, _Beam(*beams[s][b]), None)
                    _rows_close(got[b * k:(b + 1) * k], want)
                else:
                    assert np.all(synth.bf16_bits_to_f32(got[b * k:(b + 1) * k]) == 7.0)
    finally:
        D.ddd_body_destroy(body)


@pytest.mark.parametrize("shape", [("tiny", 1, 4, 256, 384, 500, 9, 5), ("k10_h1024", 1, 10, 1024, 2816, 3000, 33, 6),
                                   # the shape the benchmark's --body layer times: 7B sizes, 32 heads, 256 prompt positions
                                   ("7b_full_shape", 1, 10, 4096, 11008, 32000, 256, 3),
                                   # several sequences, more than 16 rows per call: the MFMA path of the layer and of the LM head
                                   ("b5_k6_gemm_rows", 5, 6, 512, 1024, 2000, 17, 4),
                                   # the same with a stop threshold: the sequences stop after different calls, the later
                                   # calls run the layer on the rows that are left
                                   ("b7_k6_gemm_ragged_stops", 7, 6, 512, 1024, 2000, 17, 5, 0.03),
                                   # prompts of 32 positions and more: the batched attention takes the prompt part to
                                   # the matrix cores (a ragged last tile of keys; more than 256 keys: two passes;
                                   # sequences that stop)
                                   ("b5_k6_prompt_mfma_ragged", 5, 6, 512, 1024, 2000, 70, 4),
                                   ("b3_k10_prompt_mfma_two_passes", 3, 10, 256, 384, 1000, 272, 3),
                                   ("b7_k6_prompt_mfma_stops", 7, 6, 512, 1024, 2000, 40, 5, 0.03)],
                         ids=lambda s: s[0])
def test_round_with_body_matches_oracle(gpu, shape):
    """Whole rounds with the layer as the draft body: eager calls (rows inspected after every body call), then the
    same round from one captured graph.  The oracle replays the GPU's logits, so beams and trees must agree
    bit for bit, and its own layer must reproduce every hidden row within the tolerance."""
    torch, D, SD = gpu
    name, B, k, H, F, V, L, Dm = shape[:8]
    thr = shape[8] if len(shape) > 8 else 0.0     # t = 0: every call is made, the tree is built in the last one
    print(f"[case] round with body {name} B={B} k={k} H={H} F={F} V={V} L={L} D={Dm} t={thr}", flush=True)
    m, root = 12, 3
    dev_w, dev_p, ow, op = _body_inputs(torch, SD, V, H, F, L, B, seed=4, root_token=root)
    W_bits = synth.make_lm_head(V, H, 0.08, seed=11)
    W = SD.upload_bits(W_bits)
    cfg = D.make_config(B, H, V, k, Dm, m, thr)
    ctx = D.ddd_create(cfg)
    body = D.ddd_body_create(D.ddd_body_config(B, k, H, F, V, Dm, L))
    try:
        D.ddd_body_bind(body, dev_w, dev_p)
        st, st_t = D.alloc_state(cfg)
        tree, tree_t = D.alloc_tree(cfg)
        hid = torch.zeros(B * k, H, dtype=torch.bfloat16, device="cuda")
        root_token = torch.full((B,), root, dtype=torch.int32, device="cuda")
        logits = torch.zeros(Dm, B * k, V, dtype=torch.float32, device="cuda")
        D.ddd_round_reset(ctx, st, root_token)
        hid_rows = []
        for s in range(Dm):
            D.ddd_body_step(body, s, st, hid)
            torch.cuda.synchronize()
            hid_rows.append(_bits(hid).copy())
            D.ddd_draft_step(ctx, s, W, hid, st, tree, logits[s], None)
        torch.cuda.synchronize()
        g_logits = logits.cpu().numpy()
        eager_tree = {n: t.cpu().numpy().copy() for n, t in tree_t.items()}
        depths = []
        for b in range(B):
            steps = int(st_t["steps"].cpu()[b])
            # oracle round of this sequence on the GPU's logits, with its own layer producing the rows
            obody = OB.StandInBody(ow, op[b], root_token=root)
            o_rows = []

            def body_fn(s, beam, pool):
                rows = obody(s, beam, pool)
                o_rows.append(rows)
                return rows

            def logits_fn(s, hid_bits, b=b):
                return (g_logits[s, b:b + 1] if s == 0 else g_logits[s, b * k:(b + 1) * k]), None

            res = O.run_round(None, k, Dm, m, thr, 0xFFFFFFFF, body_fn, root_token=root, logits_fn=logits_fn)
            assert res.steps == steps and (steps >= 2 or thr > 0.0)
            depths.append(steps)
            if thr > 0.0:
                print(f"[info] {name} seq {b}: P after each call {[round(rec.P, 4) for rec in res.records]}", flush=True)
            for s in range(steps):
                rows = hid_rows[s][b:b + 1] if s == 0 else hid_rows[s][b * k:(b + 1) * k]
                _rows_close(rows, o_rows[s])
            assert np.array_equal(eager_tree["tree_token"][b], res.tree.tree_token)
            assert np.array_equal(eager_tree["parent_idx"][b], res.tree.parent_idx)
        print(f"[info] {name}: calls made per sequence {depths}", flush=True)
        if thr > 0.0:
            assert len(set(depths)) >= 2          # ragged: the sequences did stop at different depths
        # the same round from a captured graph gives the same bits
        side = torch.cuda.Stream()
        for t in tree_t.values():
            t.zero_()
        D.ddd_round_capture(ctx, W, st, tree, root_token, hid, D.body_step_ptr(), body, None, None, None, None,
                            stream=side.cuda_stream)
        for _ in range(2):
            D.ddd_round_launch(ctx, stream=side.cuda_stream)
        side.synchronize()
        torch.cuda.synchronize()
        for n, t in tree_t.items():
            assert np.array_equal(t.cpu().numpy(), eager_tree[n]), n
    finally:
        D.ddd_body_destroy(body)
        D.ddd_destroy(ctx)
