"""The allocation-free variant of ddd_lmhead_topk (static device scratch) against ddd_lmhead_topk itself:
same kernels, so every output bit must be equal; two calls in a row, the second with a smaller input, so that
nothing the first call left in the shared scratch may leak into the second."""
import numpy as np
import pytest

import synth
from oracle import ddd_oracle as O

pytestmark = pytest.mark.gpu

# name,  k,  H,    V,    R, sigma_w, hidden scale
CALLS = [
    ("first_larger", 10, 1024, 5003, 10, 0.03, 3.0),
    ("second_smaller", 4, 256, 1000, 3, 0.05, 5.0),
    ("third_full_rows", 16, 2048, 3001, 16, 0.02, 3.0),
]


def test_static_entry_point_matches_the_context_one_on_consecutive_calls():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device (an MI355X)")
    import paper_2409_00142_amd as D
    from synth import device as SD
    assert D.ddd_static_scratch_bytes() == 16 * 16 * 256 * 8 + 16 * 256 * 4
    prepared = []
    for name, k, H, V, R, sigma, hscale in CALLS:
        rng = np.random.default_rng(sum(map(ord, name)))
        W_bits = synth.make_lm_head(V, H, sigma, seed=9)
        hid_bits = synth.f32_to_bf16_bits((rng.standard_normal((R, H)) * hscale).astype(np.float32))
        cfg = D.make_config(2, H, V, k, 4, 8, 0.3)
        act_np = np.ones(R, np.uint8)
        if R >= 3:
            act_np[1] = 0                                   # an inactive row stays untouched on both paths
        out = {n: (torch.full((R, k), -7, dtype=torch.int32, device="cuda"),
                   torch.full((R, k), 9.0, dtype=torch.float32, device="cuda"),
                   torch.full((R,), 9.0, dtype=torch.float32, device="cuda")) for n in ("static", "ctx")}
        prepared.append((name, cfg, SD.upload_bits(W_bits), SD.upload_bits(hid_bits), torch.from_numpy(act_np).cuda(),
                         R, k, out, W_bits, hid_bits, act_np))
    torch.cuda.synchronize()
    # the static calls back to back on one stream (they share the one scratch array, the stream orders them)
    for name, cfg, W, hid, act, R, k, out, *_ in prepared:
        print(f"[case] ddd_lmhead_topk_static {name} k={k} H={cfg.H} V={cfg.V} R={R}", flush=True)
        D.ddd_lmhead_topk_static(cfg, W, hid, R, act, *out["static"])
    torch.cuda.synchronize()
    for name, cfg, W, hid, act, R, k, out, W_bits, hid_bits, act_np in prepared:
        ctx = D.ddd_create(cfg)
        try:
            D.ddd_lmhead_topk(ctx, W, hid, R, act, *out["ctx"], None)
            torch.cuda.synchronize()
        finally:
            D.ddd_destroy(ctx)
        for a, b in zip(out["static"], out["ctx"]):
            assert torch.equal(a, b), name
        tok = out["static"][0].cpu().numpy()
        logits = O.lmhead_logits(W_bits, hid_bits)
        for r in range(R):
            if act_np[r]:
                assert set(tok[r]) == set(O.row_topk(logits[r], k).tolist()), (name, r)
            else:
                assert (tok[r] == -7).all(), (name, r)
    # beyond the static scratch: a clear status, nothing enqueued
    name, cfg, W, hid, act, R, k, out, *_ = prepared[0]
    with pytest.raises(D.DDDError) as e:
        D.ddd_lmhead_topk_static(cfg, W, hid, D.DDD_STATIC_ROWS + 1, None, *out["static"])
    assert e.value.code == D.DDD_ERR_STATIC_LIMIT
    wide = D.make_config(1, 256, 1000, 17, 3, 8, 0.3)
    with pytest.raises(D.DDDError) as e:
        D.ddd_lmhead_topk_static(wide, W, hid, 1, None, *out["static"])
    assert e.value.code == D.DDD_ERR_STATIC_LIMIT
    with pytest.raises(D.DDDError) as e:
        D.ddd_lmhead_topk_static(cfg, None, hid, 1, None, *out["static"])
    assert e.value.code == D.DDD_ERR_INVALID_ARG
