"""Device-side set-up of the synthetic workloads for the GPU tests and the benchmark.

Uploads the seeded inputs, fills the parameter block of the on-device stand-in draft body /
target model, and drives whole rounds through the C ABI binding.  Contains no method
arithmetic: every step of a round runs inside libddd.so; the stand-ins for
the draft body and the target model come from libddd_synth.so (native.py).
"""
from __future__ import annotations

import ctypes as C
from typing import Optional

import numpy as np
import torch

import paper_2409_00142_amd as D
from . import native as N
from .inputs import Workload, make_lm_head, make_plant_table


def upload_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on the GPU (bit-exact)."""
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


class GpuWorkload:
    """One context + caller-owned buffers for a synthetic workload."""

    def __init__(self, wl: Workload, W_bits: Optional[np.ndarray] = None, threshold: Optional[float] = None,
                 debug: bool = False, flags: int = 0):
        self.wl = wl
        self.W_bits = make_lm_head(wl.V, wl.H, wl.sigma_w, wl.seed, wl.dup_pairs) if W_bits is None else W_bits
        self.plant_tokens, self.plant_dir_np = make_plant_table(self.W_bits, wl)
        t = wl.threshold if threshold is None else threshold
        self.cfg = D.make_config(wl.B, wl.H, wl.V, wl.k, wl.D, wl.m, t, wl.check_mask, flags)
        self.ctx = D.ddd_create(self.cfg)
        self.W = upload_bits(self.W_bits)
        self.st, self.st_t = D.alloc_state(self.cfg)
        self.tree, self.tree_t = D.alloc_tree(self.cfg)
        B, k, H, V, Dm, m = wl.B, wl.k, wl.H, wl.V, wl.D, wl.m
        self.hid = torch.zeros(B * k, H, dtype=torch.bfloat16, device="cuda")
        self.root_token = torch.full((B,), wl.root_token, dtype=torch.int32, device="cuda")
        self.round_ctr = torch.zeros(1, dtype=torch.int64, device="cuda")
        self.plant_dir = torch.from_numpy(self.plant_dir_np).cuda() if wl.n_plant > 0 else None
        self.target = torch.full((B, m + 1), -1, dtype=torch.int32, device="cuda")
        self.accept_len = torch.zeros(B, dtype=torch.int32, device="cuda")
        self.accept_path = torch.full((B, Dm + 1), -1, dtype=torch.int32, device="cuda")
        self.bonus = torch.zeros(B, dtype=torch.int32, device="cuda")
        self.depth_hist = torch.zeros(32, dtype=torch.int64, device="cuda")
        self.accept_hist = torch.zeros(32, dtype=torch.int64, device="cuda")
        self.batch_depth_hist = torch.zeros(32, dtype=torch.int64, device="cuda")
        self.logits_dbg = torch.zeros(Dm, B * k, V, dtype=torch.float32, device="cuda") if debug else None
        self.lse_dbg = torch.zeros(Dm, B * k, dtype=torch.float32, device="cuda") if debug else None
        p = N.ddd_synth_params()
        p.cfg = self.cfg
        p.seed = wl.seed
        p.round_ctr = self.round_ctr.data_ptr()
        p.root_token = wl.root_token
        p.n_plant = wl.n_plant
        for d in range(32):
            p.scale_depth[d] = float(wl.scale(d))
        p.plant_dir = self.plant_dir.data_ptr() if self.plant_dir is not None else None
        p.plant_round_p24 = wl.plant_round_p24()
        p.plant_row_p24 = wl.plant_row_p24()
        self.params = p
        # post hook: stand-in target model, accept walk, advance the round counter (one C call per round)
        pa = N.ddd_synth_post_args()
        pa.params = C.addressof(self.params)
        pa.ctx = self.ctx
        pa.target_argmax = self.target.data_ptr()
        pa.accept_len = self.accept_len.data_ptr()
        pa.accept_path = self.accept_path.data_ptr()
        pa.bonus_token = self.bonus.data_ptr()
        # the histograms and the round counter are kept by the accept walk's own launch (ddd_stats_bind): no
        # separate statistics launch per round
        pa.depth_hist = None
        pa.accept_hist = None
        pa.batch_depth_hist = None
        D.ddd_stats_bind(self.ctx, rounds=self.round_ctr, depth_hist=self.depth_hist, accept_hist=self.accept_hist,
                         batch_depth_hist=self.batch_depth_hist, steps=self.st_t["steps"])
        pa.hash_tokens = None
        self.post_args = pa
        self.captured = False

    def set_round(self, rnd: int) -> None:
        self.round_ctr.fill_(rnd)

    def use_layer_body(self, F: int, L: int, seed: int = 0) -> None:
        """Replace the hash-based draft body by the stand-in draft layer (include/ddd_body.h) with seeded
        weights and prompt context; the workload must have at most 16 rows per call."""
        from .inputs import make_body_weights, make_prompt_context
        wl = self.wl
        wb = make_body_weights(wl.V, wl.H, F, seed)
        self.body_w = {n: (upload_bits(a) if a.dtype == np.uint16 else torch.from_numpy(a).cuda())
                       for n, a in wb.items()}
        pb = [make_prompt_context(L, wl.H, seed + 10 * b) for b in range(wl.B)]
        self.body_p = {
            "K": upload_bits(np.stack([p["K"] for p in pb])),
            "V": upload_bits(np.stack([p["V"] for p in pb])),
            "f_root": upload_bits(np.stack([p["f_root"] for p in pb])),
            "root_token": self.root_token,
        }
        self.post_args.hash_tokens = self.root_token.data_ptr()     # the layer's rounds differ by their last prompt token
        self._run_args = None
        self.body = D.ddd_body_create(D.ddd_body_config(wl.B, wl.k, wl.H, F, wl.V, wl.D, L))
        D.ddd_body_bind(self.body, self.body_w, self.body_p)
        self.body_bytes = sum(int(np.prod(wb[n].shape)) * 2 for n in ("Wfc", "Wqkv", "Wo", "Wgu", "Wd"))

    def _round_args(self):
        if getattr(self, "body", None) is not None:
            return (self.ctx, self.W, self.st, self.tree, self.root_token, self.hid, D.body_step_ptr(), self.body,
                    N.synth_post_ptr(), C.addressof(self.post_args), self.logits_dbg, self.lse_dbg)
        return (self.ctx, self.W, self.st, self.tree, self.root_token, self.hid, N.synth_draft_body_ptr(),
                C.addressof(self.params), N.synth_post_ptr(), C.addressof(self.post_args), self.logits_dbg, self.lse_dbg)

    def enqueue_round(self, stream: Optional[int] = None) -> None:
        """The whole round (reset, draft calls, tree, stand-in target, accept walk) without a graph."""
        D.ddd_round_enqueue(*self._round_args(), stream=stream)

    def run_round(self, stream: Optional[int] = None) -> int:
        """The whole round with the host pacing the draft calls (ddd_round_run); returns the calls queued."""
        a = getattr(self, "_run_args", None)
        if a is None:       # none of these pointers changes while the workload lives: marshal them once
            r = self._round_args()
            a = self._run_args = (r[0], r[1].data_ptr(), C.byref(r[2]), C.byref(r[3]), r[4].data_ptr(), r[5].data_ptr(),
                                  r[6], r[7], r[8], r[9])
            self._run_fn = D.load_library().ddd_round_run
        rc = self._run_fn(*a, D.current_stream() if stream is None else stream)
        if rc < 0:
            raise D.DDDError(rc, "ddd_round_run")
        return rc

    def capture(self, stream: torch.cuda.Stream) -> None:
        D.ddd_round_capture(*self._round_args(), stream=stream.cuda_stream)
        self.captured = True

    def launch(self, stream: Optional[int] = None) -> None:
        D.ddd_round_launch(self.ctx, stream=stream)

    def close(self) -> None:
        if getattr(self, "body", None) is not None:
            D.ddd_body_destroy(self.body)
            self.body = None
        if self.ctx is not None:
            D.ddd_destroy(self.ctx)
            self.ctx = None

    def snapshot(self) -> dict:
        """Host copies of state, tree and accept outputs (synchronises)."""
        torch.cuda.synchronize()
        out = {n: t.cpu().numpy() for n, t in self.st_t.items()}
        out.update({n: t.cpu().numpy() for n, t in self.tree_t.items()})
        out["target"] = self.target.cpu().numpy()
        out["accept_len"] = self.accept_len.cpu().numpy()
        out["accept_path"] = self.accept_path.cpu().numpy()
        out["bonus"] = self.bonus.cpu().numpy()
        return out
