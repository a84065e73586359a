"""ctypes binding of libddd.so.  Same names as the C ABI; argument marshalling only.

torch is used for device memory and streams.  There is no CPU fallback: if the library has
not been built, or no gfx950 device is present, the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Tuple

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libddd.so")

DDD_OK = 0
DDD_ERR_INVALID_ARG = -1
DDD_ERR_NO_DEVICE = -2
DDD_ERR_WRONG_ARCH = -3
DDD_ERR_HIP = -4
DDD_ERR_UNIMPLEMENTED = -5
DDD_ERR_STATE = -6
DDD_ERR_STATIC_LIMIT = -7

DDD_KMAX = 16
DDD_KWIDE_MAX = 128
DDD_MMAX = 128
DDD_DMAX = 31
DDD_POOL_MAX = 4096
DDD_POOL_WIDE_MAX = 65536
DDD_STATIC_ROWS = 16


class DDDError(RuntimeError):
    def __init__(self, code: int, where: str):
        lib = load_library()
        msg = lib.ddd_strerror(code).decode()
        hip = lib.ddd_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({code})" + (f" [{hip}]" if code == DDD_ERR_HIP and hip else ""))
        self.code = code


class ddd_config(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("V", C.c_int32), ("k", C.c_int32),
                ("max_depth", C.c_int32), ("m", C.c_int32), ("threshold", C.c_float),
                ("check_mask", C.c_uint32), ("flags", C.c_uint32)]


_STATE_FIELDS = ["logprobsum", "beam_node", "beam_token", "beam_parent_slot", "pool_token", "pool_parent",
                 "pool_depth", "pool_score", "n_nodes", "steps", "active", "row_active", "conf"]
_TREE_FIELDS = ["sel_node", "n_sel", "tree_token", "pos", "parent_idx", "mask"]


class ddd_state(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _STATE_FIELDS]


class ddd_tree(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _TREE_FIELDS]


class ddd_round_stats(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("rounds", "depth_hist", "accept_hist", "batch_depth_hist", "steps")]


class ddd_body_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "k", "H", "F", "V", "max_depth", "L")]


class ddd_body_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("E", "Wfc", "g1", "Wqkv", "Wo", "g2", "Wgu", "Wd")]


class ddd_body_prompt(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("K", "V", "f_root", "root_token")]


DRAFT_BODY_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int32, C.POINTER(ddd_state), C.c_void_p, C.c_void_p)
POST_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.POINTER(ddd_state), C.POINTER(ddd_tree), C.c_void_p)

_lib = None


def load_library() -> C.CDLL:
    """dlopen libddd.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    cfgp, stp, trp = C.POINTER(ddd_config), C.POINTER(ddd_state), C.POINTER(ddd_tree)
    sig = {
        "ddd_strerror": (C.c_char_p, [C.c_int]),
        "ddd_last_hip_error": (C.c_char_p, []),
        "ddd_config_validate": (C.c_int, [cfgp]),
        "ddd_pool_capacity": (sz, [cfgp]),
        "ddd_scratch_bytes": (sz, [cfgp]),
        "ddd_create": (C.c_int, [cfgp, C.POINTER(vp)]),
        "ddd_destroy": (C.c_int, [vp]),
        "ddd_num_slices": (C.c_int, [vp]),
        "ddd_round_reset": (C.c_int, [vp, stp, vp, vp]),
        "ddd_lmhead_topk": (C.c_int, [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]),
        "ddd_lmhead_topk_static": (C.c_int, [cfgp, vp, vp, i32, vp, vp, vp, vp, vp]),
        "ddd_static_scratch_bytes": (sz, []),
        "ddd_beam_select": (C.c_int, [vp, i32, vp, vp, stp, vp]),
        "ddd_depth_continue": (C.c_int, [vp, i32, stp, vp]),
        "ddd_draft_step": (C.c_int, [vp, i32, vp, vp, stp, trp, vp, vp, vp]),
        "ddd_tree_finalize": (C.c_int, [vp, stp, trp, vp]),
        "ddd_verify_accept": (C.c_int, [vp, trp, vp, vp, vp, vp, vp]),
        "ddd_verify_sample": (C.c_int, [vp, trp, vp, C.c_float, vp, vp, vp, vp, vp, vp]),
        "ddd_round_enqueue": (C.c_int, [vp, vp, stp, trp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "ddd_round_capture": (C.c_int, [vp, vp, stp, trp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "ddd_round_launch": (C.c_int, [vp, vp]),
        "ddd_stats_bind": (C.c_int, [vp, vp]),
        "ddd_trace_enable": (C.c_int, [vp, i32]),
        "ddd_trace_read": (C.c_int, [vp, vp, sz]),
        "ddd_trace_words": (sz, []),
        "ddd_round_run_stats": (C.c_int, [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                                          C.POINTER(C.c_double)]),
        "ddd_round_run": (C.c_int, [vp, vp, stp, trp, vp, vp, vp, vp, vp, vp, vp]),
        "ddd_weights_pack": (C.c_int, [vp, vp, vp]),
        "ddd_tree_attention_workspace": (sz, [vp, i32, i32]),
        "ddd_kv_pack": (C.c_int, [vp, vp, vp, i32, i32, vp, vp, vp]),
        "ddd_tree_attention": (C.c_int, [vp, trp, vp, vp, vp, vp, vp, i32, i32, vp, sz, vp, vp]),
        "ddd_body_create": (C.c_int, [C.POINTER(ddd_body_config), C.POINTER(vp)]),
        "ddd_body_destroy": (C.c_int, [vp]),
        "ddd_body_bind": (C.c_int, [vp, C.POINTER(ddd_body_weights), C.POINTER(ddd_body_prompt)]),
        "ddd_body_step": (C.c_int, [vp, i32, C.POINTER(ddd_state), vp, vp]),
        "ddd_body_linear": (C.c_int, [vp, vp, i32, i32, vp, i32, vp, i32, vp]),
        "ddd_profile_lmhead": (C.c_int, [vp, vp, vp, i32, i32, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device (or host) pointer of a torch tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _check(code: int, where: str) -> None:
    if code != DDD_OK:
        raise DDDError(code, where)


def current_stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


DDD_FLAG_FORWARD_SWEEPS = 1
DDD_FLAG_POISON_SCRATCH = 2


def make_config(B, H, V, k, max_depth, m, threshold, check_mask=0xFFFFFFFF, flags=0) -> ddd_config:
    return ddd_config(B, H, V, k, max_depth, m, float(threshold), check_mask & 0xFFFFFFFF, flags)


def ddd_config_validate(cfg: ddd_config) -> int:
    return load_library().ddd_config_validate(C.byref(cfg))


def ddd_pool_capacity(cfg: ddd_config) -> int:
    return load_library().ddd_pool_capacity(C.byref(cfg))


def ddd_scratch_bytes(cfg: ddd_config) -> int:
    return load_library().ddd_scratch_bytes(C.byref(cfg))


def ddd_strerror(code: int) -> str:
    return load_library().ddd_strerror(code).decode()


def ddd_create(cfg: ddd_config) -> int:
    out = C.c_void_p()
    _check(load_library().ddd_create(C.byref(cfg), C.byref(out)), "ddd_create")
    return out.value


def ddd_destroy(ctx: int) -> None:
    _check(load_library().ddd_destroy(ctx), "ddd_destroy")


def ddd_num_slices(ctx: int) -> int:
    return load_library().ddd_num_slices(ctx)


def alloc_state(cfg: ddd_config, device="cuda") -> Tuple[ddd_state, Dict[str, "object"]]:
    """Caller-owned device buffers of a ddd_state, as torch tensors, plus the struct of their pointers."""
    import torch
    B, k, nmax = cfg.B, cfg.k, ddd_pool_capacity(cfg)
    i32, f32 = torch.int32, torch.float32
    t = {
        "logprobsum": torch.zeros(B, k, dtype=f32, device=device),
        "beam_node": torch.zeros(B, k, dtype=i32, device=device),
        "beam_token": torch.zeros(B, k, dtype=i32, device=device),
        "beam_parent_slot": torch.zeros(B, k, dtype=i32, device=device),
        "pool_token": torch.full((B, nmax), -1, dtype=i32, device=device),
        "pool_parent": torch.full((B, nmax), -1, dtype=i32, device=device),
        "pool_depth": torch.zeros(B, nmax, dtype=i32, device=device),
        "pool_score": torch.zeros(B, nmax, dtype=f32, device=device),
        "n_nodes": torch.ones(B, dtype=i32, device=device),
        "steps": torch.zeros(B, dtype=i32, device=device),
        "active": torch.ones(B, dtype=torch.uint8, device=device),
        "row_active": torch.ones(B * k, dtype=torch.uint8, device=device),
        "conf": torch.ones(B, dtype=torch.float64, device=device),
    }
    return ddd_state(*[t[n].data_ptr() for n in _STATE_FIELDS]), t


def alloc_tree(cfg: ddd_config, device="cuda") -> Tuple[ddd_tree, Dict[str, "object"]]:
    import torch
    B, m = cfg.B, cfg.m
    i32 = torch.int32
    t = {
        "sel_node": torch.full((B, m), -1, dtype=i32, device=device),
        "n_sel": torch.zeros(B, dtype=i32, device=device),
        "tree_token": torch.full((B, m + 1), -1, dtype=i32, device=device),
        "pos": torch.zeros(B, m + 1, dtype=i32, device=device),
        "parent_idx": torch.full((B, m + 1), -1, dtype=i32, device=device),
        "mask": torch.zeros(B, m + 1, m + 1, dtype=torch.uint8, device=device),
    }
    return ddd_tree(*[t[n].data_ptr() for n in _TREE_FIELDS]), t


def ddd_round_reset(ctx, st: ddd_state, root_token=None, stream=None) -> None:
    _check(load_library().ddd_round_reset(ctx, C.byref(st), _ptr(root_token),
                                          current_stream() if stream is None else stream), "ddd_round_reset")


def ddd_lmhead_topk(ctx, W, hid, n_rows, row_active, topk_token, topk_logprob, lse, logits_dbg=None, stream=None):
    _check(load_library().ddd_lmhead_topk(ctx, _ptr(W), _ptr(hid), n_rows, _ptr(row_active), _ptr(topk_token),
                                          _ptr(topk_logprob), _ptr(lse), _ptr(logits_dbg),
                                          current_stream() if stream is None else stream), "ddd_lmhead_topk")


def ddd_lmhead_topk_static(cfg: ddd_config, W, hid, n_rows, row_active, topk_token, topk_logprob, lse, stream=None):
    """ddd_lmhead_topk without a context and without any allocation (static device scratch)."""
    _check(load_library().ddd_lmhead_topk_static(C.byref(cfg), _ptr(W), _ptr(hid), n_rows, _ptr(row_active),
                                                 _ptr(topk_token), _ptr(topk_logprob), _ptr(lse),
                                                 current_stream() if stream is None else stream),
           "ddd_lmhead_topk_static")


def ddd_static_scratch_bytes() -> int:
    return int(load_library().ddd_static_scratch_bytes())


def ddd_beam_select(ctx, step, topk_token, topk_logprob, st: ddd_state, stream=None):
    _check(load_library().ddd_beam_select(ctx, step, _ptr(topk_token), _ptr(topk_logprob), C.byref(st),
                                          current_stream() if stream is None else stream), "ddd_beam_select")


def ddd_depth_continue(ctx, steps_done, st: ddd_state, stream=None):
    _check(load_library().ddd_depth_continue(ctx, steps_done, C.byref(st),
                                             current_stream() if stream is None else stream), "ddd_depth_continue")


def ddd_draft_step(ctx, step, W, hid, st: ddd_state, tree: Optional[ddd_tree] = None, logits_dbg=None, lse_dbg=None,
                   stream=None):
    _check(load_library().ddd_draft_step(ctx, step, _ptr(W), _ptr(hid), C.byref(st),
                                         C.byref(tree) if tree is not None else None, _ptr(logits_dbg), _ptr(lse_dbg),
                                         current_stream() if stream is None else stream), "ddd_draft_step")


def ddd_tree_finalize(ctx, st: ddd_state, tree: ddd_tree, stream=None):
    _check(load_library().ddd_tree_finalize(ctx, C.byref(st), C.byref(tree),
                                            current_stream() if stream is None else stream), "ddd_tree_finalize")


def ddd_verify_accept(ctx, tree: ddd_tree, target_argmax, accept_len, accept_path, bonus_token, stream=None):
    _check(load_library().ddd_verify_accept(ctx, C.byref(tree), _ptr(target_argmax), _ptr(accept_len),
                                            _ptr(accept_path), _ptr(bonus_token),
                                            current_stream() if stream is None else stream), "ddd_verify_accept")


def ddd_verify_sample(ctx, tree: ddd_tree, target_logits, temperature, u_accept, u_bonus, accept_len, accept_path,
                      bonus_token, stream=None):
    _check(load_library().ddd_verify_sample(ctx, C.byref(tree), _ptr(target_logits), float(temperature), _ptr(u_accept),
                                            _ptr(u_bonus), _ptr(accept_len), _ptr(accept_path), _ptr(bonus_token),
                                            current_stream() if stream is None else stream), "ddd_verify_sample")


def _fn_ptr(fn) -> Optional[int]:
    if fn is None:
        return None
    if isinstance(fn, int):
        return fn
    return C.cast(fn, C.c_void_p).value


def ddd_round_enqueue(ctx, W, st, tree, root_token, hid_buf, body, body_user, post=None, post_user=None,
                      logits_dbg=None, lse_dbg=None, stream=None):
    _check(load_library().ddd_round_enqueue(ctx, _ptr(W), C.byref(st), C.byref(tree), _ptr(root_token), _ptr(hid_buf),
                                            _fn_ptr(body), body_user, _fn_ptr(post), post_user, _ptr(logits_dbg),
                                            _ptr(lse_dbg), current_stream() if stream is None else stream),
           "ddd_round_enqueue")


def ddd_round_capture(ctx, W, st, tree, root_token, hid_buf, body, body_user, post=None, post_user=None,
                      logits_dbg=None, lse_dbg=None, stream=None):
    _check(load_library().ddd_round_capture(ctx, _ptr(W), C.byref(st), C.byref(tree), _ptr(root_token), _ptr(hid_buf),
                                            _fn_ptr(body), body_user, _fn_ptr(post), post_user, _ptr(logits_dbg),
                                            _ptr(lse_dbg), current_stream() if stream is None else stream),
           "ddd_round_capture")


def ddd_round_run(ctx, W, st, tree, root_token, hid_buf, body, body_user, post=None, post_user=None, stream=None) -> int:
    """Host-paced round; returns the number of draft calls queued."""
    rc = load_library().ddd_round_run(ctx, _ptr(W), C.byref(st), C.byref(tree), _ptr(root_token), _ptr(hid_buf),
                                      _fn_ptr(body), body_user, _fn_ptr(post), post_user,
                                      current_stream() if stream is None else stream)
    if rc < 0:
        _check(rc, "ddd_round_run")
    return rc


def ddd_round_run_stats(ctx) -> Dict[str, float]:
    """Counters of ddd_round_run's host waits: rounds, waits, timeouts (waits that ran into their limit), max_wait_us."""
    r, w, t, m = C.c_uint64(), C.c_uint64(), C.c_uint64(), C.c_double()
    _check(load_library().ddd_round_run_stats(ctx, C.byref(r), C.byref(w), C.byref(t), C.byref(m)), "ddd_round_run_stats")
    return {"rounds": r.value, "waits": w.value, "timeouts": t.value, "max_wait_us": m.value}


def ddd_round_launch(ctx, stream=None):
    _check(load_library().ddd_round_launch(ctx, current_stream() if stream is None else stream), "ddd_round_launch")


def ddd_tree_attention_workspace(ctx, n_heads, L) -> int:
    return int(load_library().ddd_tree_attention_workspace(ctx, n_heads, L))


def ddd_kv_pack(ctx, k, v, L, n_heads, k_packed, v_packed, stream=None):
    _check(load_library().ddd_kv_pack(ctx, _ptr(k), _ptr(v), L, n_heads, _ptr(k_packed), _ptr(v_packed),
                                      current_stream() if stream is None else stream), "ddd_kv_pack")


def ddd_tree_attention(ctx, tree: ddd_tree, q, k_tree, vt_tree, k_packed, v_packed, L, n_heads, workspace, out,
                       stream=None):
    nbytes = workspace.numel() * workspace.element_size()
    _check(load_library().ddd_tree_attention(ctx, C.byref(tree), _ptr(q), _ptr(k_tree), _ptr(vt_tree), _ptr(k_packed),
                                             _ptr(v_packed), L, n_heads, _ptr(workspace), nbytes, _ptr(out),
                                             current_stream() if stream is None else stream), "ddd_tree_attention")


def ddd_weights_pack(ctx, W, stream=None):
    """Tile-major copy of W for the GEMM path (W=None forgets it)."""
    _check(load_library().ddd_weights_pack(ctx, _ptr(W), current_stream() if stream is None else stream),
           "ddd_weights_pack")


# ---- stand-in draft layer (include/ddd_body.h) -------------------------------------------------
def ddd_body_create(cfg: ddd_body_config) -> int:
    out = C.c_void_p()
    _check(load_library().ddd_body_create(C.byref(cfg), C.byref(out)), "ddd_body_create")
    return out.value


def ddd_body_destroy(body: int) -> None:
    _check(load_library().ddd_body_destroy(body), "ddd_body_destroy")


def ddd_body_bind(body: int, weights: Dict[str, "object"], prompt: Dict[str, "object"]) -> None:
    """weights / prompt: dicts of device tensors named as the struct fields; the caller keeps them alive."""
    w = ddd_body_weights(*[_ptr(weights[n]) for n, _ in ddd_body_weights._fields_])
    p = ddd_body_prompt(*[_ptr(prompt[n]) for n, _ in ddd_body_prompt._fields_])
    _check(load_library().ddd_body_bind(body, C.byref(w), C.byref(p)), "ddd_body_bind")


def body_step_ptr() -> int:
    """Address of ddd_body_step, usable as the `body` argument of the round calls (user = the body handle)."""
    return C.cast(load_library().ddd_body_step, C.c_void_p).value


def ddd_body_step(body: int, step, st: ddd_state, hid_out, stream=None):
    _check(load_library().ddd_body_step(body, step, C.byref(st), _ptr(hid_out),
                                        current_stream() if stream is None else stream), "ddd_body_step")


def ddd_body_linear(body: int, W, N, K, x, R, y, accumulate=False, stream=None):
    _check(load_library().ddd_body_linear(body, _ptr(W), N, K, _ptr(x), R, _ptr(y), 1 if accumulate else 0,
                                          current_stream() if stream is None else stream), "ddd_body_linear")


def ddd_profile_lmhead(ctx, W, hid, n_rows, iters, stream=None):
    """(mean_ms, min_ms) per launch of the LM-head kernel alone; synchronises."""
    mean, mn = C.c_float(), C.c_float()
    _check(load_library().ddd_profile_lmhead(ctx, _ptr(W), _ptr(hid), n_rows, iters, C.byref(mean), C.byref(mn),
                                                    current_stream() if stream is None else stream),
           "ddd_profile_lmhead")
    return mean.value, mn.value


def ddd_stats_bind(ctx, rounds=None, depth_hist=None, accept_hist=None, batch_depth_hist=None, steps=None) -> None:
    """Binds device statistics arrays (int64; `steps` int32) that the context's verify calls add their rounds to;
    all None unbinds.  The tensors must outlive the binding."""
    if rounds is None and depth_hist is None and accept_hist is None and batch_depth_hist is None:
        _check(load_library().ddd_stats_bind(ctx, None), "ddd_stats_bind")
        return
    s = ddd_round_stats(_ptr(rounds), _ptr(depth_hist), _ptr(accept_hist), _ptr(batch_depth_hist), _ptr(steps))
    _check(load_library().ddd_stats_bind(ctx, C.byref(s)), "ddd_stats_bind")


def ddd_trace_enable(ctx, on: bool = True) -> None:
    _check(load_library().ddd_trace_enable(ctx, 1 if on else 0), "ddd_trace_enable")


def ddd_trace_read(ctx):
    """The context's device-timestamp trace as a numpy uint64 array [DDD_DMAX + 1, DDD_TRACE_CALL_WORDS]
    (100 MHz ticks, 0 = not written); synchronises and clears the device buffer."""
    import numpy as np
    n = int(load_library().ddd_trace_words())
    out = np.zeros(n, dtype=np.uint64)
    _check(load_library().ddd_trace_read(ctx, out.ctypes.data, n), "ddd_trace_read")
    return out.reshape(DDD_DMAX + 1, -1)
