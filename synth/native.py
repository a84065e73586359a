"""ctypes binding of synth/libddd_synth.so: the device-side workload generators and measurement kernels
declared in include/ddd_synth.h.  Test and benchmark harness, not product: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import paper_2409_00142_amd as D
from paper_2409_00142_amd.binding import _check, _ptr, current_stream, ddd_config, ddd_state, ddd_tree

SYNTH_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(SYNTH_DIR, "libddd_synth.so")


class ddd_synth_params(C.Structure):
    _fields_ = [("cfg", ddd_config), ("seed", C.c_uint64), ("round_ctr", C.c_void_p),
                ("root_token", C.c_int32), ("n_plant", C.c_int32), ("scale_depth", C.c_float * 32),
                ("plant_dir", C.c_void_p), ("plant_round_p24", C.c_uint32), ("plant_row_p24", C.c_uint32)]


class ddd_synth_post_args(C.Structure):
    _fields_ = [("params", C.c_void_p), ("ctx", C.c_void_p)] + [(n, C.c_void_p) for n in (
        "target_argmax", "accept_len", "accept_path", "bonus_token", "depth_hist", "accept_hist", "batch_depth_hist",
        "hash_tokens")]


_lib = None


def load_library() -> C.CDLL:
    """dlopen libddd_synth.so (after the product library it is linked against); raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    D.load_library()
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    stp, trp = C.POINTER(ddd_state), C.POINTER(ddd_tree)
    sig = {
        "ddd_synth_draft_body": (C.c_int, [vp, i32, stp, vp, vp]),
        "ddd_synth_target_argmax": (C.c_int, [C.POINTER(ddd_synth_params), stp, trp, vp, vp]),
        "ddd_synth_next_round": (C.c_int, [vp, vp]),
        "ddd_synth_post": (C.c_int, [vp, stp, trp, vp]),
        "ddd_synth_read_stream": (C.c_int, [vp, sz, vp, i32, vp]),
        "ddd_synth_mfma_rate": (C.c_int, [vp, i32, i32, vp]),
        "ddd_synth_round_stats": (C.c_int, [vp, vp, vp, i32, vp, vp, vp, vp]),
        "ddd_synth_hash_tokens": (C.c_int, [vp, vp, i32, i32, C.c_uint64, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _stream(stream):
    return current_stream() if stream is None else stream


def synth_post_ptr() -> int:
    """Address of ddd_synth_post, usable as the `post` argument of the round calls (user = ddd_synth_post_args)."""
    return C.cast(load_library().ddd_synth_post, C.c_void_p).value


def synth_draft_body_ptr() -> int:
    """Address of ddd_synth_draft_body, usable as the `body` argument of the round calls."""
    return C.cast(load_library().ddd_synth_draft_body, C.c_void_p).value


def ddd_synth_draft_body(params: ddd_synth_params, step, st: ddd_state, hid_out, stream=None):
    _check(load_library().ddd_synth_draft_body(C.addressof(params), step, C.byref(st), _ptr(hid_out), _stream(stream)),
           "ddd_synth_draft_body")


def ddd_synth_target_argmax(params: ddd_synth_params, st: ddd_state, tree: ddd_tree, target_argmax, stream=None):
    _check(load_library().ddd_synth_target_argmax(C.byref(params), C.byref(st), C.byref(tree), _ptr(target_argmax),
                                                  _stream(stream)), "ddd_synth_target_argmax")


def ddd_synth_next_round(round_ctr, stream=None):
    _check(load_library().ddd_synth_next_round(_ptr(round_ctr), _stream(stream)), "ddd_synth_next_round")


def ddd_synth_round_stats(round_ctr, steps, accept_len, B, depth_hist, accept_hist, batch_depth_hist=None, stream=None):
    _check(load_library().ddd_synth_round_stats(_ptr(round_ctr), _ptr(steps), _ptr(accept_len), B, _ptr(depth_hist),
                                                _ptr(accept_hist), _ptr(batch_depth_hist), _stream(stream)),
           "ddd_synth_round_stats")


def ddd_synth_hash_tokens(round_ctr, tokens, n, V, seed, stream=None):
    _check(load_library().ddd_synth_hash_tokens(_ptr(round_ctr), _ptr(tokens), n, V, seed, _stream(stream)),
           "ddd_synth_hash_tokens")


def ddd_synth_mfma_rate(sink, iters, n_blocks, stream=None):
    _check(load_library().ddd_synth_mfma_rate(_ptr(sink), iters, n_blocks, _stream(stream)), "ddd_synth_mfma_rate")


def ddd_synth_read_stream(src, n_bytes, sink, n_blocks, stream=None):
    _check(load_library().ddd_synth_read_stream(_ptr(src), n_bytes, _ptr(sink), n_blocks, _stream(stream)),
           "ddd_synth_read_stream")
