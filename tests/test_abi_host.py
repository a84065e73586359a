"""Host-only checks of the C ABI: the library loads, exports every declared symbol, validates
configurations and reports errors as status codes.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def D():
    import paper_2409_00142_amd as D
    if not os.path.exists(D.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    D.load_library()
    return D


def _declared_symbols(headers):
    names = []
    for hdr in headers:
        text = open(os.path.join(ROOT, "include", hdr)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"^\s*(?:const\s+char\s*\*|int|size_t)\s+(ddd_\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def _exported_symbols(path):
    """Dynamic symbols a shared object defines (nm -D --defined-only)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], check=True, capture_output=True, text=True).stdout
    return {line.split()[-1] for line in out.splitlines() if line.strip()}


def test_every_declared_symbol_is_exported(D):
    lib = D.load_library()
    names = _declared_symbols(("ddd.h", "ddd_body.h"))
    assert len(names) >= 24
    for n in ("ddd_lmhead_topk", "ddd_beam_select", "ddd_depth_continue", "ddd_tree_finalize", "ddd_verify_accept",
              "ddd_verify_sample", "ddd_tree_attention", "ddd_body_step"):
        assert n in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/ but not exported"


def test_harness_lives_in_its_own_shared_object(D):
    """The workload generators and measurement kernels of the tests and the benchmark (include/ddd_synth.h) are
    exported by synth/libddd_synth.so; the product library exports none of them."""
    from synth import native
    slib = native.load_library()
    names = _declared_symbols(("ddd_synth.h",))
    assert len(names) >= 8 and all(n.startswith("ddd_synth_") for n in names)
    for n in names:
        assert hasattr(slib, n), f"{n} declared in include/ddd_synth.h but not exported by libddd_synth.so"
    product = _exported_symbols(D.LIB_PATH)
    assert "ddd_lmhead_topk" in product
    assert not [n for n in product if "synth" in n]
    harness = _exported_symbols(native.LIB_PATH)
    assert not [n for n in harness if n.startswith("ddd_") and not n.startswith("ddd_synth_")]


def test_struct_layouts_match_the_header(D):
    assert C.sizeof(D.ddd_config) == 36
    assert C.sizeof(D.ddd_state) == 13 * 8
    assert C.sizeof(D.ddd_tree) == 6 * 8
    from synth import native
    assert native.ddd_synth_params.seed.offset == 40 and native.ddd_synth_params.scale_depth.offset == 64
    assert C.sizeof(native.ddd_synth_params) == 208


def test_config_validation(D):
    ok = D.make_config(1, 4096, 32000, 10, 10, 60, 0.3)
    assert D.ddd_config_validate(ok) == D.DDD_OK
    assert D.ddd_pool_capacity(ok) == 1 + 10 + 9 * 100
    for name in ("tiny", "7b_b1", "13b_b1", "7b_b64", "large_vocab"):
        import synth
        wl = synth.WORKLOADS[name]
        cfg = D.make_config(wl.B, wl.H, wl.V, wl.k, wl.D, wl.m, wl.threshold)
        assert D.ddd_config_validate(cfg) == D.DDD_OK, name
        assert D.ddd_pool_capacity(cfg) == wl.pool_capacity
    bad = [
        dict(B=0), dict(k=0), dict(k=129), dict(V=5), dict(V=1 << 24), dict(max_depth=0), dict(max_depth=32),
        dict(k=17, V=(1 << 17) + 1), dict(B=2, V=(1 << 17) + 1), dict(k=100, max_depth=8), dict(k=128, max_depth=6),
        # ^ the GEMM path (wide beams, or more than 16 rows): V <= 2^17; wide pools <= 65536
        dict(m=0), dict(m=129), dict(H=100), dict(H=4096 + 64), dict(H=128 * 64), dict(H=5632), dict(threshold=-0.1),
        dict(threshold=float("nan")), dict(k=16, max_depth=20),
    ]
    base = dict(B=1, H=4096, V=32000, k=10, max_depth=10, m=60, threshold=0.3)
    for b in bad:
        kw = dict(base, **b)
        cfg = D.make_config(**kw)
        assert D.ddd_config_validate(cfg) == D.DDD_ERR_INVALID_ARG, b
        assert D.ddd_pool_capacity(cfg) == 0
    for good in (dict(k=17), dict(k=100, max_depth=6), dict(k=128, max_depth=4), dict(k=64, V=1 << 17), dict(V=(1 << 24) - 1)):
        cfg = D.make_config(**dict(base, **good))
        assert D.ddd_config_validate(cfg) == D.DDD_OK, good
        assert D.ddd_pool_capacity(cfg) == 1 + cfg.k + (cfg.max_depth - 1) * cfg.k * cfg.k
    # hidden rows of the MFMA path are addressed by 32-bit byte offsets: B*k*H*2 must stay below 2^32
    big = dict(base, B=4096, k=128, H=5120, V=1000, max_depth=4)
    assert D.ddd_config_validate(D.make_config(**big)) == D.DDD_ERR_INVALID_ARG
    assert D.ddd_config_validate(D.make_config(**dict(big, H=4096))) == D.DDD_ERR_INVALID_ARG      # exactly 2^32 bytes
    assert D.ddd_config_validate(D.make_config(**dict(big, H=4096, B=4095))) == D.DDD_OK
    flagged = D.make_config(**base)
    flagged.flags = D.DDD_FLAG_FORWARD_SWEEPS
    assert D.ddd_config_validate(flagged) == D.DDD_OK
    flagged.flags = D.DDD_FLAG_FORWARD_SWEEPS | D.DDD_FLAG_POISON_SCRATCH
    assert D.ddd_config_validate(flagged) == D.DDD_OK
    flagged.flags = 4
    assert D.ddd_config_validate(flagged) == D.DDD_ERR_INVALID_ARG
    assert D.load_library().ddd_config_validate(None) == D.DDD_ERR_INVALID_ARG


def test_error_strings_and_null_arguments(D):
    lib = D.load_library()
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        assert D.ddd_strerror(code) not in ("", "unknown status")
    assert D.ddd_strerror(-99) == "unknown status"
    assert lib.ddd_create(None, None) == D.DDD_ERR_INVALID_ARG
    assert lib.ddd_destroy(None) == D.DDD_ERR_INVALID_ARG
    assert lib.ddd_round_launch(None, None) == D.DDD_ERR_INVALID_ARG
    assert lib.ddd_lmhead_topk(None, None, None, 1, None, None, None, None, None, None) == D.DDD_ERR_INVALID_ARG
    from synth import native
    assert native.load_library().ddd_synth_next_round(None, None) == D.DDD_ERR_INVALID_ARG
    assert lib.ddd_round_run_stats(None, None, None, None, None) == D.DDD_ERR_INVALID_ARG
    assert lib.ddd_stats_bind(None, None) == D.DDD_ERR_INVALID_ARG
    # the allocation-free entry point validates before it touches a device
    assert lib.ddd_static_scratch_bytes() == 16 * 16 * 256 * 8 + 16 * 256 * 4
    cfg = D.make_config(1, 256, 1000, 4, 6, 16, 0.35)
    one = C.c_void_p(8)       # any non-null address: rejected calls never look at it
    assert lib.ddd_lmhead_topk_static(None, one, one, 1, None, one, one, one, None) == D.DDD_ERR_INVALID_ARG
    assert lib.ddd_lmhead_topk_static(C.byref(cfg), None, one, 1, None, one, one, one, None) == D.DDD_ERR_INVALID_ARG
    assert lib.ddd_lmhead_topk_static(C.byref(cfg), one, one, 0, None, one, one, one, None) == D.DDD_ERR_INVALID_ARG
    assert lib.ddd_lmhead_topk_static(C.byref(cfg), one, one, 17, None, one, one, one, None) == D.DDD_ERR_STATIC_LIMIT
    wide = D.make_config(1, 256, 1000, 17, 3, 16, 0.35)
    assert lib.ddd_lmhead_topk_static(C.byref(wide), one, one, 1, None, one, one, one, None) == D.DDD_ERR_STATIC_LIMIT


def test_create_without_a_device_fails_with_a_status():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a device is present")
    import paper_2409_00142_amd as D
    with pytest.raises(D.DDDError) as e:
        D.ddd_create(D.make_config(1, 256, 1000, 4, 6, 16, 0.35))
    assert e.value.code == D.DDD_ERR_NO_DEVICE


def test_sanitized_host_build_of_the_abi_checks(tmp_path):
    """The library's host code (argument validation, size arithmetic, dispatch) compiled with AddressSanitizer and
    UndefinedBehaviorSanitizer and driven through every entry point's rejection paths by tests/sanitize/abi_check.cpp:
    extreme field values, null pointers, sizes beyond the limits.  Device code is compiled as usual and nothing is
    launched, so this runs without a GPU."""
    import subprocess
    from paper_2409_00142_amd.build import build_sanitized_check
    exe = build_sanitized_check(str(tmp_path / "san"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0 and "ABI_SANITIZE_OK" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]


def test_product_package_does_not_import_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2409_00142_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f"{f} mentions the oracle"
